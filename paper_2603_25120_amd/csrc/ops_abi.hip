// C ABI for the single operations (mllm_op_*): argument checks, then the same launchers the
// stage uses.  The attention entry points build their tile lists on the host in pinned staging
// memory (a per-thread ring of slots) and copy them into the caller's workspace on the caller's
// stream, in front of the kernel that reads them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/mllm_stage.h"
#include "kernels.h"
#include "attn_items.h"
#include "pinned_ring.h"

using namespace mllm;

namespace {

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

}  // namespace

// One thread-local error slot for the whole library; it lives beside mllm_last_error().
namespace mllm_detail { void set_last_error(const char* msg); }

namespace {
mllm_status_t op_fail(mllm_status_t st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  mllm_detail::set_last_error(buf);
  return st;
}

mllm_status_t check_pack(const mllm_pack_t* p) {
  if (!p || !p->cu_seqlens_host || (p->n_segments > 0 && !p->mask_kind_host)) return op_fail(MLLM_ERR_NULL, "pack or its arrays are NULL");
  if (p->n_segments < 0 || p->total_tokens < 0) return op_fail(MLLM_ERR_SHAPE, "negative sizes");
  if (p->cu_seqlens_host[0] != 0) return op_fail(MLLM_ERR_CU_SEQLENS, "cu_seqlens[0] != 0");
  int longest = 0;
  for (int s = 0; s < p->n_segments; s++) {
    int len = p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
    if (len < 0) return op_fail(MLLM_ERR_CU_SEQLENS, "cu_seqlens decreases at segment %d", s);
    longest = std::max(longest, len);
    if (p->mask_kind_host[s] > 1) return op_fail(MLLM_ERR_MASK_KIND, "mask kind %d at segment %d", (int)p->mask_kind_host[s], s);
  }
  if (p->cu_seqlens_host[p->n_segments] != p->total_tokens) return op_fail(MLLM_ERR_CU_SEQLENS, "cu_seqlens does not end at total_tokens");
  if (p->max_seqlen < longest) return op_fail(MLLM_ERR_SHAPE, "max_seqlen below the longest segment");
  return MLLM_OK;
}

mllm_status_t check_attn(const mllm_pack_t* pack, int32_t hq, int32_t hkv, int32_t hd, int64_t qs,
                         int64_t kvs, int64_t os, const void* ws, size_t ws_bytes) {
  mllm_status_t r = check_pack(pack);
  if (r != MLLM_OK) return r;
  if (hd != 64 && hd != 128) return op_fail(MLLM_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (hq <= 0 || hkv <= 0 || hq % hkv) return op_fail(MLLM_ERR_SHAPE, "n_q_heads must be a positive multiple of n_kv_heads");
  if (qs < (int64_t)hq * hd || kvs < (int64_t)hkv * hd || os < (int64_t)hq * hd || qs % 8 || kvs % 8 || os % 8)
    return op_fail(MLLM_ERR_SHAPE, "row strides too small or not multiples of 8");
  if (!ws) return op_fail(MLLM_ERR_NULL, "workspace is NULL");
  if (ws_bytes < mllm_op_attn_workspace_bytes(pack->n_segments, pack->total_tokens, hq)) return op_fail(MLLM_ERR_WORKSPACE, "attention workspace too small");
  return MLLM_OK;
}

#define OP_TRY(expr)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return op_fail(MLLM_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// One ring per host thread (the library keeps no other state between op calls); never freed.
PinnedRing& op_staging() {
  thread_local PinnedRing* ring = new PinnedRing();
  return *ring;
}

mllm_status_t upload_tiles(const mllm_pack_t* pack, void* ws, AttnArgs& a, hipStream_t stream) {
  char* w = (char*)ws;
  const size_t qbytes = attn_list_bytes(*pack, ATTN_FWD_Q_TILE, a.n_q_heads);
  const size_t koff = align_up(qbytes);
  const size_t bytes = koff + attn_list_bytes(*pack, ATTN_BWD_KV_TILE, a.n_kv_heads);
  PinnedRing& ring = op_staging();
  PinnedRing::Slot* slot = nullptr;
  OP_TRY(ring.acquire(bytes, &slot));
  char* h = (char*)slot->p;
  a.q_grid = build_attn_list(*pack, ATTN_FWD_Q_TILE, false, a.n_kv_heads, a.n_q_heads / a.n_kv_heads, 64, h);
  a.kv_grid = build_attn_list(*pack, ATTN_BWD_KV_TILE, true, a.n_kv_heads, a.n_q_heads / a.n_kv_heads,
                              a.head_dim == 64 ? 64 : 32, h + koff);
  if (a.q_grid) OP_TRY(hipMemcpyAsync(w, h, (size_t)a.q_grid * sizeof(AttnItem), hipMemcpyHostToDevice, stream));
  if (a.kv_grid) OP_TRY(hipMemcpyAsync(w + koff, h + koff, (size_t)a.kv_grid * sizeof(AttnItem), hipMemcpyHostToDevice, stream));
  OP_TRY(ring.commit(slot, stream));
  a.q_list = w;
  a.kv_list = w + koff;
  double pairs = 0;
  for (int s = 0; s < pack->n_segments; s++) {
    const double len = pack->cu_seqlens_host[s + 1] - pack->cu_seqlens_host[s];
    pairs += pack->mask_kind_host[s] == MLLM_MASK_CAUSAL ? 0.5 * len * len : len * len;
  }
  a.fwd_flops = 4.0 * pairs * a.n_q_heads * a.head_dim;
  return MLLM_OK;
}

}  // namespace

// Scratch of mllm_op_colsum_static, the entry point for callers that cannot allocate: the fp32
// partial column sums that mllm_op_colsum takes as its `partial` argument live in this array
// instead.  Every GPU the library runs on holds its own copy until the process ends.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];       // device address of `scratch` on each device, resolved on first use
std::mutex g_scratch_mutex;

// The array's name is only a host-side handle: its device address on the current device comes
// from hipGetSymbolAddress, once per device.
mllm_status_t static_scratch(void** out) {
  int dev = -1;
  OP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return op_fail(MLLM_ERR_UNSUPPORTED, "device index %d beyond %d", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    OP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return op_fail(MLLM_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MLLM_OK;
}
}  // namespace

extern "C" {

mllm_status_t mllm_op_gemm(const void* a, const void* b, void* c, int64_t m, int64_t n, int64_t k,
                           int a_layout, int b_layout, int out_fp32, int accumulate,
                           const void* bias, const void* residual, void* hip_stream) {
  if (!a || !b || !c) return op_fail(MLLM_ERR_NULL, "a, b or c is NULL");
  if (m < 0 || n < 0 || k < 0) return op_fail(MLLM_ERR_SHAPE, "negative size");
  if ((a_layout | b_layout) & ~1) return op_fail(MLLM_ERR_SHAPE, "layouts must be 0 or 1");
  const int64_t lda = a_layout ? m : k, ldb = b_layout ? k : n;
  if (lda % 8 || ldb % 8 || n % 8) return op_fail(MLLM_ERR_SHAPE, "contiguous dimensions must be multiples of 8");
  if (out_fp32 && residual) return op_fail(MLLM_ERR_UNSUPPORTED, "residual needs a bf16 output");
  if (!out_fp32 && accumulate) return op_fail(MLLM_ERR_UNSUPPORTED, "accumulate needs an fp32 output");
  GemmArgs g;
  g.a = a; g.b = b; g.c = c; g.m = m; g.n = n; g.k = k; g.lda = lda; g.ldb = ldb; g.ldc = n;
  g.a_layout = a_layout; g.b_layout = b_layout; g.out_fp32 = out_fp32; g.accumulate = accumulate;
  g.bias = bias; g.residual = residual; g.ldres = n;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  OP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_gemm_swiglu(const void* x, const void* w_gu, void* pre, void* act, int64_t m,
                                  int64_t f, int64_t k, void* hip_stream) {
  if (!x || !w_gu || !pre || !act) return op_fail(MLLM_ERR_NULL, "a tensor pointer is NULL");
  if (m < 0 || f <= 0 || k <= 0) return op_fail(MLLM_ERR_SHAPE, "sizes must be positive");
  if (!gemm_swiglu_fusable(m, 2 * f, k))
    return op_fail(MLLM_ERR_UNSUPPORTED, "the fused form needs f a multiple of 128, k a multiple of 64 and at least 200 output tiles of 256 x 256");
  GemmArgs g;
  g.a = x; g.b = w_gu; g.c = pre; g.m = m; g.n = 2 * f; g.k = k; g.lda = k; g.ldb = 2 * f; g.ldc = 2 * f;
  g.a_layout = 0; g.b_layout = 0; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = nullptr; g.residual = nullptr; g.ldres = 0;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.swiglu_act = act;
  OP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_gemm_swiglu_bwd(const void* dy, const void* w_d, const void* pre, void* dpre,
                                      int64_t m, int64_t f, int64_t k, void* hip_stream) {
  if (!dy || !w_d || !pre || !dpre) return op_fail(MLLM_ERR_NULL, "a tensor pointer is NULL");
  if (m < 0 || f <= 0 || k <= 0) return op_fail(MLLM_ERR_SHAPE, "sizes must be positive");
  if (!gemm_swiglu_bwd_fusable(m, f, k))
    return op_fail(MLLM_ERR_UNSUPPORTED, "the fused form needs f a multiple of 8, k a multiple of 64 and at least 200 tiles of 256 x 256 of [m, f]");
  GemmArgs g;
  g.a = dy; g.b = w_d; g.c = nullptr; g.m = m; g.n = f; g.k = k; g.lda = k; g.ldb = k; g.ldc = 2 * f;
  g.a_layout = 0; g.b_layout = 1; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = nullptr; g.residual = nullptr; g.ldres = 0;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.swiglu_pre = pre; g.swiglu_dpre = dpre;
  OP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_rope_table(float* table, int64_t n_pos, int32_t head_dim, float rope_base, void* hip_stream) {
  if (!table) return op_fail(MLLM_ERR_NULL, "table is NULL");
  if (n_pos < 0 || head_dim <= 0 || head_dim % 16 || !(rope_base > 1.f)) return op_fail(MLLM_ERR_SHAPE, "bad rope table geometry");
  OP_TRY(launch_rope_table(table, n_pos, head_dim, rope_base, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_gemm_rope(const void* x, const void* w, const void* bias, void* y, int64_t m, int64_t n,
                                int64_t k, const int32_t* pos, const float* rope_table, int64_t rope_cols,
                                int32_t head_dim, void* hip_stream) {
  if (!x || !w || !y || !pos || !rope_table) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (m < 0 || n <= 0 || k <= 0 || n % 8 || k % 8) return op_fail(MLLM_ERR_SHAPE, "sizes must be positive, n and k multiples of 8");
  if (rope_cols < 0 || rope_cols > n || rope_cols % 128 || (head_dim != 64 && head_dim != 128))
    return op_fail(MLLM_ERR_SHAPE, "rope_cols must be a multiple of 128 within n, head_dim 64 or 128");
  if (!gemm_rope_fusable(m, n, k, head_dim))
    return op_fail(MLLM_ERR_UNSUPPORTED, "the fused form needs k a multiple of 64 and at least 200 output tiles of 256 x 256");
  GemmArgs g;
  g.a = x; g.b = w; g.c = y; g.m = m; g.n = n; g.k = k; g.lda = k; g.ldb = n; g.ldc = n;
  g.a_layout = 0; g.b_layout = 0; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = bias; g.residual = nullptr; g.ldres = 0;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.rope_table = rope_table; g.rope_pos = pos; g.rope_cols = rope_cols; g.rope_head_dim = head_dim;
  OP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_attn_work_list(const mllm_pack_t* pack, int32_t kv_major, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim, void* out_host, size_t out_bytes, size_t* bytes_needed,
                                  int32_t* grid_out) {
  mllm_status_t r = check_pack(pack);
  if (r != MLLM_OK) return r;
  if (head_dim != 64 && head_dim != 128) return op_fail(MLLM_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads) return op_fail(MLLM_ERR_SHAPE, "n_q_heads must be a positive multiple of n_kv_heads");
  const int tile = kv_major ? ATTN_BWD_KV_TILE : ATTN_FWD_Q_TILE;
  const size_t need = attn_list_bytes(*pack, tile, kv_major ? n_kv_heads : n_q_heads);
  if (bytes_needed) *bytes_needed = need;
  if (!out_host) return MLLM_OK;
  if (out_bytes < need) return op_fail(MLLM_ERR_WORKSPACE, "work list needs %zu bytes, %zu given", need, out_bytes);
  const int grid = build_attn_list(*pack, tile, kv_major != 0, n_kv_heads, n_q_heads / n_kv_heads,
                                   kv_major ? (head_dim == 64 ? 64 : 32) : 64, (char*)out_host);
  if (grid_out) *grid_out = grid;
  return MLLM_OK;
}

size_t mllm_op_attn_workspace_bytes(int32_t n_segments, int32_t total_tokens, int32_t n_q_heads) {
  const size_t max_tiles = (size_t)std::max(0, total_tokens) / 128 + (size_t)std::max(0, n_segments) + 1;
  return 2 * align_up((size_t)ATTN_XCDS * sizeof(AttnItem) * max_tiles * (size_t)std::max(1, n_q_heads));
}

mllm_status_t mllm_op_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                               const mllm_pack_t* pack, int32_t n_q_heads, int32_t n_kv_heads,
                               int32_t head_dim, int64_t q_stride, int64_t kv_stride,
                               int64_t o_stride, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  if (!q || !k || !v || !o || !lse) return op_fail(MLLM_ERR_NULL, "a tensor pointer is NULL");
  mllm_status_t r = check_attn(pack, n_q_heads, n_kv_heads, head_dim, q_stride, kv_stride, o_stride, workspace, workspace_bytes);
  if (r != MLLM_OK) return r;
  AttnArgs a = {};
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
  a.q_stride = q_stride; a.kv_stride = kv_stride; a.o_stride = o_stride;
  a.total_tokens = pack->total_tokens; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
  if ((r = upload_tiles(pack, workspace, a, (hipStream_t)hip_stream)) != MLLM_OK) return r;
  OP_TRY(launch_attn_fwd(a, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_attn_bwd(const void* q, const void* k, const void* v, const void* o,
                               const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                               float* delta, const mllm_pack_t* pack, int32_t n_q_heads,
                               int32_t n_kv_heads, int32_t head_dim, int64_t q_stride,
                               int64_t kv_stride, int64_t o_stride, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  return mllm_op_attn_bwd_rope(q, k, v, o, lse, d_o, dq, dk, dv, delta, pack, n_q_heads, n_kv_heads, head_dim, q_stride,
                               kv_stride, o_stride, nullptr, workspace, workspace_bytes, hip_stream);
}

mllm_status_t mllm_op_attn_bwd_rope(const void* q, const void* k, const void* v, const void* o,
                                    const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                                    float* delta, const mllm_pack_t* pack, int32_t n_q_heads,
                                    int32_t n_kv_heads, int32_t head_dim, int64_t q_stride,
                                    int64_t kv_stride, int64_t o_stride, const float* rope_table,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !delta) return op_fail(MLLM_ERR_NULL, "a tensor pointer is NULL");
  mllm_status_t r = check_attn(pack, n_q_heads, n_kv_heads, head_dim, q_stride, kv_stride, o_stride, workspace, workspace_bytes);
  if (r != MLLM_OK) return r;
  AttnArgs a = {};
  a.q = q; a.k = k; a.v = v; a.o = const_cast<void*>(o); a.lse = const_cast<float*>(lse);
  a.d_o = d_o; a.dq = dq; a.dk = dk; a.dv = dv; a.delta = delta;
  a.rope_table = rope_table;
  a.q_stride = q_stride; a.kv_stride = kv_stride; a.o_stride = o_stride;
  a.total_tokens = pack->total_tokens; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
  if ((r = upload_tiles(pack, workspace, a, (hipStream_t)hip_stream)) != MLLM_OK) return r;
  OP_TRY(launch_attn_bwd(a, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_norm_fwd(int kind, const void* x, const void* gamma, const void* beta,
                               void* y, float* stats, int64_t t, int64_t d, float eps,
                               void* hip_stream) {
  if (!x || !gamma || !y || !stats || (kind == 0 && !beta)) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (kind != 0 && kind != 1) return op_fail(MLLM_ERR_SHAPE, "kind must be 0 or 1");
  if (t < 0 || d <= 0 || d % 8 || d > 8192) return op_fail(MLLM_ERR_SHAPE, "d must be a multiple of 8, at most 8192");
  OP_TRY(launch_norm_fwd(kind, x, gamma, beta, y, stats, t, d, d, eps, (hipStream_t)hip_stream));
  return MLLM_OK;
}

size_t mllm_op_norm_bwd_partial_bytes(int64_t t, int64_t d) {
  return (size_t)norm_bwd_partial_rows(t) * (size_t)d * 4 * 3;
}

mllm_status_t mllm_op_norm_bwd(int kind, const void* dy, const void* x, const void* gamma,
                               const float* stats, const void* dres, void* dx, float* dgamma,
                               float* dbeta, int accumulate, float* partial, int64_t t, int64_t d,
                               void* hip_stream) {
  if (!dy || !x || !gamma || !stats || !dx || !dgamma || !partial || (kind == 0 && !dbeta)) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (kind != 0 && kind != 1) return op_fail(MLLM_ERR_SHAPE, "kind must be 0 or 1");
  if (t < 0 || d <= 0 || d % 8 || d > 8192) return op_fail(MLLM_ERR_SHAPE, "d must be a multiple of 8, at most 8192");
  OP_TRY(launch_norm_bwd(kind, dy, x, gamma, stats, dres, dx, dgamma, dbeta, accumulate, partial, t, d, d, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_norm_bwd_colsum(int kind, const void* dy, const void* x, const void* gamma,
                                      const float* stats, const void* dres, void* dx, float* dgamma,
                                      float* dbeta, float* dx_colsum, int accumulate, float* partial,
                                      int64_t t, int64_t d, void* hip_stream) {
  if (!dy || !x || !gamma || !stats || !dx || !dgamma || !dx_colsum || !partial || (kind == 0 && !dbeta))
    return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (kind != 0 && kind != 1) return op_fail(MLLM_ERR_SHAPE, "kind must be 0 or 1");
  if (t < 0 || d <= 0 || d % 8 || !norm_bwd_colsum_fusable(d))
    return op_fail(MLLM_ERR_SHAPE, "d must be a multiple of 8, at most 1024");
  OP_TRY(launch_norm_bwd(kind, dy, x, gamma, stats, dres, dx, dgamma, dbeta, accumulate, partial, t, d, d,
                         (hipStream_t)hip_stream, dx_colsum));
  return MLLM_OK;
}

mllm_status_t mllm_op_rope(void* qk, const int32_t* pos, int64_t t, int64_t row_stride,
                           int64_t col0, int32_t n_heads, int32_t head_dim, float rope_base,
                           int inverse, void* hip_stream) {
  if (!qk || !pos) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (t < 0 || n_heads < 0 || head_dim <= 0 || head_dim % 16 || row_stride % 8 || col0 % 8 ||
      col0 + (int64_t)n_heads * head_dim > row_stride)
    return op_fail(MLLM_ERR_SHAPE, "bad rope geometry");
  OP_TRY(launch_rope(qk, pos, t, row_stride, col0, n_heads, head_dim, rope_base, inverse, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_act_fwd(int act, const void* pre, void* a, int64_t t, int64_t f, void* hip_stream) {
  if (!pre || !a) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (act < 0 || act > 2 || t < 0 || f <= 0 || f % 8) return op_fail(MLLM_ERR_SHAPE, "bad activation arguments");
  OP_TRY(launch_act_fwd(act, pre, a, t, f, (hipStream_t)hip_stream));
  return MLLM_OK;
}

mllm_status_t mllm_op_act_bwd(int act, const void* da, const void* pre, void* dpre, int64_t t, int64_t f, void* hip_stream) {
  if (!da || !pre || !dpre) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (act < 0 || act > 2 || t < 0 || f <= 0 || f % 8) return op_fail(MLLM_ERR_SHAPE, "bad activation arguments");
  OP_TRY(launch_act_bwd(act, da, pre, dpre, t, f, (hipStream_t)hip_stream));
  return MLLM_OK;
}

size_t mllm_op_colsum_partial_bytes(int64_t t, int64_t n) { return (size_t)colsum_partial_rows(t) * (size_t)n * 4; }

mllm_status_t mllm_op_colsum(const void* x, float* out, int accumulate, float* partial, int64_t t, int64_t n, void* hip_stream) {
  if (!x || !out || !partial) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (t < 0 || n <= 0 || n % 8) return op_fail(MLLM_ERR_SHAPE, "n must be a positive multiple of 8");
  OP_TRY(launch_colsum(x, n, out, accumulate, partial, t, n, (hipStream_t)hip_stream));
  return MLLM_OK;
}

size_t mllm_op_colsum_static_max_bytes(void) { return STATIC_SCRATCH_BYTES; }

mllm_status_t mllm_op_colsum_static(const void* x, float* out, int accumulate, int64_t t, int64_t n, void* hip_stream) {
  if (!x || !out) return op_fail(MLLM_ERR_NULL, "a pointer is NULL");
  if (t < 0 || n <= 0 || n % 8) return op_fail(MLLM_ERR_SHAPE, "n must be a positive multiple of 8");
  const size_t need = mllm_op_colsum_partial_bytes(t, n);
  if (need > STATIC_SCRATCH_BYTES)
    return op_fail(MLLM_ERR_WORKSPACE, "a [%lld, %lld] column sum needs %zu bytes of partial sums, the static scratch holds %zu",
                   (long long)t, (long long)n, need, STATIC_SCRATCH_BYTES);
  void* partial = nullptr;
  mllm_status_t r = static_scratch(&partial);
  if (r != MLLM_OK) return r;
  // every partial sum the second kernel reads is written by the first: nothing to clear
  OP_TRY(launch_colsum(x, n, out, accumulate, (float*)partial, t, n, (hipStream_t)hip_stream));
  return MLLM_OK;
}

}  // extern "C"
