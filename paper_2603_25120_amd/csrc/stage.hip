// Host side of the library: stage handle, argument validation, buffer plan, the launch sequence
// of one stage forward / backward pass, and the C ABI declared in mllm_stage.h.
//
// One call runs every layer of the stage over one packed microbatch (Background and Motivation,
// Fig. 1: the forward and backward boxes of one stage).  Linear operations run over the whole
// packed token matrix; attention runs per instance from a tile list built here from cu_seqlens
// (Model Profiler, "Throughput Profiling").
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/mllm_stage.h"
#include "kernels.h"
#include "attn_items.h"
#include "pinned_ring.h"

using namespace mllm;

namespace {

thread_local std::string g_last_error;

mllm_status_t fail(mllm_status_t st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return st;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(MLLM_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));         \
  } while (0)

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct ParamInfo {
  const char* name;
  int32_t layer;
  int64_t rows, cols;
};

int64_t nqkv_of(const mllm_layer_desc_t& L) { return (int64_t)(L.n_q_heads + 2 * L.n_kv_heads) * L.head_dim; }

}  // namespace

namespace mllm_detail {
void set_last_error(const char* msg) { g_last_error = msg; }
}  // namespace mllm_detail

struct mllm_stage {
  std::vector<mllm_layer_desc_t> layers;
  std::vector<ParamInfo> params;
  std::vector<int> param_off;  // first parameter index of each layer
  int n_vit = 0, n_dec = 0, proj = -1;
  // pinned host staging for the per-call metadata upload; sized by mllm_stage_sizes (hence
  // mutable: that call takes a const handle), so that fwd / bwd neither allocate nor wait
  mutable PinnedRing staging;
};

namespace {

// -------------------------------------------------------------------------------------------
// validation
// -------------------------------------------------------------------------------------------
mllm_status_t check_layer(const mllm_layer_desc_t& L, int i) {
  auto m64 = [](int64_t v) { return v > 0 && v % 64 == 0; };
  if (L.kind == MLLM_LAYER_PROJECTOR) {
    if (!m64(L.d_model) || !m64(L.d_out)) return fail(MLLM_ERR_DESC, "layer %d: projector widths must be positive multiples of 64", i);
    if (L.has_bias != 1) return fail(MLLM_ERR_DESC, "layer %d: projector needs has_bias = 1", i);
    if (L.pool < 0 || L.pool > 64) return fail(MLLM_ERR_DESC, "layer %d: the connector's pooling width must be in 0..64", i);
    if (L.merge < 0 || L.merge > 64) return fail(MLLM_ERR_DESC, "layer %d: the connector's merge width must be in 0..64", i);
    if (L.merge > 1 && L.pool > 1) return fail(MLLM_ERR_DESC, "layer %d: a connector either pools or merges", i);
    if (L.qk_norm != 0) return fail(MLLM_ERR_DESC, "layer %d: a connector has no QK normalisation", i);
    if (L.d_ff != 0) {
      if (!m64(L.d_ff)) return fail(MLLM_ERR_DESC, "layer %d: the connector's hidden width must be 0 or a positive multiple of 64", i);
      if (L.act != MLLM_ACT_GELU_ERF && L.act != MLLM_ACT_GELU_TANH) return fail(MLLM_ERR_DESC, "layer %d: an MLP connector's activation must be GELU", i);
    }
    return MLLM_OK;
  }
  if (L.kind != MLLM_LAYER_VIT && L.kind != MLLM_LAYER_DECODER) return fail(MLLM_ERR_DESC, "layer %d: unknown kind %d", i, L.kind);
  if (L.head_dim != 64 && L.head_dim != 128) return fail(MLLM_ERR_DESC, "layer %d: head_dim must be 64 or 128", i);
  if (L.n_q_heads <= 0 || L.n_kv_heads <= 0 || L.n_q_heads % L.n_kv_heads != 0)
    return fail(MLLM_ERR_DESC, "layer %d: n_q_heads must be a positive multiple of n_kv_heads", i);
  if (L.d_model != L.n_q_heads * L.head_dim) return fail(MLLM_ERR_DESC, "layer %d: d_model != n_q_heads * head_dim", i);
  if (!m64(L.d_model) || !m64(L.d_ff)) return fail(MLLM_ERR_DESC, "layer %d: widths must be positive multiples of 64", i);
  if (L.d_model > 8192) return fail(MLLM_ERR_DESC, "layer %d: d_model above 8192", i);
  if (!(L.norm_eps > 0.f)) return fail(MLLM_ERR_DESC, "layer %d: norm_eps must be positive", i);
  if (L.qk_norm != 0 && L.qk_norm != 1) return fail(MLLM_ERR_DESC, "layer %d: qk_norm must be 0 or 1", i);
  if (L.kind == MLLM_LAYER_VIT) {
    if (L.has_bias != 1) return fail(MLLM_ERR_DESC, "layer %d: ViT layer needs has_bias = 1", i);
    if (L.act != MLLM_ACT_GELU_ERF && L.act != MLLM_ACT_GELU_TANH) return fail(MLLM_ERR_DESC, "layer %d: ViT activation must be GELU", i);
    if (L.n_q_heads != L.n_kv_heads) return fail(MLLM_ERR_DESC, "layer %d: ViT layer needs n_kv_heads == n_q_heads", i);
  } else {
    if (L.has_bias != 0 && L.has_bias != 1) return fail(MLLM_ERR_DESC, "layer %d: decoder layer needs has_bias = 0, or 1 for a QKV bias", i);
    if (L.act != MLLM_ACT_SWIGLU) return fail(MLLM_ERR_DESC, "layer %d: decoder activation must be SwiGLU", i);
    if (!(L.rope_base > 1.f)) return fail(MLLM_ERR_DESC, "layer %d: rope_base must exceed 1", i);
  }
  return MLLM_OK;
}

mllm_status_t check_pack(const mllm_pack_t& p, const char* what) {
  if (p.total_tokens < 0 || p.n_segments < 0) return fail(MLLM_ERR_SHAPE, "%s: negative sizes", what);
  if (!p.cu_seqlens_host) return fail(MLLM_ERR_NULL, "%s: cu_seqlens_host is NULL", what);
  if (p.n_segments > 0 && !p.mask_kind_host) return fail(MLLM_ERR_NULL, "%s: mask_kind_host is NULL", what);
  if (p.cu_seqlens_host[0] != 0) return fail(MLLM_ERR_CU_SEQLENS, "%s: cu_seqlens[0] != 0", what);
  int32_t longest = 0;
  for (int s = 0; s < p.n_segments; s++) {
    int32_t len = p.cu_seqlens_host[s + 1] - p.cu_seqlens_host[s];
    if (len < 0) return fail(MLLM_ERR_CU_SEQLENS, "%s: cu_seqlens decreases at segment %d", what, s);
    longest = std::max(longest, len);
    if (p.mask_kind_host[s] > 1) return fail(MLLM_ERR_MASK_KIND, "%s: mask kind %d at segment %d", what, (int)p.mask_kind_host[s], s);
  }
  if (p.cu_seqlens_host[p.n_segments] != p.total_tokens)
    return fail(MLLM_ERR_CU_SEQLENS, "%s: cu_seqlens ends at %d, total_tokens is %d", what, p.cu_seqlens_host[p.n_segments], p.total_tokens);
  if (p.max_seqlen < longest) return fail(MLLM_ERR_SHAPE, "%s: max_seqlen %d below the longest segment %d", what, p.max_seqlen, longest);
  return MLLM_OK;
}

// Rows the connector produces: the encoder rows, or with pooling the windows of every segment.
int64_t connector_rows(const mllm_stage* st, const mllm_batch_t* b) {
  const int pool = st->proj >= 0 ? st->layers[st->proj].pool : 0;
  const int merge = st->proj >= 0 ? st->layers[st->proj].merge : 0;
  if (merge > 1) return b->img.total_tokens / merge;   // every segment is a multiple (check_batch)
  if (pool <= 1) return b->img.total_tokens;
  int64_t n = 0;
  for (int s = 0; s < b->img.n_segments; s++)
    n += (b->img.cu_seqlens_host[s + 1] - b->img.cu_seqlens_host[s] + pool - 1) / pool;
  return n;
}

mllm_status_t check_batch(const mllm_stage* st, const mllm_batch_t* b) {
  if (!st || !b) return fail(MLLM_ERR_NULL, "stage or batch is NULL");
  mllm_status_t r;
  const bool need_img = st->n_vit > 0 || st->proj >= 0;
  const bool need_seq = st->n_dec > 0 || st->proj >= 0;
  if (need_img && (r = check_pack(b->img, "img")) != MLLM_OK) return r;
  if (need_seq && (r = check_pack(b->seq, "seq")) != MLLM_OK) return r;
  if (st->proj >= 0) {
    const int merge = st->layers[st->proj].merge;
    if (merge > 1)
      for (int sgm = 0; sgm < b->img.n_segments; sgm++)
        if ((b->img.cu_seqlens_host[sgm + 1] - b->img.cu_seqlens_host[sgm]) % merge)
          return fail(MLLM_ERR_SHAPE, "img segment %d: length is no multiple of the connector's merge width %d", sgm, merge);
    const int64_t n_con = connector_rows(st, b);
    if (n_con > 0 && !b->img_to_seq_row_host) return fail(MLLM_ERR_NULL, "img_to_seq_row_host is NULL");
    int64_t prev = -1;
    for (int64_t i = 0; i < n_con; i++) {
      int32_t r0 = b->img_to_seq_row_host[i];
      if (r0 < 0 || r0 >= b->seq.total_tokens) return fail(MLLM_ERR_INDEX, "img_to_seq_row[%lld] = %d out of range", (long long)i, r0);
      if (r0 <= prev) return fail(MLLM_ERR_INDEX, "img_to_seq_row not strictly increasing at %lld", (long long)i);
      prev = r0;
    }
  }
  return MLLM_OK;
}

// -------------------------------------------------------------------------------------------
// buffer plan.  Every offset is a function of (stage, batch) only, so sizes(), fwd() and bwd()
// agree by construction.
// -------------------------------------------------------------------------------------------
struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += align_up(bytes);
    return o;
  }
};

struct LayerSaved {  // byte offsets into `saved`
  size_t x, stats1, n1, qkv, o, lse, x1, stats2, n2, pre, act;
  // QK normalisation only: qkv then keeps the projection's q and k, and qkn [T, nq] holds the
  // normalised (and rotated) q and k in the same columns (its v columns are unused)
  size_t qkn, statsq, statsk;
};

// Attention work lists of one (token space, head counts) combination; layers that agree in these share them.
struct AttnLists {
  bool img;
  int hq, hkv, head_dim;
  size_t q_off = 0, kv_off = 0;     // byte offsets into the metadata blob
  int q_grid = 0, kv_grid = 0;      // grid sizes, known once the lists are built (upload_meta)
};

struct Meta {  // byte offsets into the metadata blob at the head of the workspace
  std::vector<AttnLists> attn;
  size_t tables = 0;                // where the tables below begin (the attention lists come first)
  size_t pos = 0, i2s = 0;
  size_t pool_first = 0, pool_count = 0, row_window = 0;   // pooling connector: window tables
  size_t bytes = 0;
};

struct Plan {
  std::vector<LayerSaved> saved;  // per layer
  size_t saved_bytes = 0;
  Meta meta;
  std::vector<int> attn_of;       // per layer: index into meta.attn (-1: no attention)
  // workspace offsets (after the metadata)
  size_t w_partial = 0;           // fp32 partial sums of norm / bias gradients
  size_t w_a = 0, w_b = 0, w_c = 0, w_d = 0, w_e = 0, w_delta = 0, w_g0 = 0, w_g1 = 0, w_proj = 0, w_split = 0;
  size_t w_qkn = 0;               // QK normalisation: gradient of the normalised q, k  [T, nq]
  // Rotary-angle tables [longest sample, head_dim] fp32, one per distinct (rope_base, head_dim) of the
  // decoder layers; rope_of[i] = index of layer i's table (-1: the layer has none).
  struct RopeTable { float base; int32_t head_dim; size_t off; };
  std::vector<RopeTable> rope_tables;
  std::vector<int> rope_of;
  int64_t longest_seq = 0;
  size_t split_bytes = 0;
  size_t workspace_bytes = 0;
  int64_t T_img = 0, T_seq = 0;
  int64_t T_con = 0;              // rows of the connector (T_img, or the pooling windows)
  int pool = 1;
  int64_t largest_operand_bytes = 0;   // largest [tokens, width] bf16 matrix any GEMM of the stage reads
  double img_pairs = 0, seq_pairs = 0;  // sum over segments of visible (query, key) pairs
};

double visible_pairs(const mllm_pack_t& p) {
  double n = 0;
  for (int s = 0; s < p.n_segments; s++) {
    const double len = p.cu_seqlens_host[s + 1] - p.cu_seqlens_host[s];
    n += p.mask_kind_host[s] == MLLM_MASK_CAUSAL ? 0.5 * len * len : len * len;
  }
  return n;
}

Plan make_plan(const mllm_stage* st, const mllm_batch_t* b) {
  Plan P;
  const bool need_img = st->n_vit > 0 || st->proj >= 0;
  const bool need_seq = st->n_dec > 0 || st->proj >= 0;
  P.T_img = need_img ? b->img.total_tokens : 0;
  P.T_seq = need_seq ? b->seq.total_tokens : 0;
  if (st->proj >= 0) {
    P.pool = std::max(1, (int)st->layers[st->proj].pool);
    P.T_con = connector_rows(st, b);
  }
  if (st->n_vit > 0) P.img_pairs = visible_pairs(b->img);
  if (st->n_dec > 0) P.seq_pairs = visible_pairs(b->seq);
  Bump sv;
  P.saved.resize(st->layers.size());
  for (size_t i = 0; i < st->layers.size(); i++) {
    const mllm_layer_desc_t& L = st->layers[i];
    LayerSaved& S = P.saved[i];
    memset(&S, 0, sizeof S);
    if (L.kind == MLLM_LAYER_PROJECTOR) {
      S.x = sv.take((size_t)P.T_img * L.d_model * 2);   // encoder output
      if (P.pool > 1) S.n1 = sv.take((size_t)P.T_con * L.d_model * 2);   // its pooled rows: the connector's input
      if (L.d_ff) {                                      // MLP connector: hidden pre-activation and activation
        S.pre = sv.take((size_t)P.T_con * L.d_ff * 2);
        S.act = sv.take((size_t)P.T_con * L.d_ff * 2);
      }
      continue;
    }
    const size_t T = L.kind == MLLM_LAYER_VIT ? P.T_img : P.T_seq;
    const size_t d = L.d_model, f = L.d_ff;
    S.x = sv.take(T * d * 2);
    S.stats1 = sv.take(T * 2 * 4);
    S.n1 = sv.take(T * d * 2);
    S.qkv = sv.take(T * nqkv_of(L) * 2);
    if (L.qk_norm) {
      S.qkn = sv.take(T * nqkv_of(L) * 2);
      S.statsq = sv.take(T * 2 * 4);
      S.statsk = sv.take(T * 2 * 4);
    }
    S.o = sv.take(T * d * 2);
    S.lse = sv.take(T * L.n_q_heads * 4);
    S.x1 = sv.take(T * d * 2);
    S.stats2 = sv.take(T * 2 * 4);
    S.n2 = sv.take(T * d * 2);
    S.pre = sv.take(T * (L.kind == MLLM_LAYER_VIT ? f : 2 * f) * 2);
    S.act = sv.take(T * f * 2);
  }
  P.saved_bytes = std::max<size_t>(sv.off, ALIGN);

  Bump ws;
  Meta& M = P.meta;
  P.attn_of.assign(st->layers.size(), -1);
  for (size_t i = 0; i < st->layers.size(); i++) {
    const mllm_layer_desc_t& L = st->layers[i];
    if (L.kind == MLLM_LAYER_PROJECTOR) continue;
    const bool img = L.kind == MLLM_LAYER_VIT;
    int found = -1;
    for (size_t k = 0; k < M.attn.size(); k++)
      if (M.attn[k].img == img && M.attn[k].hq == L.n_q_heads && M.attn[k].hkv == L.n_kv_heads && M.attn[k].head_dim == L.head_dim)
        found = (int)k;
    if (found < 0) {
      AttnLists A;
      A.img = img; A.hq = L.n_q_heads; A.hkv = L.n_kv_heads; A.head_dim = L.head_dim;
      const mllm_pack_t& pk = img ? b->img : b->seq;
      A.q_off = ws.take(attn_list_bytes(pk, ATTN_FWD_Q_TILE, L.n_q_heads));
      A.kv_off = ws.take(attn_list_bytes(pk, ATTN_BWD_KV_TILE, L.n_kv_heads));
      found = (int)M.attn.size();
      M.attn.push_back(A);
    }
    P.attn_of[i] = found;
  }
  M.tables = ws.off;
  if (st->n_dec > 0) M.pos = ws.take(sizeof(int32_t) * P.T_seq);
  if (st->proj >= 0) M.i2s = ws.take(sizeof(int32_t) * P.T_con);
  if (st->proj >= 0 && P.pool > 1) {
    M.pool_first = ws.take(sizeof(int32_t) * P.T_con);
    M.pool_count = ws.take(sizeof(int32_t) * P.T_con);
    M.row_window = ws.take(sizeof(int32_t) * P.T_img);
  }
  M.bytes = ws.off;

  size_t part = 0, a = 0, bb = 0, c = 0, e = 0, delta = 0, g = 0, proj = 0, split = 0, qkn = 0;
  for (const mllm_layer_desc_t& L : st->layers) {
    if (L.kind == MLLM_LAYER_PROJECTOR) {
      const int64_t d_in = (int64_t)L.d_model * std::max(1, (int)L.merge);
      proj = (size_t)P.T_con * L.d_out * 2;
      P.largest_operand_bytes = std::max<int64_t>(P.largest_operand_bytes, (int64_t)P.T_img * std::max(std::max(L.d_model, L.d_out), L.d_ff) * 2);
      if (L.d_ff) {
        split = std::max(split, gemm_splitk_ws_bytes(d_in, L.d_ff, P.T_con));
        split = std::max(split, gemm_splitk_ws_bytes(L.d_ff, L.d_out, P.T_con));
        a = std::max(a, (size_t)P.T_con * L.d_ff * 2);
      } else {
        split = std::max(split, gemm_splitk_ws_bytes(d_in, L.d_out, P.T_con));
      }
      if (P.pool > 1) c = std::max(c, (size_t)P.T_con * L.d_model * 2);   // gradient of the pooled rows
      part = std::max(part, (size_t)colsum_partial_rows(P.T_con) * std::max(L.d_out, L.d_ff) * 4);
      g = std::max(g, (size_t)P.T_img * L.d_model * 2);
      g = std::max(g, (size_t)P.T_seq * L.d_out * 2);
      continue;
    }
    const size_t T = L.kind == MLLM_LAYER_VIT ? P.T_img : P.T_seq;
    const size_t d = L.d_model, f = L.d_ff, nq = nqkv_of(L);
    const size_t widest = std::max<size_t>(std::max(d, 2 * f), nq);
    P.largest_operand_bytes = std::max<int64_t>(P.largest_operand_bytes, (int64_t)(T * widest * 2));
    // the attention kernels' 32-bit row offsets may run 256 rows past the last token
    P.largest_operand_bytes = std::max<int64_t>(P.largest_operand_bytes, (int64_t)((T + 256) * std::max(nq, d) * 2));
    part = std::max(part, (size_t)norm_bwd_partial_rows(T) * d * 4 * 3);
    part = std::max(part, (size_t)colsum_partial_rows(T) * widest * 4);
    a = std::max(a, T * f * 2);
    bb = std::max(bb, L.kind == MLLM_LAYER_DECODER ? T * 2 * f * 2 : 0);
    c = std::max(c, T * d * 2);
    e = std::max(e, T * nq * 2);
    if (L.qk_norm) qkn = std::max(qkn, T * nq * 2);
    delta = std::max(delta, T * L.n_q_heads * 4);
    g = std::max(g, T * d * 2);
    const int64_t fup = L.kind == MLLM_LAYER_VIT ? f : 2 * f;
    split = std::max(split, gemm_splitk_ws_bytes(f, d, T));
    split = std::max(split, gemm_splitk_ws_bytes(d, fup, T));
    split = std::max(split, gemm_splitk_ws_bytes(d, d, T));
    split = std::max(split, gemm_splitk_ws_bytes(d, nq, T));
  }
  P.rope_of.assign(st->layers.size(), -1);
  if (st->n_dec > 0) {
    for (int sgm = 0; sgm < b->seq.n_segments; sgm++)
      P.longest_seq = std::max<int64_t>(P.longest_seq, b->seq.cu_seqlens_host[sgm + 1] - b->seq.cu_seqlens_host[sgm]);
    for (size_t i = 0; i < st->layers.size(); i++) {
      const mllm_layer_desc_t& L = st->layers[i];
      if (L.kind != MLLM_LAYER_DECODER) continue;
      int found = -1;
      for (size_t k = 0; k < P.rope_tables.size(); k++)
        if (P.rope_tables[k].base == L.rope_base && P.rope_tables[k].head_dim == L.head_dim) found = (int)k;
      if (found < 0) {
        found = (int)P.rope_tables.size();
        P.rope_tables.push_back({L.rope_base, L.head_dim, ws.take((size_t)std::max<int64_t>(P.longest_seq, 1) * L.head_dim * 4)});
      }
      P.rope_of[i] = found;
    }
  }
  P.split_bytes = split;
  P.w_split = ws.take(split);
  P.w_partial = ws.take(part);
  P.w_a = ws.take(a);
  P.w_b = ws.take(bb);
  P.w_c = ws.take(c);
  P.w_d = ws.take(c);
  P.w_e = ws.take(e);
  P.w_qkn = ws.take(qkn);
  P.w_delta = ws.take(delta);
  P.w_g0 = ws.take(g);
  P.w_g1 = ws.take(g);
  P.w_proj = ws.take(proj);
  P.workspace_bytes = std::max<size_t>(ws.off, ALIGN);
  return P;
}

// -------------------------------------------------------------------------------------------
// metadata: attention tile lists (heaviest first), positions, scatter rows
// -------------------------------------------------------------------------------------------
// Residents per XCD (32 CUs): the forward and dQ kernels keep two workgroups per CU, the dK/dV kernel
// two for heads of 64 and one for heads of 128.
int kv_residents(int head_dim) { return head_dim == 64 ? 64 : 32; }

mllm_status_t upload_meta(mllm_stage* st, const mllm_batch_t* b, Plan& P, void* workspace,
                          hipStream_t s) {
  Meta& M = P.meta;
  if (M.bytes == 0) return MLLM_OK;
  PinnedRing::Slot* slot = nullptr;
  HIP_TRY(st->staging.acquire(M.bytes, &slot));
  char* h = (char*)slot->p;
  memset(h + M.tables, 0, M.bytes - M.tables);
  for (AttnLists& A : M.attn) {
    const mllm_pack_t& pk = A.img ? b->img : b->seq;
    A.q_grid = build_attn_list(pk, ATTN_FWD_Q_TILE, false, A.hkv, A.hq / A.hkv, 64, h + A.q_off);
    A.kv_grid = build_attn_list(pk, ATTN_BWD_KV_TILE, true, A.hkv, A.hq / A.hkv, kv_residents(A.head_dim), h + A.kv_off);
  }
  if (st->n_dec > 0) {
    int32_t* pos = (int32_t*)(h + M.pos);
    for (int sgm = 0; sgm < b->seq.n_segments; sgm++)
      for (int t = b->seq.cu_seqlens_host[sgm]; t < b->seq.cu_seqlens_host[sgm + 1]; t++)
        pos[t] = t - b->seq.cu_seqlens_host[sgm];
  }
  if (st->proj >= 0 && P.T_con > 0) memcpy(h + M.i2s, b->img_to_seq_row_host, sizeof(int32_t) * P.T_con);
  if (st->proj >= 0 && P.pool > 1) {
    int32_t* first = (int32_t*)(h + M.pool_first);
    int32_t* count = (int32_t*)(h + M.pool_count);
    int32_t* window = (int32_t*)(h + M.row_window);
    int64_t j = 0;
    for (int sgm = 0; sgm < b->img.n_segments; sgm++) {
      const int end = b->img.cu_seqlens_host[sgm + 1];
      for (int r = b->img.cu_seqlens_host[sgm]; r < end; r += P.pool, j++) {
        first[j] = r;
        count[j] = std::min(P.pool, end - r);
        for (int q = 0; q < count[j]; q++) window[r + q] = (int32_t)j;
      }
    }
  }
  // the lists are reserved at their upper bound; only the entries of the launch grids are copied
  char* w = (char*)workspace;
  for (const AttnLists& A : M.attn) {
    if (A.q_grid) HIP_TRY(hipMemcpyAsync(w + A.q_off, h + A.q_off, (size_t)A.q_grid * sizeof(AttnItem), hipMemcpyHostToDevice, s));
    if (A.kv_grid) HIP_TRY(hipMemcpyAsync(w + A.kv_off, h + A.kv_off, (size_t)A.kv_grid * sizeof(AttnItem), hipMemcpyHostToDevice, s));
  }
  if (M.bytes > M.tables) HIP_TRY(hipMemcpyAsync(w + M.tables, h + M.tables, M.bytes - M.tables, hipMemcpyHostToDevice, s));
  HIP_TRY(st->staging.commit(slot, s));
  return MLLM_OK;
}

hipError_t gemm(const void* a, int64_t lda, int a_layout, const void* b, int64_t ldb, int b_layout,
                void* c, int64_t ldc, int64_t m, int64_t n, int64_t k, int out_fp32, int accumulate,
                const void* bias, const void* res, int64_t ldres, hipStream_t s,
                void* splitk_ws = nullptr, size_t splitk_ws_bytes = 0) {
  GemmArgs g;
  g.splitk_ws = splitk_ws; g.splitk_ws_bytes = splitk_ws_bytes;
  g.a = a; g.b = b; g.c = c; g.m = m; g.n = n; g.k = k; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.a_layout = a_layout; g.b_layout = b_layout; g.out_fp32 = out_fp32; g.accumulate = accumulate;
  g.bias = bias; g.residual = res; g.ldres = ldres;
  return launch_gemm(g, s);
}
// Y[T,n] = X[T,k].W[k,n] (+bias) (+res)
hipError_t linear_fwd(const void* x, const void* w, void* y, int64_t T, int64_t k, int64_t n,
                      const void* bias, const void* res, hipStream_t s) {
  return gemm(x, k, 0, w, n, 0, y, n, T, n, k, 0, 0, bias, res, n, s);
}
// Y[T,n] = X[T,k].W[k,n] (+bias) with the leading rope_cols columns (heads of head_dim) rotated by the
// rotary angle of each row's position
hipError_t linear_fwd_rope(const void* x, const void* w, void* y, int64_t T, int64_t k, int64_t n, const void* bias,
                           const float* table, const int32_t* pos, int64_t rope_cols, int32_t head_dim, hipStream_t s) {
  GemmArgs g;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.a = x; g.b = w; g.c = y; g.m = T; g.n = n; g.k = k; g.lda = k; g.ldb = n; g.ldc = n;
  g.a_layout = 0; g.b_layout = 0; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = bias; g.residual = nullptr; g.ldres = 0;
  g.rope_table = table; g.rope_pos = pos; g.rope_cols = rope_cols; g.rope_head_dim = head_dim;
  return launch_gemm(g, s);
}
// [gate | up][T,2f] = X[T,k].W[k,2f] and act[T,f] = silu(gate) * up in the same pass
hipError_t linear_fwd_swiglu(const void* x, const void* w, void* pre, void* act, int64_t T, int64_t k,
                             int64_t n, hipStream_t s) {
  GemmArgs g;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.a = x; g.b = w; g.c = pre; g.m = T; g.n = n; g.k = k; g.lda = k; g.ldb = n; g.ldc = n;
  g.a_layout = 0; g.b_layout = 0; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = nullptr; g.residual = nullptr; g.ldres = 0;
  g.swiglu_act = act;
  return launch_gemm(g, s);
}
// dX[T,k] = dY[T,n].W[k,n]^T
hipError_t linear_dx(const void* dy, const void* w, void* dx, int64_t T, int64_t k, int64_t n, hipStream_t s) {
  return gemm(dy, n, 0, w, n, 1, dx, k, T, k, n, 0, 0, nullptr, nullptr, 0, s);
}
// [d gate | d up][T,2f] from dY[T,d], W_d[f,d] and pre = [gate | up][T,2f]: dA = dY.W_d^T stays in registers
hipError_t linear_dx_swiglu(const void* dy, const void* w, const void* pre, void* dpre, int64_t T, int64_t f,
                            int64_t d, hipStream_t s) {
  GemmArgs g;
  g.splitk_ws = nullptr; g.splitk_ws_bytes = 0;
  g.a = dy; g.b = w; g.c = nullptr; g.m = T; g.n = f; g.k = d; g.lda = d; g.ldb = d; g.ldc = 2 * f;
  g.a_layout = 0; g.b_layout = 1; g.out_fp32 = 0; g.accumulate = 0;
  g.bias = nullptr; g.residual = nullptr; g.ldres = 0;
  g.swiglu_pre = pre; g.swiglu_dpre = dpre;
  return launch_gemm(g, s);
}
// dW[k,n] (+)= X[T,k]^T.dY[T,n]
struct SplitWs { void* p; size_t bytes; };
hipError_t linear_dw(const void* x, const void* dy, void* dw, int64_t T, int64_t k, int64_t n, int accumulate,
                     hipStream_t s, SplitWs ws) {
  return gemm(x, k, 1, dy, n, 0, dw, n, k, n, T, 1, accumulate, nullptr, nullptr, 0, s, ws.p, ws.bytes);
}

// qk: the [T, nq] matrix whose q and k columns attention reads; v: the one whose v columns it reads
// (the same matrix unless the layer normalises q and k).
AttnArgs attn_args(const mllm_layer_desc_t& L, char* qk, char* v, int64_t T, const char* ws, const Plan& P, bool img,
                   int list_index) {
  const AttnLists& A = P.meta.attn[list_index];
  AttnArgs a;
  memset(&a, 0, sizeof a);
  const int64_t nq = nqkv_of(L);
  a.q = qk;
  a.k = qk + (int64_t)L.n_q_heads * L.head_dim * 2;
  a.v = v + (int64_t)(L.n_q_heads + L.n_kv_heads) * L.head_dim * 2;
  a.q_stride = a.kv_stride = nq;
  a.o_stride = L.d_model;
  a.total_tokens = (int32_t)T;
  a.n_q_heads = L.n_q_heads; a.n_kv_heads = L.n_kv_heads; a.head_dim = L.head_dim;
  a.q_list = ws + A.q_off;
  a.kv_list = ws + A.kv_off;
  a.q_grid = A.q_grid;
  a.kv_grid = A.kv_grid;
  a.fwd_flops = 4.0 * (img ? P.img_pairs : P.seq_pairs) * L.n_q_heads * L.head_dim;
  return a;
}

#define K_TRY(expr)                                                                        \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return fail(MLLM_ERR_HIP, "launch failed (%s): %s", #expr, hipGetErrorString(e_));   \
  } while (0)

// -------------------------------------------------------------------------------------------
// one transformer layer, forward.  x -> y; everything backward needs goes to `saved`.
// -------------------------------------------------------------------------------------------
mllm_status_t layer_fwd(const mllm_layer_desc_t& L, const void* const* prm, const LayerSaved& S,
                        char* saved, char* ws, const Plan& P, int64_t T, void* y, const float* rope_table,
                        int attn_list, hipStream_t s) {
  const bool vit = L.kind == MLLM_LAYER_VIT;
  const int64_t d = L.d_model, f = L.d_ff, nq = nqkv_of(L);
  char* x = saved + S.x;
  char* n1 = saved + S.n1;
  char* qkv = saved + S.qkv;
  char* o = saved + S.o;
  char* x1 = saved + S.x1;
  char* n2 = saved + S.n2;
  char* pre = saved + S.pre;
  char* act = saved + S.act;
  // parameter slots
  const void *g1, *b1n = nullptr, *wqkv, *bqkv = nullptr, *wo, *bo = nullptr, *g2, *b2n = nullptr,
             *wup, *bup = nullptr, *wdn, *bdn = nullptr;
  if (vit) { g1 = prm[0]; b1n = prm[1]; wqkv = prm[2]; bqkv = prm[3]; wo = prm[4]; bo = prm[5];
             g2 = prm[6]; b2n = prm[7]; wup = prm[8]; bup = prm[9]; wdn = prm[10]; bdn = prm[11]; }
  else if (L.has_bias) { g1 = prm[0]; wqkv = prm[1]; bqkv = prm[2]; wo = prm[3]; g2 = prm[4]; wup = prm[5]; wdn = prm[6]; }
  else { g1 = prm[0]; wqkv = prm[1]; wo = prm[2]; g2 = prm[3]; wup = prm[4]; wdn = prm[5]; }
  const int n_base = vit ? 12 : (L.has_bias ? 7 : 6);   // the QK-norm gains follow the layer's other tensors
  const int64_t q_cols = (int64_t)L.n_q_heads * L.head_dim, k_cols = (int64_t)L.n_kv_heads * L.head_dim;

  K_TRY(launch_norm_fwd(vit ? 0 : 1, x, g1, b1n, n1, (float*)(saved + S.stats1), T, d, d, L.norm_eps, s));
  // Rotary positions ride on the QKV projection's epilogue whenever that product takes the
  // large-tile kernel and nothing sits between the projection and the rotation.
  const bool rope_fused = !vit && !L.qk_norm && (q_cols + k_cols) % 128 == 0 && gemm_rope_fusable(T, nq, d, L.head_dim);
  if (rope_fused)
    K_TRY(linear_fwd_rope(n1, wqkv, qkv, T, d, nq, bqkv, rope_table, (const int32_t*)(ws + P.meta.pos), q_cols + k_cols,
                          L.head_dim, s));
  else
    K_TRY(linear_fwd(n1, wqkv, qkv, T, d, nq, bqkv, nullptr, s));
  char* qk = qkv;
  if (L.qk_norm) {
    qk = saved + S.qkn;
    K_TRY(launch_norm_fwd(1, qkv, prm[n_base], nullptr, qk, (float*)(saved + S.statsq), T, q_cols, nq, L.norm_eps, s));
    K_TRY(launch_norm_fwd(1, qkv + q_cols * 2, prm[n_base + 1], nullptr, qk + q_cols * 2,
                          (float*)(saved + S.statsk), T, k_cols, nq, L.norm_eps, s));
  }
  if (!vit && !rope_fused)
    K_TRY(launch_rope(qk, (const int32_t*)(ws + P.meta.pos), T, nq, 0, L.n_q_heads + L.n_kv_heads,
                      L.head_dim, L.rope_base, 0, s));
  AttnArgs a = attn_args(L, qk, qkv, T, ws, P, vit, attn_list);
  a.o = o;
  a.lse = (float*)(saved + S.lse);
  K_TRY(launch_attn_fwd(a, s));
  K_TRY(linear_fwd(o, wo, x1, T, d, d, bo, x, s));
  K_TRY(launch_norm_fwd(vit ? 0 : 1, x1, g2, b2n, n2, (float*)(saved + S.stats2), T, d, d, L.norm_eps, s));
  if (!vit && gemm_swiglu_fusable(T, 2 * f, d)) {
    K_TRY(linear_fwd_swiglu(n2, wup, pre, act, T, d, 2 * f, s));
  } else {
    K_TRY(linear_fwd(n2, wup, pre, T, d, vit ? f : 2 * f, bup, nullptr, s));
    K_TRY(launch_act_fwd(L.act, pre, act, T, f, s));
  }
  K_TRY(linear_fwd(act, wdn, y, T, f, d, bdn, x1, s));
  return MLLM_OK;
}

// dy -> dx (both bf16 [T,d]); parameter gradients into dprm (fp32).
mllm_status_t layer_bwd(const mllm_layer_desc_t& L, const void* const* prm, void* const* dprm,
                        int accumulate, const LayerSaved& S, const char* saved, char* ws,
                        const Plan& P, int64_t T, const void* dy, void* dx, const float* rope_table,
                        int attn_list, hipStream_t s, bool dy_colsum_done, float* dx_colsum) {
  // dy_colsum_done: the layer above has already formed the column sums of dy (this layer's b_2
  // gradient) while writing dy; dx_colsum: where to leave the column sums of dx for the layer below.
  const bool vit = L.kind == MLLM_LAYER_VIT;
  const int64_t d = L.d_model, f = L.d_ff, nq = nqkv_of(L);
  const char* x = saved + S.x;
  const char* n1 = saved + S.n1;
  char* qkv = const_cast<char*>(saved + S.qkv);
  const char* o = saved + S.o;
  const char* x1 = saved + S.x1;
  const char* n2 = saved + S.n2;
  const char* pre = saved + S.pre;
  const char* act = saved + S.act;
  float* partial = (float*)(ws + P.w_partial);
  const SplitWs split{ws + P.w_split, P.split_bytes};
  char* wa = ws + P.w_a;      // d act            [T, f]
  char* wb = ws + P.w_b;      // d (gate|up)      [T, 2f]  (decoder)
  char* wc = ws + P.w_c;      // d n2 / d o / d n1 [T, d]
  char* wd = ws + P.w_d;      // d x1             [T, d]
  char* we = ws + P.w_e;      // d qkv            [T, nq]
  int ig1, ib1n = -1, iwqkv, ibqkv = -1, iwo, ibo = -1, ig2, ib2n = -1, iwup, ibup = -1, iwdn, ibdn = -1;
  if (vit) { ig1 = 0; ib1n = 1; iwqkv = 2; ibqkv = 3; iwo = 4; ibo = 5; ig2 = 6; ib2n = 7; iwup = 8; ibup = 9; iwdn = 10; ibdn = 11; }
  else if (L.has_bias) { ig1 = 0; iwqkv = 1; ibqkv = 2; iwo = 3; ig2 = 4; iwup = 5; iwdn = 6; }
  else { ig1 = 0; iwqkv = 1; iwo = 2; ig2 = 3; iwup = 4; iwdn = 5; }
  const int64_t fup = vit ? f : 2 * f;

  // MLP
  K_TRY(linear_dw(act, dy, dprm[iwdn], T, f, d, accumulate, s, split));
  if (vit && !dy_colsum_done) K_TRY(launch_colsum(dy, d, (float*)dprm[ibdn], accumulate, partial, T, d, s));
  char* dpre = vit ? wa : wb;
  if (!vit && gemm_swiglu_bwd_fusable(T, f, d)) {
    K_TRY(linear_dx_swiglu(dy, prm[iwdn], pre, dpre, T, f, d, s));
  } else {
    K_TRY(linear_dx(dy, prm[iwdn], wa, T, f, d, s));
    if (vit)   // the bias gradient (column sums of dpre) comes out of the same pass
      K_TRY(launch_gelu_bwd_colsum(L.act, wa, pre, dpre, (float*)dprm[ibup], accumulate, partial, T, f, s));
    else
      K_TRY(launch_act_bwd(L.act, wa, pre, dpre, T, f, s));
  }
  K_TRY(linear_dw(n2, dpre, dprm[iwup], T, d, fup, accumulate, s, split));
  K_TRY(linear_dx(dpre, prm[iwup], wc, T, d, fup, s));
  // the gradient that leaves this norm is that of the output projection's output: its column sums are
  // the projection's bias gradient, formed in the same pass where the row width allows
  const bool bo_fused = vit && norm_bwd_colsum_fusable(d);
  K_TRY(launch_norm_bwd(vit ? 0 : 1, wc, x1, prm[ig2], (const float*)(saved + S.stats2), dy, wd,
                        (float*)dprm[ig2], vit ? (float*)dprm[ib2n] : nullptr, accumulate, partial, T, d, d, s,
                        bo_fused ? (float*)dprm[ibo] : nullptr));
  // attention block
  K_TRY(linear_dw(o, wd, dprm[iwo], T, d, d, accumulate, s, split));
  if (vit && !bo_fused) K_TRY(launch_colsum(wd, d, (float*)dprm[ibo], accumulate, partial, T, d, s));
  K_TRY(linear_dx(wd, prm[iwo], wc, T, d, d, s));
  // With QK normalisation the gradient of the normalised q, k goes to a matrix of its own (same
  // columns as in d qkv); the norm's backward then writes the gradient of the projection's q, k
  // beside dV in d qkv.
  const int n_base = vit ? 12 : (L.has_bias ? 7 : 6);
  const int64_t q_cols = (int64_t)L.n_q_heads * L.head_dim, k_cols = (int64_t)L.n_kv_heads * L.head_dim;
  char* qk = L.qk_norm ? const_cast<char*>(saved + S.qkn) : qkv;
  char* dqk = L.qk_norm ? ws + P.w_qkn : we;
  AttnArgs a = attn_args(L, qk, qkv, T, ws, P, vit, attn_list);
  a.o = const_cast<char*>(o);
  a.lse = (float*)const_cast<char*>(saved + S.lse);
  a.d_o = wc;
  a.dq = dqk;
  a.dk = dqk + q_cols * 2;
  a.dv = we + (q_cols + k_cols) * 2;
  a.delta = (float*)(ws + P.w_delta);
  a.rope_table = vit ? nullptr : rope_table;   // dq, dk leave the kernels rotated back (the rotation's gradient)
  K_TRY(launch_attn_bwd(a, s));
  if (L.qk_norm) {
    K_TRY(launch_norm_bwd(1, dqk, qkv, prm[n_base], (const float*)(saved + S.statsq), nullptr, we,
                          (float*)dprm[n_base], nullptr, accumulate, partial, T, q_cols, nq, s));
    K_TRY(launch_norm_bwd(1, dqk + q_cols * 2, qkv + q_cols * 2, prm[n_base + 1], (const float*)(saved + S.statsk),
                          nullptr, we + q_cols * 2, (float*)dprm[n_base + 1], nullptr, accumulate, partial,
                          T, k_cols, nq, s));
  }
  K_TRY(linear_dw(n1, we, dprm[iwqkv], T, d, nq, accumulate, s, split));
  if (ibqkv >= 0) K_TRY(launch_colsum(we, nq, (float*)dprm[ibqkv], accumulate, partial, T, nq, s));
  K_TRY(linear_dx(we, prm[iwqkv], wc, T, d, nq, s));
  K_TRY(launch_norm_bwd(vit ? 0 : 1, wc, x, prm[ig1], (const float*)(saved + S.stats1), wd, dx,
                        (float*)dprm[ig1], vit ? (float*)dprm[ib1n] : nullptr, accumulate, partial, T, d, d, s, dx_colsum));
  return MLLM_OK;
}

mllm_status_t check_plan(const Plan& P) {
  if (P.largest_operand_bytes > GEMM_MAX_OPERAND_BYTES)
    return fail(MLLM_ERR_SHAPE, "microbatch too large: a [tokens, width] matrix of %lld bytes exceeds the 4 GiB the GEMM kernels address",
                (long long)P.largest_operand_bytes);
  return MLLM_OK;
}

mllm_status_t check_io(const mllm_stage* st, const mllm_batch_t* b, const void* const* params,
                       const Plan& P, size_t saved_bytes, size_t workspace_bytes, const void* saved,
                       const void* workspace) {
  if (!params) return fail(MLLM_ERR_NULL, "params is NULL");
  for (size_t i = 0; i < st->params.size(); i++)
    if (!params[i]) return fail(MLLM_ERR_NULL, "params[%zu] (%s) is NULL", i, st->params[i].name);
  if (!saved || !workspace) return fail(MLLM_ERR_NULL, "saved or workspace is NULL");
  if (((uintptr_t)saved | (uintptr_t)workspace) % ALIGN) return fail(MLLM_ERR_WORKSPACE, "saved and workspace must be 256-byte aligned");
  if (saved_bytes < P.saved_bytes) return fail(MLLM_ERR_WORKSPACE, "saved buffer has %zu bytes, %zu needed", saved_bytes, P.saved_bytes);
  if (workspace_bytes < P.workspace_bytes) return fail(MLLM_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, P.workspace_bytes);
  (void)b;
  return MLLM_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

const char* mllm_last_error(void) { return g_last_error.c_str(); }

mllm_status_t mllm_stage_create(const mllm_stage_desc_t* desc, mllm_stage_t** out) {
  if (!desc || !out) return fail(MLLM_ERR_NULL, "desc or out is NULL");
  *out = nullptr;
  if (desc->n_layers <= 0 || !desc->layers) return fail(MLLM_ERR_DESC, "stage needs at least one layer");
  mllm_stage* st = new mllm_stage();
  int phase = 0;  // 0: ViT layers, 1: after projector / decoder layers
  int64_t width = -1;
  for (int i = 0; i < desc->n_layers; i++) {
    const mllm_layer_desc_t& L = desc->layers[i];
    mllm_status_t r = check_layer(L, i);
    if (r != MLLM_OK) { delete st; return r; }
    if (width >= 0 && L.d_model != width) { delete st; return fail(MLLM_ERR_DESC, "layer %d: input width %d does not follow the previous layer's %lld", i, L.d_model, (long long)width); }
    if (L.kind == MLLM_LAYER_VIT) {
      if (phase != 0) { delete st; return fail(MLLM_ERR_DESC, "layer %d: ViT layer after projector / decoder", i); }
      st->n_vit++;
      width = L.d_model;
    } else if (L.kind == MLLM_LAYER_PROJECTOR) {
      if (phase != 0) { delete st; return fail(MLLM_ERR_DESC, "layer %d: projector must come before the decoder layers and only once", i); }
      st->proj = i;
      phase = 1;
      width = L.d_out;
    } else {
      if (st->n_vit > 0 && st->proj < 0) { delete st; return fail(MLLM_ERR_DESC, "layer %d: decoder after ViT needs a projector in between", i); }
      phase = 1;
      st->n_dec++;
      width = L.d_model;
    }
    st->layers.push_back(L);
    st->param_off.push_back((int)st->params.size());
    const int64_t d = L.d_model, f = L.d_ff, nq = nqkv_of(L);
    if (L.kind == MLLM_LAYER_VIT) {
      const ParamInfo ps[] = {{"ln1_g", i, 1, d}, {"ln1_b", i, 1, d}, {"w_qkv", i, d, nq}, {"b_qkv", i, 1, nq},
                              {"w_o", i, d, d}, {"b_o", i, 1, d}, {"ln2_g", i, 1, d}, {"ln2_b", i, 1, d},
                              {"w_1", i, d, f}, {"b_1", i, 1, f}, {"w_2", i, f, d}, {"b_2", i, 1, d}};
      st->params.insert(st->params.end(), std::begin(ps), std::end(ps));
    } else if (L.kind == MLLM_LAYER_DECODER) {
      st->params.push_back({"rms1_g", i, 1, d});
      st->params.push_back({"w_qkv", i, d, nq});
      if (L.has_bias) st->params.push_back({"b_qkv", i, 1, nq});
      const ParamInfo ps[] = {{"w_o", i, d, d}, {"rms2_g", i, 1, d}, {"w_gu", i, d, 2 * f}, {"w_d", i, f, d}};
      st->params.insert(st->params.end(), std::begin(ps), std::end(ps));
    } else if (L.d_ff) {
      const int64_t d_in = d * std::max(1, (int)L.merge);
      const ParamInfo ps[] = {{"w_p1", i, d_in, f}, {"b_p1", i, 1, f}, {"w_p2", i, f, L.d_out}, {"b_p2", i, 1, L.d_out}};
      st->params.insert(st->params.end(), std::begin(ps), std::end(ps));
    } else {
      const int64_t d_in = d * std::max(1, (int)L.merge);
      const ParamInfo ps[] = {{"w_p", i, d_in, L.d_out}, {"b_p", i, 1, L.d_out}};
      st->params.insert(st->params.end(), std::begin(ps), std::end(ps));
    }
    if (L.kind != MLLM_LAYER_PROJECTOR && L.qk_norm) {
      st->params.push_back({"qkn_q_g", i, 1, (int64_t)L.n_q_heads * L.head_dim});
      st->params.push_back({"qkn_k_g", i, 1, (int64_t)L.n_kv_heads * L.head_dim});
    }
  }
  *out = st;
  return MLLM_OK;
}

void mllm_stage_destroy(mllm_stage_t* st) {
  if (!st) return;
  st->staging.destroy();
  delete st;
}

size_t mllm_stage_param_count(const mllm_stage_t* st) { return st ? st->params.size() : 0; }

mllm_status_t mllm_stage_param_info(const mllm_stage_t* st, size_t i, const char** name, int32_t* layer,
                                    int64_t* rows, int64_t* cols) {
  if (!st) return fail(MLLM_ERR_NULL, "stage is NULL");
  if (i >= st->params.size()) return fail(MLLM_ERR_SHAPE, "parameter index %zu out of range", i);
  if (name) *name = st->params[i].name;
  if (layer) *layer = st->params[i].layer;
  if (rows) *rows = st->params[i].rows;
  if (cols) *cols = st->params[i].cols;
  return MLLM_OK;
}

mllm_status_t mllm_stage_sizes(const mllm_stage_t* st, const mllm_batch_t* b, size_t* saved_bytes,
                               size_t* workspace_bytes) {
  mllm_status_t r = check_batch(st, b);
  if (r != MLLM_OK) return r;
  Plan P = make_plan(st, b);
  if ((r = check_plan(P)) != MLLM_OK) return r;
  // The staging ring grows here, where the caller sizes its own buffers, so that fwd / bwd find it
  // large enough.  Best effort: a failure (no device in this process) is left to fwd / bwd, which
  // grow the slot they take if they must and report the error then.
  if (P.meta.bytes && st->staging.reserve(P.meta.bytes) != hipSuccess) (void)hipGetLastError();
  if (saved_bytes) *saved_bytes = P.saved_bytes;
  if (workspace_bytes) *workspace_bytes = P.workspace_bytes;
  return MLLM_OK;
}

mllm_status_t mllm_stage_fwd(mllm_stage_t* st, const mllm_batch_t* b, const void* const* params,
                             const void* x_img, const void* x_seq, void* y, void* saved_v,
                             size_t saved_bytes, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  mllm_status_t r = check_batch(st, b);
  if (r != MLLM_OK) return r;
  Plan P = make_plan(st, b);
  if ((r = check_plan(P)) != MLLM_OK) return r;
  if ((r = check_io(st, b, params, P, saved_bytes, workspace_bytes, saved_v, workspace)) != MLLM_OK) return r;
  const bool need_img = st->n_vit > 0 || st->proj >= 0;
  const bool need_seq = st->n_dec > 0 || st->proj >= 0;
  if (need_img && P.T_img > 0 && !x_img) return fail(MLLM_ERR_NULL, "x_img is NULL");
  if (need_seq && P.T_seq > 0 && !x_seq) return fail(MLLM_ERR_NULL, "x_seq is NULL");
  if (!y) return fail(MLLM_ERR_NULL, "y is NULL");
  hipStream_t s = (hipStream_t)hip_stream;
  char* saved = (char*)saved_v;
  char* ws = (char*)workspace;
  if ((r = upload_meta(st, b, P, workspace, s)) != MLLM_OK) return r;
  for (const Plan::RopeTable& t : P.rope_tables)
    K_TRY(launch_rope_table((float*)(ws + t.off), P.longest_seq, t.head_dim, t.base, s));

  const int n = (int)st->layers.size();
  for (int i = 0; i < n; i++) {
    const mllm_layer_desc_t& L = st->layers[i];
    const bool last = i == n - 1;
    const void* const* prm = params + st->param_off[i];
    if (L.kind == MLLM_LAYER_PROJECTOR) {
      // input = x_img if this is the first layer (copied so that backward owns it), else the
      // previous ViT layer already wrote its output into S.x
      if (i == 0) K_TRY(launch_copy(x_img, saved + P.saved[i].x, (size_t)P.T_img * L.d_model * 2, s));
      void* dst = last ? y : (void*)(saved + P.saved[i + 1].x);
      K_TRY(launch_copy(x_seq, dst, (size_t)P.T_seq * L.d_out * 2, s));
      const char* xin = saved + P.saved[i].x;
      // token merging: the [T_img, d] rows read as [T_img / r, r d] rows (no data movement)
      const int64_t d_in = (int64_t)L.d_model * std::max(1, (int)L.merge);
      if (P.pool > 1) {   // average pooling at the end of the encoder
        K_TRY(launch_pool_rows(xin, saved + P.saved[i].n1, (const int32_t*)(ws + P.meta.pool_first),
                               (const int32_t*)(ws + P.meta.pool_count), P.T_con, L.d_model, s));
        xin = saved + P.saved[i].n1;
      }
      if (L.d_ff) {   // p = act(x.W1 + b1).W2 + b2
        char* pre = saved + P.saved[i].pre;
        char* act = saved + P.saved[i].act;
        K_TRY(linear_fwd(xin, prm[0], pre, P.T_con, d_in, L.d_ff, prm[1], nullptr, s));
        K_TRY(launch_act_fwd(L.act, pre, act, P.T_con, L.d_ff, s));
        K_TRY(linear_fwd(act, prm[2], ws + P.w_proj, P.T_con, L.d_ff, L.d_out, prm[3], nullptr, s));
      } else {
        K_TRY(linear_fwd(xin, prm[0], ws + P.w_proj, P.T_con, d_in, L.d_out, prm[1], nullptr, s));
      }
      K_TRY(launch_scatter_rows(ws + P.w_proj, dst, (const int32_t*)(ws + P.meta.i2s), P.T_con, L.d_out, 0, s));
      continue;
    }
    const bool vit = L.kind == MLLM_LAYER_VIT;
    const int64_t T = vit ? P.T_img : P.T_seq;
    if (i == 0) K_TRY(launch_copy(vit ? x_img : x_seq, saved + P.saved[i].x, (size_t)T * L.d_model * 2, s));
    void* out = last ? y : (void*)(saved + P.saved[i + 1].x);
    const float* rope_table = P.rope_of[i] >= 0 ? (const float*)(ws + P.rope_tables[P.rope_of[i]].off) : nullptr;
    if ((r = layer_fwd(L, prm, P.saved[i], saved, ws, P, T, out, rope_table, P.attn_of[i], s)) != MLLM_OK) return r;
  }
  return MLLM_OK;
}

mllm_status_t mllm_stage_bwd(mllm_stage_t* st, const mllm_batch_t* b, const void* const* params,
                             const void* dy, const void* saved_v, size_t saved_bytes, void* dx_img,
                             void* dx_seq, void* const* dparams, int accumulate, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  mllm_status_t r = check_batch(st, b);
  if (r != MLLM_OK) return r;
  Plan P = make_plan(st, b);
  if ((r = check_plan(P)) != MLLM_OK) return r;
  if ((r = check_io(st, b, params, P, saved_bytes, workspace_bytes, saved_v, workspace)) != MLLM_OK) return r;
  if (!dy) return fail(MLLM_ERR_NULL, "dy is NULL");
  if (!dparams) return fail(MLLM_ERR_NULL, "dparams is NULL");
  for (size_t i = 0; i < st->params.size(); i++)
    if (!dparams[i]) return fail(MLLM_ERR_NULL, "dparams[%zu] (%s) is NULL", i, st->params[i].name);
  hipStream_t s = (hipStream_t)hip_stream;
  const char* saved = (const char*)saved_v;
  char* ws = (char*)workspace;
  if ((r = upload_meta(st, b, P, workspace, s)) != MLLM_OK) return r;
  for (const Plan::RopeTable& t : P.rope_tables)
    K_TRY(launch_rope_table((float*)(ws + t.off), P.longest_seq, t.head_dim, t.base, s));

  const int n = (int)st->layers.size();
  const void* cur = dy;  // gradient w.r.t. the output of layer i
  char* pp[2] = {ws + P.w_g0, ws + P.w_g1};
  int flip = 0;
  bool colsum_done = false;   // the column sums of `cur` are already in the bias gradient they belong to
  for (int i = n - 1; i >= 0; i--) {
    const mllm_layer_desc_t& L = st->layers[i];
    const void* const* prm = params + st->param_off[i];
    void* const* dprm = dparams + st->param_off[i];
    if (L.kind == MLLM_LAYER_PROJECTOR) {
      const int32_t* i2s = (const int32_t*)(ws + P.meta.i2s);
      char* dproj = ws + P.w_proj;
      K_TRY(launch_scatter_rows(cur, dproj, i2s, P.T_con, L.d_out, 1, s));
      if (dx_seq) {
        K_TRY(launch_copy(cur, dx_seq, (size_t)P.T_seq * L.d_out * 2, s));
        K_TRY(launch_zero_rows(dx_seq, i2s, P.T_con, L.d_out, s));
      }
      const SplitWs split{ws + P.w_split, P.split_bytes};
      float* partial = (float*)(ws + P.w_partial);
      void* out = (i == 0 && dx_img) ? dx_img : (void*)pp[flip];
      const char* xin = P.pool > 1 ? saved + P.saved[i].n1 : saved + P.saved[i].x;
      const int64_t d_in = (int64_t)L.d_model * std::max(1, (int)L.merge);
      void* dxin = P.pool > 1 ? (void*)(ws + P.w_c) : out;   // gradient of the connector's input rows
      if (L.d_ff) {
        const char* pre = saved + P.saved[i].pre;
        const char* act = saved + P.saved[i].act;
        char* dh = ws + P.w_a;     // d act, then d pre in place   [T_con, d_ff]
        K_TRY(linear_dw(act, dproj, dprm[2], P.T_con, L.d_ff, L.d_out, accumulate, s, split));
        K_TRY(launch_colsum(dproj, L.d_out, (float*)dprm[3], accumulate, partial, P.T_con, L.d_out, s));
        K_TRY(linear_dx(dproj, prm[2], dh, P.T_con, L.d_ff, L.d_out, s));
        K_TRY(launch_gelu_bwd_colsum(L.act, dh, pre, dh, (float*)dprm[1], accumulate, partial, P.T_con, L.d_ff, s));
        K_TRY(linear_dw(xin, dh, dprm[0], P.T_con, d_in, L.d_ff, accumulate, s, split));
        K_TRY(linear_dx(dh, prm[0], dxin, P.T_con, d_in, L.d_ff, s));
      } else {
        K_TRY(linear_dw(xin, dproj, dprm[0], P.T_con, d_in, L.d_out, accumulate, s, split));
        K_TRY(launch_colsum(dproj, L.d_out, (float*)dprm[1], accumulate, partial, P.T_con, L.d_out, s));
        K_TRY(linear_dx(dproj, prm[0], dxin, P.T_con, d_in, L.d_out, s));
      }
      if (P.pool > 1)
        K_TRY(launch_unpool_rows(dxin, out, (const int32_t*)(ws + P.meta.row_window),
                                 (const int32_t*)(ws + P.meta.pool_count), P.T_img, L.d_model, s));
      cur = out;
      flip ^= 1;
      colsum_done = false;
      continue;
    }
    const bool vit = L.kind == MLLM_LAYER_VIT;
    const int64_t T = vit ? P.T_img : P.T_seq;
    void* out = pp[flip];
    if (i == 0) {
      void* want = vit ? dx_img : dx_seq;
      if (want) out = want;
    }
    const float* rope_table = P.rope_of[i] >= 0 ? (const float*)(ws + P.rope_tables[P.rope_of[i]].off) : nullptr;
    // An encoder layer's input gradient is the output gradient of the encoder layer below it, whose last
    // linear map has a bias (index 11 of its parameters): its gradient, the column sums of that tensor, is
    // formed while this layer's last norm writes the tensor.
    float* below = nullptr;
    if (vit && i > 0 && st->layers[i - 1].kind == MLLM_LAYER_VIT && st->layers[i - 1].d_model == L.d_model &&
        norm_bwd_colsum_fusable(L.d_model))
      below = (float*)(dparams + st->param_off[i - 1])[11];
    if ((r = layer_bwd(L, prm, dprm, accumulate, P.saved[i], saved, ws, P, T, cur, out, rope_table, P.attn_of[i], s,
                       colsum_done, below)) != MLLM_OK) return r;
    colsum_done = below != nullptr;
    cur = out;
    flip ^= 1;
  }
  return MLLM_OK;
}

}  // extern "C"
