// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mllm {

struct GemmArgs {
  const void* a;
  const void* b;
  void* c;
  int64_t m, n, k;
  int64_t lda, ldb, ldc;   // leading dimensions (elements) of the matrices as stored
  int a_layout;            // 0: A stored [M,K]; 1: A stored [K,M]
  int b_layout;            // 0: B stored [K,N]; 1: B stored [N,K]
  int out_fp32;            // 0: bf16 C; 1: fp32 C
  int accumulate;          // fp32 C only: C += product
  const void* bias;        // bf16 [N] or null
  const void* residual;    // bf16 [M,N] (ld = ldres) or null; bf16 C only
  int64_t ldres;
  void* splitk_ws;         // optional fp32 scratch for split-K partial products (null: never split)
  size_t splitk_ws_bytes;
  // SwiGLU fused into the product's epilogue: C = [gate | up] is [M, N] bf16 as usual and
  // swiglu_act [M, N/2] bf16 also receives silu(gate) * up.  Only where gemm_swiglu_fusable().
  void* swiglu_act = nullptr;
  // SwiGLU's gradient fused into the epilogue of dA = dY.W_d^T ([M, N], N = f): with
  // swiglu_pre = [gate | up] ([M, 2N] bf16) the product itself is not stored; swiglu_dpre
  // ([M, 2N] bf16) receives [d gate | d up].  C is unused.  Only where gemm_swiglu_bwd_fusable().
  const void* swiglu_pre = nullptr;
  void* swiglu_dpre = nullptr;
  // Rotary positions fused into the epilogue of a forward product Y = X.W (+ bias): the leading
  // rope_cols columns of Y are heads of rope_head_dim (64 or 128) whose half-split pairs are rotated,
  // on the fp32 accumulators, by the angles of row rope_pos[row] of rope_table (launch_rope_table).
  // Only where gemm_rope_fusable().
  const float* rope_table = nullptr;
  const int32_t* rope_pos = nullptr;   // device int32 [M]
  int64_t rope_cols = 0;
  int32_t rope_head_dim = 0;
};
// Whether launch_gemm can rotate the q and k columns of a forward product in its epilogue (large-tile
// kernel, K a multiple of 64, heads of 64 or 128 so that a wavefront's 128 columns hold whole heads).
bool gemm_rope_fusable(int64_t m, int64_t n, int64_t k, int32_t head_dim);
bool gemm_swiglu_bwd_fusable(int64_t m, int64_t n, int64_t k);
// Whether launch_gemm can write the SwiGLU activation of a forward product X[M,K].W[K,N] along
// with it (large-tile kernel, N/2 a multiple of 128, K a multiple of 64).
bool gemm_swiglu_fusable(int64_t m, int64_t n, int64_t k);
// A and B are addressed through 32-bit byte offsets: each operand must stay below this size.
constexpr int64_t GEMM_MAX_OPERAND_BYTES = 0xFFFFFFF0ll - 16;
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);
// Scratch bytes launch_gemm wants for an fp32-output product of this shape (0: it will not split).
size_t gemm_splitk_ws_bytes(int64_t m, int64_t n, int64_t k);
// out[i] (+)= sum over s of partial[s][i], s ascending.
hipError_t launch_splitk_reduce(const float* partial, float* out, int splits, int64_t n, int accumulate,
                                hipStream_t s);

// One workgroup of an attention kernel: a tile of a segment and a head (query head for the forward
// and dQ passes, kv head for the dK/dV pass).  The lists are built on the host (attn_items.h).
struct AttnItem {
  int32_t seg_start;  // first packed row of the segment
  int32_t seg_len;
  int32_t tile0;      // first row of the tile inside the segment
  int32_t causal;
  int32_t head;
};
struct AttnArgs {
  const void* q; const void* k; const void* v; void* o; float* lse;
  const void* d_o; void* dq; void* dk; void* dv; float* delta;
  int64_t q_stride, kv_stride, o_stride;   // row strides in elements (dq/dk/dv/do share them)
  int32_t total_tokens, n_q_heads, n_kv_heads, head_dim;
  const void* q_list; int32_t q_grid;      // device work list of the forward / dQ passes and its grid size
  const void* kv_list; int32_t kv_grid;    // device work list of the dK/dV pass and its grid size
  // backward only: when set (launch_rope_table, head_dim floats per position, positions counted from
  // the start of each segment), dq and dk leave rotated by the negative rotary angle of their row,
  // i.e. as gradients of the q and k that entered the rotation
  const float* rope_table;
  double fwd_flops;                               // algorithmic forward FLOPs of this call (for timing reports)
};
constexpr int ATTN_FWD_Q_TILE = 128;   // query rows per workgroup, forward and dQ pass
constexpr int ATTN_BWD_KV_TILE = 128;  // key rows per workgroup, dK/dV pass
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s);

// kind 0 LayerNorm, 1 RMSNorm.  stats: [2][T] fp32 (rstd, mean).  ld = elements between rows of
// every [t, d] operand (d for dense matrices; more when they are column slices of a wider one).
hipError_t launch_norm_fwd(int kind, const void* x, const void* gamma, const void* beta, void* y,
                           float* stats, int64_t t, int64_t d, int64_t ld, float eps, hipStream_t s);
int64_t norm_bwd_partial_rows(int64_t t);
hipError_t launch_norm_bwd(int kind, const void* dy, const void* x, const void* gamma,
                           const float* stats, const void* dres, void* dx, float* dgamma,
                           float* dbeta, int accumulate, float* partial, int64_t t, int64_t d,
                           int64_t ld, hipStream_t s, float* dx_colsum = nullptr);
// dx_colsum (optional, fp32 [d]): the column sums of dx, formed in the same pass; only for rows of at
// most 1024 elements (norm_bwd_colsum_fusable).  `partial` then holds three sets of sums.
bool norm_bwd_colsum_fusable(int64_t d);
hipError_t launch_rope(void* qk, const int32_t* pos, int64_t t, int64_t row_stride, int64_t col0,
                       int32_t n_heads, int32_t head_dim, float rope_base, int inverse,
                       hipStream_t s);
// table [n_pos, head_dim] fp32: cos then sin of pos * rope_base^(-2i/head_dim), i < head_dim / 2.
hipError_t launch_rope_table(float* table, int64_t n_pos, int32_t head_dim, float rope_base, hipStream_t s);
hipError_t launch_act_fwd(int act, const void* pre, void* a, int64_t t, int64_t f, hipStream_t s);
hipError_t launch_act_bwd(int act, const void* da, const void* pre, void* dpre, int64_t t,
                          int64_t f, hipStream_t s);
// GELU backward that also leaves the column sums of dpre (the gradient of the bias in front of the
// activation) in colsum [f] fp32 (accumulate != 0: +=).  partial: fp32 scratch of colsum_partial_rows(t) x f.
hipError_t launch_gelu_bwd_colsum(int act, const void* da, const void* pre, void* dpre, float* colsum,
                                  int accumulate, float* partial, int64_t t, int64_t f, hipStream_t s);
int64_t colsum_partial_rows(int64_t t);
hipError_t launch_colsum(const void* x, int64_t ldx, float* out, int accumulate, float* partial,
                         int64_t t, int64_t n, hipStream_t s);
// dst[rows[i], :] = src[i, :] (scatter) or dst[i, :] = src[rows[i], :] (gather); bf16 rows of d.
hipError_t launch_scatter_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows,
                               int64_t d, int gather, hipStream_t s);
// dst[j, :] = mean of src[first[j] .. first[j] + count[j]) (bf16 rows of d, fp32 sum).
hipError_t launch_pool_rows(const void* src, void* dst, const int32_t* first, const int32_t* count,
                            int64_t n_out, int64_t d, hipStream_t s);
// dst[i, :] = src[window[i], :] / count[window[i]]: the gradient of launch_pool_rows.
hipError_t launch_unpool_rows(const void* src, void* dst, const int32_t* window, const int32_t* count,
                              int64_t n_rows, int64_t d, hipStream_t s);
// Zero the rows named by rows[] of a bf16 [*, d] matrix.
hipError_t launch_zero_rows(void* dst, const int32_t* rows, int64_t n_rows, int64_t d,
                            hipStream_t s);
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

// Optional per-launch timing with HIP events on the launch stream (off by default).  Classes:
enum ProfClass { PROF_GEMM_FWD = 0, PROF_GEMM_DX = 1, PROF_GEMM_DW = 2, PROF_ATTN_FWD = 3,
                 PROF_ATTN_BWD = 4, PROF_ELEMENTWISE = 5, PROF_GEMM_SMALL = 6, PROF_GEMM_ROWS192 = 7,
                 PROF_N_CLASSES = 8 };
struct ProfScope {   // records a start event now and a stop event when it goes out of scope
  ProfScope(int cls, double work, hipStream_t s);
  ~ProfScope();
  int slot;
  hipStream_t stream;
};

}  // namespace mllm
