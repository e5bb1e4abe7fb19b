/*
 * mllm_stage.h -- C ABI of the MI355X (gfx950) pipeline-stage library.
 *
 * One call = the forward (or backward) pass of ONE pipeline stage's transformer layers over
 * ONE packed microbatch on ONE GPU: the unit of work that a 1F1B pipeline schedule repeats per
 * microbatch and per stage (Background and Motivation, Fig. 1).  A stage is a run of ViT encoder
 * layers over visual tokens, optionally a linear connector, optionally LLM decoder layers over
 * visual + text tokens (MLLM Architecture, Section 2.1; Fig. 1 caption).  The microbatch is a
 * set of items, each with a variable number of visual and text tokens (Table 1: E_seq_len,
 * L_seq_len; Data Profiler, Section 3.2), concatenated along the sequence dimension with batch
 * size 1 (Model Profiler, "Memory Profiling").  Attention handles every original instance
 * separately and causally; linear operations run over the whole concatenated sequence (Model
 * Profiler, "Throughput Profiling").
 *
 * General rules
 *   - Plain C99 types only.  "device" pointers are HIP device memory of the current device,
 *     "host" pointers are ordinary host memory.  All bf16 tensors are row-major, raw 16-bit
 *     patterns; matrices are stored [in, out] so that Y = X.W.
 *   - The caller owns every buffer and the stream.  The library owns only the opaque handle.
 *     mllm_stage_fwd / mllm_stage_bwd / mllm_op_* allocate nothing on the device.
 *   - Every call returns a status.  All argument validation happens before the first kernel is
 *     enqueued: on a status other than MLLM_OK and MLLM_ERR_HIP nothing was launched and no
 *     output was touched.  mllm_last_error() returns a thread-local message for the last failure.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and return without waiting.  Host arrays are consumed before the call returns: the small
 *     per-call metadata (attention tile lists, positions, scatter rows) are built in pinned host
 *     memory owned by the handle (mllm_op_attn_*: by the calling thread) and copied on
 *     `hip_stream` in front of the kernels.  That staging is a ring of 4 slots: a call waits only
 *     when the host runs 4 calls ahead of the GPU.  mllm_stage_sizes reserves the slots for the
 *     microbatch it is asked about; mllm_stage_fwd / mllm_stage_bwd allocate pinned host memory
 *     only for a microbatch whose metadata exceed every earlier reservation.
 *   - One handle must not be used from two threads at once.  Same inputs give bitwise-identical
 *     outputs (no atomics in any reduction).
 */
#ifndef MLLM_STAGE_H
#define MLLM_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mllm_stage mllm_stage_t; /* opaque, library-owned */

typedef enum {
  MLLM_OK = 0,
  MLLM_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  MLLM_ERR_DESC = 2,        /* inconsistent layer / stage descriptor                       */
  MLLM_ERR_SHAPE = 3,       /* sizes do not fit the descriptor or the kernels' limits      */
  MLLM_ERR_CU_SEQLENS = 4,  /* cu_seqlens not starting at 0, decreasing, or wrong total    */
  MLLM_ERR_MASK_KIND = 5,   /* mask kind outside {BIDIR, CAUSAL}                           */
  MLLM_ERR_INDEX = 6,       /* img_to_seq_row out of range or not strictly increasing      */
  MLLM_ERR_WORKSPACE = 7,   /* saved / workspace buffer smaller than mllm_stage_sizes says */
  MLLM_ERR_UNSUPPORTED = 8, /* valid request that this build does not implement            */
  MLLM_ERR_HIP = 9          /* a HIP call or kernel launch reported an error               */
} mllm_status_t;

enum { MLLM_MASK_BIDIR = 0, MLLM_MASK_CAUSAL = 1 };                       /* per segment */
enum { MLLM_LAYER_VIT = 0, MLLM_LAYER_DECODER = 1, MLLM_LAYER_PROJECTOR = 2 };
enum { MLLM_ACT_GELU_ERF = 0, MLLM_ACT_GELU_TANH = 1, MLLM_ACT_SWIGLU = 2 };

/*
 * One layer.  The paper names layers only by model family (Evaluation, Table 4), so the layer
 * arithmetic is the standard pre-norm transformer:
 *   VIT:       n = LayerNorm(x); [q|k|v] = n.W_qkv + b; o = attention (mask per segment);
 *              x1 = x + o.W_o + b_o; n2 = LayerNorm(x1); y = x1 + GELU(n2.W_1 + b_1).W_2 + b_2
 *   DECODER:   n = RMSNorm(x); [q|k|v] = n.W_qkv (+ b_qkv when has_bias = 1, the layout of the 7B
 *              LLM of the paper's Table 4); rotary positions on q, k (half-split pairs
 *              (i, i + head_dim/2), angle pos * rope_base^(-2i/head_dim), pos restarting at 0 in
 *              every segment); grouped-query attention (kv head = q head / (n_q/n_kv));
 *              x1 = x + o.W_o; n2 = RMSNorm(x1); y = x1 + (SiLU(n2.W_g) * n2.W_u).W_d
 *   PROJECTOR: p = x.W_p + b_p, or with a hidden width d_ff > 0 the two-layer perceptron
 *              p = GELU(x.W_p1 + b_p1).W_p2 + b_p2; row i of p is written to row img_to_seq_row[i]
 *              of the packed sequence (the learnable connector of Section 2.1, which names linear
 *              projectors and multi-layer perceptrons).  With pool = r > 1 the encoder rows are
 *              average-pooled first (Evaluation, audio modality: pooling at the end of the encoder
 *              reduces the tokens fed to the LLM): inside every img segment, consecutive windows of
 *              r rows are replaced by their mean, a shorter last window by the mean of what it
 *              holds; the connector then has sum over segments of ceil(length / r) rows, and
 *              img_to_seq_row has that many entries.  With merge = r > 1 the connector instead
 *              reads rows that concatenate r consecutive encoder rows (token merging of the
 *              pixel-shuffle kind, Data Profiler: connectors that shorten the modality sequence; the
 *              caller orders patches so that those to be merged are adjacent): every img segment
 *              length must be a multiple of r, the connector has total / r rows of width r * d_model
 *              and its first matrix is [r * d_model, .].
 *   qk_norm = 1 (VIT, DECODER): QK normalisation as in the InternViT encoders of the evaluated
 *              models (Evaluation, Table 4).  After the QKV projection the q row of a token (its
 *              n_q_heads * head_dim values, all heads together) is replaced by
 *              q * rsqrt(mean(q^2) + norm_eps) * qkn_q_g, and the k row (n_kv_heads * head_dim values)
 *              likewise with qkn_k_g; in a DECODER layer this comes before the rotary positions.
 * Parameter tensors per layer, in order (all bf16, matrices [in, out], vectors [n]):
 *   VIT:       ln1_g, ln1_b, w_qkv [d, 3d], b_qkv, w_o [d, d], b_o, ln2_g, ln2_b,
 *              w_1 [d, f], b_1, w_2 [f, d], b_2
 *   DECODER:   rms1_g, w_qkv [d, (n_q + 2 n_kv) hd], (b_qkv when has_bias = 1,) w_o [n_q hd, d],
 *              rms2_g, w_gu [d, 2f] = [W_gate | W_up], w_d [f, d]
 *   PROJECTOR: w_p [d_model, d_out], b_p; or w_p1 [d_model, d_ff], b_p1, w_p2 [d_ff, d_out], b_p2
 *   with qk_norm = 1 a VIT / DECODER layer's list ends with qkn_q_g [n_q hd], qkn_k_g [n_kv hd]
 * Limits: head_dim in {64, 128}; d_model == n_q_heads * head_dim for VIT / DECODER; every width
 * a multiple of 64; n_q_heads a multiple of n_kv_heads; act GELU_* for VIT and for a two-layer
 * PROJECTOR, SWIGLU for DECODER.
 * A microbatch is limited by tokens * widest layer width * 2 bytes < 4 GiB (MLLM_ERR_SHAPE beyond:
 * about 74 000 packed tokens for the 8B-shaped decoder layer).
 */
typedef struct {
  int32_t kind;       /* MLLM_LAYER_*                                   */
  int32_t d_model;    /* input width                                    */
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t d_ff;       /* MLP width f; PROJECTOR: hidden width, 0 = linear */
  int32_t d_out;      /* PROJECTOR only: output width                   */
  int32_t act;        /* MLLM_ACT_*                                     */
  int32_t has_bias;   /* 1 for VIT / PROJECTOR; DECODER: 0, or 1 = QKV bias */
  float norm_eps;
  float rope_base;    /* DECODER only                                   */
  int32_t pool;       /* PROJECTOR only: average this many consecutive encoder tokens of a segment
                         before the connector's map (0 or 1: none)  */
  int32_t merge;      /* PROJECTOR only: concatenate this many consecutive encoder tokens of a segment
                         into one connector row of width merge * d_model (0 or 1: none; not with pool) */
  int32_t qk_norm;    /* VIT / DECODER: 1 = RMS-normalise the q row and the k row of every token before
                         attention (0: none; PROJECTOR: must be 0) */
} mllm_layer_desc_t;

/* Layers in execution order: zero or more VIT, then at most one PROJECTOR, then zero or more
 * DECODER.  Widths of consecutive layers must chain. */
typedef struct {
  int32_t n_layers;
  const mllm_layer_desc_t* layers; /* host */
} mllm_stage_desc_t;

/* A packed token space: segment s covers rows cu_seqlens[s] .. cu_seqlens[s+1]-1.  Zero-length
 * segments are allowed.  max_seqlen must be >= the longest segment. */
typedef struct {
  int32_t total_tokens;
  int32_t n_segments;
  int32_t max_seqlen;
  const int32_t* cu_seqlens_host; /* host [n_segments + 1] */
  const uint8_t* mask_kind_host;  /* host [n_segments], MLLM_MASK_* */
} mllm_pack_t;

/* img: segments are images (used by VIT and PROJECTOR layers).  seq: segments are samples
 * (used by PROJECTOR and DECODER layers).  img_to_seq_row: host [img.total_tokens], the row of
 * the packed sequence that each projected image token lands on; strictly increasing. */
typedef struct {
  mllm_pack_t img;
  mllm_pack_t seq;
  const int32_t* img_to_seq_row_host;
} mllm_batch_t;

/* Create / destroy a stage handle.  The descriptor is copied. */
mllm_status_t mllm_stage_create(const mllm_stage_desc_t* desc, mllm_stage_t** out);
void mllm_stage_destroy(mllm_stage_t* stage);

/* Number of parameter tensors of the stage, and name / shape of tensor i (layer-major, in the
 * order listed above).  `name` points to static storage. */
size_t mllm_stage_param_count(const mllm_stage_t* stage);
mllm_status_t mllm_stage_param_info(const mllm_stage_t* stage, size_t i, const char** name,
                                    int32_t* layer, int64_t* rows, int64_t* cols);

/* Bytes of the `saved` buffer (activations kept from forward to backward) and of the scratch
 * `workspace` that fwd and bwd need for this microbatch. */
mllm_status_t mllm_stage_sizes(const mllm_stage_t* stage, const mllm_batch_t* batch,
                               size_t* saved_bytes, size_t* workspace_bytes);

/*
 * Forward pass of the stage.
 *   params   host array of mllm_stage_param_count() device pointers (bf16)
 *   x_img    device bf16 [img.total_tokens, d_model of the first layer]; required when the first
 *            layer is VIT or PROJECTOR, ignored otherwise
 *   x_seq    device bf16 [seq.total_tokens, d_llm]; required when the stage has a PROJECTOR or a
 *            DECODER layer.  With a PROJECTOR the rows named by img_to_seq_row are ignored and
 *            replaced by the projected image tokens; the buffer itself is not modified
 *   y        device bf16 output: [img.total_tokens, d] when the last layer is VIT, else
 *            [seq.total_tokens, d_llm]
 *   saved    device buffer (256-byte aligned) that mllm_stage_bwd reads back
 *   workspace device scratch (256-byte aligned); contents are undefined afterwards
 */
mllm_status_t mllm_stage_fwd(mllm_stage_t* stage, const mllm_batch_t* batch,
                             const void* const* params, const void* x_img, const void* x_seq,
                             void* y, void* saved, size_t saved_bytes, void* workspace,
                             size_t workspace_bytes, void* hip_stream);

/*
 * Backward pass for the microbatch that the preceding mllm_stage_fwd call with the same `saved`
 * buffer processed.
 *   dy       device bf16, same shape as y
 *   dx_img   device bf16 like x_img, or NULL if not wanted / not applicable
 *   dx_seq   device bf16 like x_seq, or NULL; rows named by img_to_seq_row are written as 0
 *   dparams  host array of device pointers, fp32, same shapes as params
 *   accumulate  0: dparams are overwritten; non-zero: dparams += gradient (microbatches of one
 *            optimizer step accumulate, cf. the N_mb microbatches of the Problem Formulation)
 */
mllm_status_t mllm_stage_bwd(mllm_stage_t* stage, const mllm_batch_t* batch,
                             const void* const* params, const void* dy, const void* saved,
                             size_t saved_bytes, void* dx_img, void* dx_seq, void* const* dparams,
                             int accumulate, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/* Thread-local description of the last error on this thread; never NULL, never freed. */
const char* mllm_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Single operations of the path, exported so that each kernel can be checked on its own.
 * They are the same kernels the stage calls.  All pointers are device pointers unless named
 * *_host.
 * ------------------------------------------------------------------------------------------ */

/* Dense contraction of the linear layers, which run over the whole packed sequence in one
 * call (Model Profiler, "Throughput Profiling"): C[M,N] = op(A).op(B) (+ bias) (+ residual).
 *   a_layout 0: A stored [M,K] row-major; 1: A stored [K,M] row-major (contraction over rows)
 *   b_layout 0: B stored [K,N] row-major; 1: B stored [N,K] row-major
 *   out_fp32 0: C is bf16 [M,N]; 1: C is fp32 [M,N]; accumulate != 0 (fp32 only): C += product
 *   bias bf16 [N] or NULL; residual bf16 [M,N] or NULL (bf16 output only)
 * Contiguous dimensions must be multiples of 8. */
mllm_status_t mllm_op_gemm(const void* a, const void* b, void* c, int64_t m, int64_t n, int64_t k,
                           int a_layout, int b_layout, int out_fp32, int accumulate,
                           const void* bias, const void* residual, void* hip_stream);

/* The decoder's MLP up-projection with its activation in one pass (the linear operations of the
 * LLM run over the whole packed sequence: Model Profiler, "Throughput Profiling"):
 * pre [M, 2f] = x [M, K] . w_gu [K, 2f] with w_gu = [W_gate | W_up], and
 * act [M, f] = silu(pre[:, :f]) * pre[:, f:], all bf16 row-major, act computed from the fp32
 * accumulators.  The stage takes this form whenever it applies: f a multiple of 128, K a multiple
 * of 64, at least 200 output tiles of 256 x 256; otherwise MLLM_ERR_UNSUPPORTED (then
 * mllm_op_gemm followed by mllm_op_act_fwd computes the same). */
mllm_status_t mllm_op_gemm_swiglu(const void* x, const void* w_gu, void* pre, void* act, int64_t m,
                                  int64_t f, int64_t k, void* hip_stream);

/* The backward counterpart: with dy [M, K] (gradient of the MLP output), w_d [f, K] (the
 * down-projection, stored [in, out]) and pre [M, 2f] = [gate | up], writes
 * dpre [M, 2f] = [d gate | d up], where dA = dy . w_d^T [M, f] is kept in fp32 and never stored:
 * d gate = dA * up * s * (1 + gate * (1 - s)), d up = dA * gate * s, s = sigmoid(gate).
 * All bf16 row-major.  Applies with K a multiple of 64 and at least 200 tiles of 256 x 256 in
 * [M, f]; otherwise MLLM_ERR_UNSUPPORTED (mllm_op_gemm followed by mllm_op_act_bwd computes the same). */
mllm_status_t mllm_op_gemm_swiglu_bwd(const void* dy, const void* w_d, const void* pre, void* dpre,
                                      int64_t m, int64_t f, int64_t k, void* hip_stream);

/* Per-instance attention over a packed sequence (Model Profiler, "Throughput Profiling").
 *   q [T, n_q, hd], k, v [T, n_kv, hd] bf16 with row strides (in elements) q_stride / kv_stride,
 *   o [T, n_q, hd] bf16 (row stride o_stride), lse fp32 [n_q, T] (natural log-sum-exp of the
 *   scaled scores), scale = 1/sqrt(hd) applied inside.
 *   workspace: device scratch of at least mllm_op_attn_workspace_bytes(n_segments, T, n_q_heads)
 *   bytes (it receives the kernels' work lists: one item per (segment, tile, head)). */
size_t mllm_op_attn_workspace_bytes(int32_t n_segments, int32_t total_tokens, int32_t n_q_heads);
mllm_status_t mllm_op_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                               const mllm_pack_t* pack, int32_t n_q_heads, int32_t n_kv_heads,
                               int32_t head_dim, int64_t q_stride, int64_t kv_stride,
                               int64_t o_stride, void* workspace, size_t workspace_bytes,
                               void* hip_stream);
/* The order in which the attention kernels visit a packed token space (host only, no GPU work;
 * exported so that the order can be checked).  One work item = one workgroup = (segment, tile of
 * 128 rows, head): query tiles x query heads for the forward and dQ passes (kv_major = 0), key tiles
 * x kv heads for the dK/dV pass (kv_major != 0).  Forward / dQ: items that read the same K / V rows
 * (the tiles and query heads of one (segment, kv head), in runs of about one XCD's resident
 * workgroups) are kept together on one XCD; the runs go to the eight XCDs heaviest first, each to the
 * least loaded one, and workgroup pid of the launch takes item number pid / 8 of XCD pid % 8.  dK/dV:
 * one list, heaviest key tile first, the kv heads of a tile adjacent.
 * out_host (may be NULL to query the size) receives *grid_out entries of 5 int32 words: seg_start,
 * seg_len, tile0, causal, head; entry pid is workgroup pid's item; seg_len = 0 marks the empty entries
 * that pad the shorter XCD lists.  *bytes_needed = an upper bound of the bytes written (the size to
 * allocate); *grid_out = workgroups launched = 8 * the longest XCD list. */
mllm_status_t mllm_attn_work_list(const mllm_pack_t* pack, int32_t kv_major, int32_t n_q_heads,
                                  int32_t n_kv_heads, int32_t head_dim, void* out_host,
                                  size_t out_bytes, size_t* bytes_needed, int32_t* grid_out);

/* Backward of the above from (q, k, v, o, lse, do): dq, dk, dv bf16 with the strides of q / k / v.
 * delta: fp32 scratch [n_q, T] (rowsum(dO * O)), overwritten. */
mllm_status_t mllm_op_attn_bwd(const void* q, const void* k, const void* v, const void* o,
                               const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                               float* delta, const mllm_pack_t* pack, int32_t n_q_heads,
                               int32_t n_kv_heads, int32_t head_dim, int64_t q_stride,
                               int64_t kv_stride, int64_t o_stride, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/* The same with the gradient of the rotary positions folded into the write-out: dq and dk leave
 * rotated by the negative angle of their row's position inside its segment, i.e. they are the
 * gradients of the q and k that entered the rotation (what mllm_op_attn_bwd followed by
 * mllm_op_rope with inverse != 0 computes, with one rounding instead of two).  rope_table: device
 * fp32 [positions, head_dim] from mllm_op_rope_table, at least max_seqlen positions; NULL: no
 * rotation (identical to mllm_op_attn_bwd). */
mllm_status_t mllm_op_attn_bwd_rope(const void* q, const void* k, const void* v, const void* o,
                                    const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                                    float* delta, const mllm_pack_t* pack, int32_t n_q_heads,
                                    int32_t n_kv_heads, int32_t head_dim, int64_t q_stride,
                                    int64_t kv_stride, int64_t o_stride, const float* rope_table,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Row normalisation.  kind 0: LayerNorm (gamma, beta), 1: RMSNorm (gamma).  x, y bf16 [T, d];
 * stats fp32 [2, T]: row 0 = 1/sqrt(var+eps) (or 1/sqrt(mean sq+eps)), row 1 = mean (LayerNorm). */
mllm_status_t mllm_op_norm_fwd(int kind, const void* x, const void* gamma, const void* beta,
                               void* y, float* stats, int64_t t, int64_t d, float eps,
                               void* hip_stream);
/* dx = norm backward of dy (bf16), plus `dres` (bf16 [T,d] or NULL) added to it; dgamma / dbeta
 * fp32 [d] (accumulate != 0: +=).  partial: fp32 scratch of mllm_op_norm_bwd_partial_bytes. */
size_t mllm_op_norm_bwd_partial_bytes(int64_t t, int64_t d);
mllm_status_t mllm_op_norm_bwd(int kind, const void* dy, const void* x, const void* gamma,
                               const float* stats, const void* dres, void* dx, float* dgamma,
                               float* dbeta, int accumulate, float* partial, int64_t t, int64_t d,
                               void* hip_stream);
/* The same, and the column sums of dx (fp32 [d], accumulate != 0: +=), taken from the values of dx
 * before they are rounded to bf16, in the same pass.  dx is the output gradient of the linear map in
 * front of the residual stream (an encoder layer's output projection, or the second MLP matrix of the
 * encoder layer below), so these sums are that map's bias gradient (Model Profiler, "Throughput
 * Profiling": the encoder's linear operations).  Only for d <= 1024 (MLLM_ERR_SHAPE beyond). */
mllm_status_t mllm_op_norm_bwd_colsum(int kind, const void* dy, const void* x, const void* gamma,
                                      const float* stats, const void* dres, void* dx, float* dgamma,
                                      float* dbeta, float* dx_colsum, int accumulate, float* partial,
                                      int64_t t, int64_t d, void* hip_stream);

/* Rotary positions applied in place to the q and k column blocks of a packed [T, row_stride]
 * bf16 buffer (n_heads heads of head_dim starting at column col0).  pos: device int32 [T];
 * inverse != 0 rotates by the negative angle (the backward pass). */
mllm_status_t mllm_op_rope(void* qk, const int32_t* pos, int64_t t, int64_t row_stride,
                           int64_t col0, int32_t n_heads, int32_t head_dim, float rope_base,
                           int inverse, void* hip_stream);

/* Table of rotary factors for the kernels that rotate inside another operation: row p (p <
 * n_pos) holds cos(p * rope_base^(-2i/head_dim)) for i < head_dim/2, then the sines; device fp32
 * [n_pos, head_dim].  Angles and their sines are formed in fp64. */
mllm_status_t mllm_op_rope_table(float* table, int64_t n_pos, int32_t head_dim, float rope_base,
                                 void* hip_stream);

/* The decoder's QKV projection with the rotary positions in its epilogue (the stage takes this
 * form whenever it applies): y [M, N] = x [M, K] . w [K, N] (+ bias [N]), all bf16 row-major; the
 * leading rope_cols columns of y (a multiple of 128) are heads of head_dim (64 or 128) whose
 * half-split pairs (i, i + head_dim/2) are rotated, on the fp32 accumulators and after the bias, by
 * the angles of row pos[row] of rope_table (pos: device int32 [M], every entry below the table's
 * n_pos).  Applies with K a multiple of 64 and at least 200 output tiles of 256 x 256; otherwise
 * MLLM_ERR_UNSUPPORTED (mllm_op_gemm followed by mllm_op_rope computes the same with one more
 * rounding). */
mllm_status_t mllm_op_gemm_rope(const void* x, const void* w, const void* bias, void* y, int64_t m,
                                int64_t n, int64_t k, const int32_t* pos, const float* rope_table,
                                int64_t rope_cols, int32_t head_dim, void* hip_stream);

/* Activations.  act GELU_*: a = GELU(h), h [T, f].  act SWIGLU: a = SiLU(g) * u with
 * gu = [g | u] of shape [T, 2f].  Backward writes dh [T, f] or dgu [T, 2f] from da and the
 * saved pre-activation. */
mllm_status_t mllm_op_act_fwd(int act, const void* pre, void* a, int64_t t, int64_t f,
                              void* hip_stream);
mllm_status_t mllm_op_act_bwd(int act, const void* da, const void* pre, void* dpre, int64_t t,
                              int64_t f, void* hip_stream);

/* Column sums of a bf16 [T, n] matrix into fp32 [n] (bias gradients); accumulate != 0: +=.
 * partial: fp32 scratch of mllm_op_colsum_partial_bytes(t, n). */
size_t mllm_op_colsum_partial_bytes(int64_t t, int64_t n);
mllm_status_t mllm_op_colsum(const void* x, float* out, int accumulate, float* partial, int64_t t,
                             int64_t n, void* hip_stream);

/* mllm_op_colsum for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * result bit for bit; the partial sums live in a static device array of the library
 * (mllm_op_colsum_static_max_bytes() = 8 MiB per GPU, held until the process ends) instead of a
 * `partial` argument.  The call allocates nothing (the array's device address is looked up once
 * per device, on the first call there).  MLLM_ERR_WORKSPACE when
 * mllm_op_colsum_partial_bytes(t, n) exceeds the array (n <= 4096 always fits).  All calls on one
 * GPU share the array: calls that overlap on one GPU (different streams) race; calls on one
 * stream are ordered and safe. */
size_t mllm_op_colsum_static_max_bytes(void);
mllm_status_t mllm_op_colsum_static(const void* x, float* out, int accumulate, int64_t t, int64_t n,
                                    void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Online microbatch scheduler (host only, no GPU work; Online Microbatch Scheduler, "Problem
 * Formulation" and "Scheduling Optimization").  Item i of a global batch has an encoder-stage
 * duration e_dur[i] and an LLM-stage duration l_dur[i] (host arrays, non-negative).  The items are
 * assigned to n_buckets buckets, bucket_out[i] in [0, n_buckets) (host array, caller-owned), to
 * make C_max = max over buckets of max(sum of e_dur, sum of l_dur) small.
 *   mllm_schedule_lpt: longest-processing-time-first -- items by descending max(e, l), each into
 *     the bucket with the lowest max(E_j, L_j); ties to the lower index.
 *   mllm_schedule: exact branch-and-bound search started from the LPT solution and limited to
 *     node_limit search nodes (the deterministic stand-in for the solver's time limit); when the
 *     limit is hit, *optimal_out = 0 and the best assignment found (never worse than LPT) is
 *     returned.  *cmax_out receives the objective of the returned assignment.
 * ------------------------------------------------------------------------------------------ */
mllm_status_t mllm_schedule_lpt(int64_t n_items, const double* e_dur, const double* l_dur,
                                int32_t n_buckets, int32_t* bucket_out);
mllm_status_t mllm_schedule(int64_t n_items, const double* e_dur, const double* l_dur,
                            int32_t n_buckets, int64_t node_limit, int32_t* bucket_out,
                            double* cmax_out, int32_t* optimal_out);

/* ------------------------------------------------------------------------------------------
 * Profiled performance model and parallelism search (host only, no GPU work).
 *
 * Model Profiler, "Throughput Profiling" / "Memory Profiling": throughput and memory are measured
 * on a grid of input sizes and TP degrees and read off in between by linear interpolation.
 *
 * mllm_interp: out[j] = the piecewise-linear function through (x[k], y[k]), k < n (x strictly
 *   ascending, n >= 1), at q[j], j < nq.  Outside [x[0], x[n-1]]: the end value when
 *   extrapolate == 0 (used for throughput), the end segment's straight line otherwise (used for
 *   memory).  All arrays are host memory, caller-owned.
 *
 * mllm_item_durations (Data-aware 3D Parallelism Optimizer, "Problem Formulation"; Online
 *   Microbatch Scheduler, "Scheduling Optimization"): duration = load / throughput at the item's
 *   own shape.  Item i has an effective batch size b[i] (its images), an LLM sequence length s[i],
 *   encoder FLOPs e_flop[i], LLM linear-layer FLOPs l_lin_flop[i] and LLM attention FLOPs
 *   l_attn_flop[i].  e_dur_out[i] = e_flop[i] / E_thr(b[i]); l_dur_out[i] = l_lin_flop[i] /
 *   L_lin_thr(s[i]) + l_attn_flop[i] / L_attn_thr(s[i]); a zero load costs zero time.  Each
 *   throughput curve is a grid (n, x, y) as in mllm_interp with extrapolate == 0, y > 0.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n;          /* grid points, >= 1                          */
  const double* x;    /* [n] host, strictly ascending               */
  const double* y;    /* [n] host                                   */
} mllm_curve_t;

mllm_status_t mllm_interp(const mllm_curve_t* curve, int64_t nq, const double* q, int32_t extrapolate,
                          double* out);
mllm_status_t mllm_item_durations(int64_t n_items, const double* b, const double* s,
                                  const double* e_flop, const double* l_lin_flop,
                                  const double* l_attn_flop, const mllm_curve_t* e_thr,
                                  const mllm_curve_t* l_lin_thr, const mllm_curve_t* l_attn_thr,
                                  double* e_dur_out, double* l_dur_out);

/* What the Model Profiler and the Data Profiler hand to the parallelism search for one module
 * (modality encoder or LLM).  x is the module's input dimension: effective batch size for the
 * encoder, packed sequence length for the LLM.  A TP degree between two profiled ones interpolates
 * linearly between their curves; memory is a straight line in the layer count through the two
 * profiled layer counts.  All pointers are host memory. */
typedef struct {
  int32_t n_tp;               /* profiled TP degrees                                        */
  const int32_t* tp;          /* [n_tp] strictly ascending                                  */
  int32_t n_x;                /* grid points of the input dimension                         */
  const double* x;            /* [n_x] strictly ascending                                   */
  const double* thr;          /* [n_tp][n_x] FLOP/s per GPU, > 0                            */
  double layers_lo, layers_hi;/* the two profiled layer counts, lo < hi                     */
  const double* model_state;  /* [n_tp][2] bytes: parameters, gradients, optimizer states   */
  const double* act_state;    /* [n_tp][2][n_x] bytes of activations kept for backward      */
  int32_t n_layers;           /* E_l or L_l: layers of the module to be trained             */
  double flop_per_item;       /* data-set average FLOPs of one item through the whole module */
} mllm_module_profile_t;

/* Algorithm 1, Phase 1 helper: all (tp, pp, dp) with tp * pp * dp == gpus, tp <= n_gpu_node
 * (Eq. 2), pp <= max_pp, ordered by tp then pp.  Writes up to capacity triples to triples_out
 * (host, [capacity][3], may be NULL when capacity == 0) and the full count to *count_out. */
mllm_status_t mllm_find_combs(int32_t gpus, int32_t n_gpu_node, int32_t max_pp, int64_t capacity,
                              int32_t* triples_out, int64_t* count_out);

/* Eq. 1 with the stage durations of Algorithm 1 for ONE configuration theta = (E_tp, E_pp, E_dp,
 * L_tp, L_pp, L_dp, N_mb): *makespan_out = (N_mb + E_pp + L_pp - 1) * max(E_dur, L_dur);
 * *e_mem_out / *l_mem_out = Eq. 4 / Eq. 5 at the mean microbatch shape; *feasible_out = both
 * fit in m_gpu.  Any of the four outputs may be NULL. */
mllm_status_t mllm_evaluate_parallelism(const mllm_module_profile_t* enc, const mllm_module_profile_t* llm,
                                        const int32_t theta[7], double m_gpu, int32_t gbs,
                                        double mean_bsz, double mean_seq_len, double* makespan_out,
                                        double* e_mem_out, double* l_mem_out, int32_t* feasible_out);

/* Algorithm 1: the configuration with the smallest estimated makespan among all splits of n_gpus
 * between the two modules (Eq. 3), all (tp, pp, dp) of each side and all microbatch counts
 * 1 .. gbs / L_dp that fit in m_gpu bytes per GPU (Eq. 4, 5).  Enumeration order: encoder GPUs,
 * encoder (tp, pp), LLM (tp, pp), microbatch count, all ascending; only a strictly smaller makespan
 * replaces the incumbent.  *found_out = 0 (theta_out zeroed, *min_t_out = +inf) when nothing fits. */
mllm_status_t mllm_optimize_parallelism(const mllm_module_profile_t* enc, const mllm_module_profile_t* llm,
                                        int32_t n_gpus, int32_t n_gpu_node, double m_gpu, int32_t gbs,
                                        double mean_bsz, double mean_seq_len, int32_t theta_out[7],
                                        double* min_t_out, int32_t* found_out);

/* ------------------------------------------------------------------------------------------
 * Per-launch timing, for measurement only (off by default; adds two event records per launch).
 * mllm_profile_begin(max_records) creates the events and starts recording every kernel launch of
 * the calling process' later mllm_* calls, bracketing each with HIP events on its launch stream.
 * mllm_profile_end stops recording, waits for the recorded events, and sums per class
 * (0 / 1 / 2: the 256x256-tile GEMM kernel in its Y=X.W / dX / dW layouts, 3 attention forward,
 * 4 attention backward, 5 the norm / rotary / activation / reduction / copy kernels, 6 the
 * 128x128-tile GEMM kernel in any layout, 7 the 192x256-tile form of the large GEMM kernel in any
 * layout): launches[8], milliseconds[8] and work[8] (algorithmic FLOPs for the GEMM and attention
 * classes, algorithmic bytes for class 5) are host arrays.
 * Not thread-safe; records beyond max_records are dropped and counted in *dropped.
 * ------------------------------------------------------------------------------------------ */
mllm_status_t mllm_profile_begin(int32_t max_records);
mllm_status_t mllm_profile_end(int64_t* launches, double* milliseconds, double* work,
                               int64_t* dropped);

#ifdef __cplusplus
}
#endif
#endif /* MLLM_STAGE_H */
