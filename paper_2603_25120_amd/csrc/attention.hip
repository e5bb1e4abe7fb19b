// Varlen block-diagonal flash attention for gfx950, forward and backward.
//
// Attention depends on the length of every single sample and has to treat each packed sample
// on its own so that no sample sees another (Model Profiler, "Throughput Profiling"): a packed
// [T, heads, hd] sequence is cut into segments by cu_seqlens; each segment
// attends only to itself, bidirectionally (an image inside the ViT) or causally (a sample inside
// the LLM).  The host turns the segments into lists of (segment, tile, head) work items, one list
// per XCD, in which workgroups that share rows sit together (attn_items.h).
//
// All three kernels compute score blocks TRANSPOSED so that a lane owns one query (or one key)
// column of the 32x32 MFMA result: row statistics are then per-lane scalars plus one exchange
// between the two half-wavefronts, and the probability block can be fed straight back as the
// B operand of the next MFMA without leaving registers (the contraction-slot order of that
// operand is a fixed permutation of the key/query rows, applied identically to the A operand,
// which is fetched from LDS with the transposing read).
//
//   forward:  S^T = K.Q^T, online softmax, O^T += V^T.P^T
//   dQ pass:  delta = rowsum(dO*O); S^T, dP^T = V.dO^T, dS^T = P^T*(dP^T - delta), dQ^T += K^T.dS^T
//   dK/dV:    S = Q.K^T, dP = dO.V^T, dV^T += dO^T.P, dK^T += Q^T.dS, looping the query tiles
//             and the query heads of the GQA group, so dK/dV need no atomics.
#include <algorithm>
#include <utility>

#include "common.h"
#include "kernels.h"

namespace mllm {

namespace {

#define MLLM_LDS_VOID(ptr) ((MLLM_LDS void*)(ptr))
constexpr int WAIT_VMCNT_0 = (0x7 << 4) | (0xF << 8);
constexpr int BKV = 64;   // key rows staged per step (forward, dQ)
constexpr int BQ = 64;    // query rows staged per step (dK/dV)

// LDS tiles are [rows][HD] bf16 without padding; 16-byte chunk c of row r lives at chunk position
// c ^ swz<HD>(r).  LDS serves 256 B per clock: a 16-byte read is processed 16 lanes at a time (16
// consecutive rows, same logical chunk) and a transposing 8-byte read 32 lanes at a time (4
// consecutive rows x 64 B).  The permutations below make both patterns conflict-free on the same
// tile: HD = 128 (256-byte rows) maps the 16 rows to 16 different chunks and the 4 rows of a
// transposing read to the 4 quarters of the row; HD = 64 (128-byte rows, two rows per 256-byte
// window) does the same over row pairs.
template <int HD>
__device__ __forceinline__ int swz(int r) {
  if constexpr (HD == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  else { const int t = (r >> 1) & 7; return ((t & 1) << 2) | (t >> 1); }
}
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// Descriptor over rows [0, rows) of a row-major bf16 matrix slice of `width` columns.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_rsrc(const bf16_t* base, int64_t stride, int rows, int width) {
  const uint32_t bytes = rows > 0 ? (uint32_t)(((int64_t)(rows - 1) * stride + width) * 2) : 0u;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, (int)bytes, 0x00020000);
}
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// v_exp_f32: flushes tiny results to zero, which is what a masked or negligible probability wants.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct AttnParams {
  const bf16_t* q; const bf16_t* k; const bf16_t* v; bf16_t* o; float* lse;
  const bf16_t* d_o; bf16_t* dq; bf16_t* dk; bf16_t* dv; float* delta;
  int64_t q_stride, kv_stride, o_stride;
  int32_t T, Hq, Hkv;
  const AttnItem* list;      // work list, one entry per workgroup
  float scale_log2e, scale;
  const float* rope_table;   // backward: dq, dk are rotated back by the rotary angle of their row (null: not)
};

// Gradient of the rotary positions on an accumulator of ND = HD/32 blocks whose lane owns row `pos`
// of its segment: the pair (c, c + HD/2) sits in blocks (d, d + ND/2) of the same lane.  Forward was
// y1 = x1 cos - x2 sin, y2 = x2 cos + x1 sin, so dx1 = dy1 cos + dy2 sin, dx2 = dy2 cos - dy1 sin.
// `scale` multiplies the result.
template <int HD>
__device__ __forceinline__ void rope_unrotate(f32x16 (&acc)[HD / 32], const float* table, int pos, int h, float scale) {
  constexpr int ND = HD / 32, HALF = HD / 2;
  const float* trow = table + (int64_t)pos * HD;
#pragma unroll
  for (int d = 0; d < ND / 2; d++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      const int f0 = 32 * d + 8 * g4 + 4 * h;
      const float4 c = *reinterpret_cast<const float4*>(trow + f0);
      const float4 sn = *reinterpret_cast<const float4*>(trow + HALF + f0);
      const float cs[4] = {c.x * scale, c.y * scale, c.z * scale, c.w * scale};
      const float ss[4] = {sn.x * scale, sn.y * scale, sn.z * scale, sn.w * scale};
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const float y1 = acc[d][4 * g4 + e], y2 = acc[d + ND / 2][4 * g4 + e];
        acc[d][4 * g4 + e] = y1 * cs[e] + y2 * ss[e];
        acc[d + ND / 2][4 * g4 + e] = y2 * cs[e] - y1 * ss[e];
      }
    }
}

// The work item of this workgroup (entry blockIdx.x of the list; the host has arranged the entries so
// that workgroups sharing rows run on one XCD).  Returns false, for the whole workgroup, on the empty
// items that pad the shorter XCD lists.
__device__ __forceinline__ bool work_item(const AttnItem* list, AttnItem& t) {
  const AttnItem x = list[blockIdx.x];
  // the same for every lane: keep the fields in scalar registers
  t.seg_start = __builtin_amdgcn_readfirstlane(x.seg_start);
  t.seg_len = __builtin_amdgcn_readfirstlane(x.seg_len);
  t.tile0 = __builtin_amdgcn_readfirstlane(x.tile0);
  t.causal = __builtin_amdgcn_readfirstlane(x.causal);
  t.head = __builtin_amdgcn_readfirstlane(x.head);
  return t.seg_len > 0;
}

// Natural-layout operand: row (r0 + lane%32), contraction values 16c + 8*(lane/32) .. +7.
template <int HD>
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* tile, int r0, int c, int lane) {
  Frag8 f;
  const int r = r0 + (lane & 31);
  f.u = *reinterpret_cast<const uint4*>(tile + r * HD + 8 * ((2 * c + (lane >> 5)) ^ swz<HD>(r)));
  return f.v;
}
// Transposed operand for the register-resident B operand built from a 32x32 accumulator:
// output row (n0 + lane%32) of the tile's columns, contraction slots e = 0..7 standing for tile
// rows k16 + 8*(e/4) + 4*(lane/32) + e%4.  Each transposing read returns tile[k0 + e][n] for
// e = 0..3 when lane i of a 16-lane group addresses tile[k0 + i/4][n0' + 4*(i%4)].
template <int HD>
__device__ __forceinline__ bf16x8 frag_cols_permuted(const bf16_t* tile, int k16, int n0, int lane) {
  Frag8 f;
  const int h = lane >> 5, i16 = lane & 15;
  const int n = n0 + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
  const int k = k16 + 4 * h + (i16 >> 2);
  const bf16_t* p0 = tile + k * HD + 8 * ((n >> 3) ^ swz<HD>(k)) + (n & 7);
  const bf16_t* p1 = tile + (k + 8) * HD + 8 * ((n >> 3) ^ swz<HD>(k + 8)) + (n & 7);
  f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)p0);
  f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)p1);
  return f.v;
}
// Accumulator values 8*cc .. 8*cc+7 of a 32x32 block as a bf16 B operand.
__device__ __forceinline__ bf16x8 acc_to_frag(const f32x16& a, int cc) {
  Frag8 f;
#pragma unroll
  for (int e = 0; e < 4; e++) f.w[e] = pack_bf16x2(a[8 * cc + 2 * e], a[8 * cc + 2 * e + 1]);
  return f.v;
}
__device__ __forceinline__ bf16x8 global_frag(const bf16_t* p, bool ok) {
  Frag8 f;
  f.u = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
  return f.v;
}
// Row index inside a 32x32 accumulator block held at position v by a lane of half h.
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// Scheduling patterns (one call per slot): an MFMA followed by N LDS reads; four LDS reads
// followed by a pair of MFMAs.
template <int N, int... Is>
__device__ __forceinline__ void reads_behind_mfmas(std::integer_sequence<int, Is...>) {
  ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0), __builtin_amdgcn_sched_group_barrier(0x100, N, 0), (void)Is), ...);
}
// An MFMA followed by one LDS read and one load from memory.
template <int... Is>
__device__ __forceinline__ void reads_and_loads_behind_mfmas(std::integer_sequence<int, Is...>) {
  ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0), __builtin_amdgcn_sched_group_barrier(0x100, 1, 0),
    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0), (void)Is), ...);
}
// N LDS reads followed by one MFMA.
template <int N, int... Is>
__device__ __forceinline__ void reads_before_mfmas(std::integer_sequence<int, Is...>) {
  ((__builtin_amdgcn_sched_group_barrier(0x100, N, 0), __builtin_amdgcn_sched_group_barrier(0x008, 1, 0), (void)Is), ...);
}
template <int... Is>
__device__ __forceinline__ void reads_before_mfma_pairs(std::integer_sequence<int, Is...>) {
  ((__builtin_amdgcn_sched_group_barrier(0x100, 4, 0), __builtin_amdgcn_sched_group_barrier(0x008, 2, 0), (void)Is), ...);
}

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(AttnParams p) {
  constexpr int NC = HD / 16, ND = HD / 32, NB = BKV / 32, TILE = BKV * HD;
  // K and V tiles go from global memory straight into LDS (`buffer_load ... lds`), two stages
  // each in arrays of their own so that every access names its stage statically.
  __shared__ __attribute__((aligned(1024))) bf16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vs0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vs1[TILE];
  AttnItem t;
  if (!work_item(p.list, t)) return;
  const int head = t.head, kvh = head / (p.Hq / p.Hkv);
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qrow = t.tile0 + 32 * wave + (lane & 31);
  const bool qok = qrow < t.seg_len;
  const bf16_t* qp = p.q + (int64_t)(t.seg_start + qrow) * p.q_stride + head * HD + 8 * h;
  bf16x8 qf[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) qf[c] = global_frag(qp + 16 * c, qok);

  const bf16_t* kbase = p.k + (int64_t)t.seg_start * p.kv_stride + kvh * HD;
  const bf16_t* vbase = p.v + (int64_t)t.seg_start * p.kv_stride + kvh * HD;
  const int kv_end = t.causal ? min(t.seg_len, t.tile0 + ATTN_FWD_Q_TILE) : t.seg_len;
  const int wave_first_q = t.tile0 + 32 * wave, wave_last_q = wave_first_q + 31;

  f32x16 oacc[ND];
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int v = 0; v < 16; v++) oacc[d][v] = 0.f;
  // Running maximum in units of log2: m = max(score) * scale * log2(e); l = sum of exp2(...).
  float m = -INFINITY, l = 0.f;
  const float c2 = p.scale_log2e;

  // One direct-to-LDS instruction moves 64 lanes x 16 bytes = RPI rows of the tile; lane l's
  // chunk lands at position l of that 1 KiB, so the lane fetches the global chunk that the
  // permutation puts there.  Rows past kv_end are outside the descriptor: zeros, no traffic.
  const __amdgpu_buffer_rsrc_t rk = rows_rsrc(kbase, p.kv_stride, kv_end, HD), rv = rows_rsrc(vbase, p.kv_stride, kv_end, HD);
  constexpr int CPR = HD / 8, RPI = 64 / CPR, PER_WAVE = BKV / RPI / 4;
  uint32_t kv_off[PER_WAVE];
#pragma unroll
  for (int i = 0; i < PER_WAVE; i++) {
    const int r = (wave * PER_WAVE + i) * RPI + lane / CPR, c = (lane % CPR) ^ swz<HD>(r);
    kv_off[i] = (uint32_t)((r * p.kv_stride + 8 * c) * 2);
  }
  const uint32_t tile_bytes = (uint32_t)(BKV * p.kv_stride * 2);
  auto issue = [&](int kv0, bf16_t* kn, bf16_t* vn) {
    const uint32_t row = (uint32_t)(kv0 / BKV) * tile_bytes;
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, MLLM_LDS_VOID(kn + (wave * PER_WAVE + i) * 512), 16,
                                               (int)kv_off[i], (int)row, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, MLLM_LDS_VOID(vn + (wave * PER_WAVE + i) * 512), 16,
                                               (int)kv_off[i], (int)row, 0, 0);
    }
  };

  // One key tile: wait for its loads (enqueued a tile ago), barrier (every wavefront is now done
  // with the other stage), multiply; the loads of the next tile into the other stage go out one
  // behind each of the first score MFMAs, so the wavefront does not stand still while the memory
  // pipeline takes them (issued in one run behind the barrier they held it for 0.2 us per tile).
  auto tile = [&](const bf16_t* Ks, const bf16_t* Vs, bf16_t* Kn, bf16_t* Vn, int kv0, bool live) {
    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s[NB];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) s[b][v] = 0.f;
    // Scores: the LDS reads of the K fragments run four ahead of their MFMAs.
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < NC; c++)
#pragma unroll
      for (int b = 0; b < NB; b++)
        s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<HD>(Ks, 32 * b, c, lane), qf[c], s[b], 0, 0, 0);
    issue(kv0 + BKV, Kn, Vn);
    static_assert(NC * NB >= 4 + 2 * PER_WAVE, "a slot behind an MFMA for every load");
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    reads_and_loads_behind_mfmas(std::make_integer_sequence<int, 2 * PER_WAVE>{});
    reads_behind_mfmas<1>(std::make_integer_sequence<int, NC * NB - 4 - 2 * PER_WAVE>{});
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    __builtin_amdgcn_sched_barrier(0);
    // A tile past the end, or wholly above the diagonal of this wavefront's rows (wavefront-uniform):
    // its score MFMAs have carried the next tile's loads, their results are dropped.  (Leaving
    // before them would need a second copy of the loads on that path, which costs the main path
    // some fifty registers.)
    if (!live || (t.causal && kv0 > wave_last_q)) return;
    // First V fragment: its LDS latency runs under the softmax.
    bf16x8 fv = frag_cols_permuted<HD>(Vs, 0, 0, lane);
    __builtin_amdgcn_sched_barrier(0);
    // Only tiles that cross the segment end or the diagonal need the mask (wavefront-uniform).
    const bool need_mask = (kv0 + BKV > t.seg_len) || (t.causal && kv0 + BKV - 1 > wave_first_q);
    if (need_mask) {
#pragma unroll
      for (int b = 0; b < NB; b++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int kv = kv0 + 32 * b + acc_row(v, h);
          const bool vis = kv < t.seg_len && (!t.causal || kv <= qrow);
          s[b][v] = vis ? s[b][v] : -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) mx = fmaxf(mx, s[b][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;
    // The reference maximum follows the row maximum lazily: it moves only when a tile exceeds it by
    // more than 8 (log2 units).  Probabilities then reach 2^8 at most, which fp32 sums and the bf16
    // operand carry at the same relative precision, and the 64-value rescaling of the output
    // accumulator below is needed on a few tiles instead of on nearly every one (with 64 query rows
    // per wavefront some row finds a slightly larger score in almost every tile).
    const float m_new = mx > m + 8.f ? mx : m;
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m - m_use);
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        s[b][v] = fast_exp2(fmaf(s[b][v], c2, -m_use));
        rs += s[b][v];
      }
    l = l * alpha + rs;
    if (__any(m_new != m)) {  // the accumulator only needs rescaling when some row's maximum moved
#pragma unroll
      for (int d = 0; d < ND; d++)
#pragma unroll
        for (int v = 0; v < 16; v++) oacc[d][v] *= alpha;
    }
    m = m_new;
    bf16x8 pf[NB][2];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
      for (int cc = 0; cc < 2; cc++) pf[b][cc] = acc_to_frag(s[b], cc);
    __builtin_amdgcn_sched_barrier(0);
    // O^T += V^T.P^T: each MFMA is preceded by the two LDS reads of the next V fragment.
    constexpr int NPV = NB * 2 * ND;
#pragma unroll
    for (int i = 0; i < NPV; i++) {
      const int bc = i / ND, d = i % ND;          // bc = 2 b + cc
      bf16x8 nv = fv;
      if (i + 1 < NPV) nv = frag_cols_permuted<HD>(Vs, 16 * ((i + 1) / ND), 32 * ((i + 1) % ND), lane);
      oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, pf[bc / 2][bc % 2], oacc[d], 0, 0, 0);
      fv = nv;
    }
    reads_before_mfmas<2>(std::make_integer_sequence<int, NPV - 1>{});
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_barrier(0);
  };

  issue(0, Ks0, Vs0);
  for (int kv0 = 0; kv0 < kv_end; kv0 += 2 * BKV) {
    tile(Ks0, Vs0, Ks1, Vs1, kv0, true);
    tile(Ks1, Vs1, Ks0, Vs0, kv0 + BKV, kv0 + BKV < kv_end);
  }
  // the last enqueued loads (rows past the end: zeros) must have landed before this workgroup's
  // LDS can be handed to another one
  __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);
  l += __shfl_xor(l, 32, 64);
  if (!qok) return;
  const float inv = 1.f / l;
  bf16_t* op = p.o + (int64_t)(t.seg_start + qrow) * p.o_stride + head * HD;
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      uint2 w;
      w.x = pack_bf16x2(oacc[d][4 * g4] * inv, oacc[d][4 * g4 + 1] * inv);
      w.y = pack_bf16x2(oacc[d][4 * g4 + 2] * inv, oacc[d][4 * g4 + 3] * inv);
      *reinterpret_cast<uint2*>(op + 32 * d + 8 * g4 + 4 * h) = w;
    }
  if (h == 0) p.lse[(int64_t)head * p.T + t.seg_start + qrow] = (m + log2f(l)) * LN2;
}

// ---------------------------------------------------------------------------------------------
// dQ pass: one workgroup per (query tile of 128, head), looping over key tiles.  It runs first in
// the backward pass and also produces delta[h][t] = sum_d dO[t,h,d] * O[t,h,d] for the dK/dV pass.
// ---------------------------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(AttnParams p) {
  constexpr int NC = HD / 16, ND = HD / 32, TILE = BKV * HD;
  // K and V tiles go straight to LDS, two stages each (as in the forward kernel).
  __shared__ __attribute__((aligned(1024))) bf16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vs0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Vs1[TILE];
  AttnItem t;
  if (!work_item(p.list, t)) return;
  const int head = t.head, kvh = head / (p.Hq / p.Hkv);
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qrow = t.tile0 + 32 * wave + (lane & 31);
  const bool qok = qrow < t.seg_len;
  const int64_t grow = t.seg_start + (qok ? qrow : 0);
  const bf16_t* qp = p.q + grow * p.q_stride + head * HD + 8 * h;
  const bf16_t* dop = p.d_o + grow * p.o_stride + head * HD + 8 * h;
  bf16x8 qf[NC], dof[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) {
    qf[c] = global_frag(qp + 16 * c, qok);
    dof[c] = global_frag(dop + 16 * c, qok);
  }
  // Rows beyond the segment get lse = +inf, so their probabilities are exp2(-inf) = 0.
  const float lse2 = qok ? p.lse[(int64_t)head * p.T + grow] * LOG2E : INFINITY;
  // delta = rowsum(dO * O) of the lane's query row: each half-wavefront holds half of the row's
  // columns (the dO fragments above, O fetched the same way).  The dK/dV pass, which runs after this
  // kernel, reads it from p.delta.
  float delta = 0.f;
  {
    const bf16_t* op = p.o + grow * p.o_stride + head * HD + 8 * h;
#pragma unroll
    for (int c = 0; c < NC; c++) {
      Frag8 fo, fd;
      fo.v = global_frag(op + 16 * c, qok);
      fd.v = dof[c];
#pragma unroll
      for (int w = 0; w < 4; w++) delta += bf16lo(fo.w[w]) * bf16lo(fd.w[w]) + bf16hi(fo.w[w]) * bf16hi(fd.w[w]);
    }
    delta += __shfl_xor(delta, 32, 64);
    if (qok && h == 0) p.delta[(int64_t)head * p.T + grow] = delta;
  }
  const int wave_first_q = t.tile0 + 32 * wave;

  const bf16_t* kbase = p.k + (int64_t)t.seg_start * p.kv_stride + kvh * HD;
  const bf16_t* vbase = p.v + (int64_t)t.seg_start * p.kv_stride + kvh * HD;
  const int kv_end = t.causal ? min(t.seg_len, t.tile0 + ATTN_FWD_Q_TILE) : t.seg_len;
  const int wave_last_q = t.tile0 + 32 * wave + 31;

  f32x16 dqacc[ND];
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int v = 0; v < 16; v++) dqacc[d][v] = 0.f;

  const __amdgpu_buffer_rsrc_t rk = rows_rsrc(kbase, p.kv_stride, kv_end, HD), rv = rows_rsrc(vbase, p.kv_stride, kv_end, HD);
  constexpr int CPR = HD / 8, RPI = 64 / CPR, PER_WAVE = BKV / RPI / 4;
  uint32_t kv_off[PER_WAVE];
#pragma unroll
  for (int i = 0; i < PER_WAVE; i++) {
    const int r = (wave * PER_WAVE + i) * RPI + lane / CPR, c = (lane % CPR) ^ swz<HD>(r);
    kv_off[i] = (uint32_t)((r * p.kv_stride + 8 * c) * 2);
  }
  const uint32_t tile_bytes = (uint32_t)(BKV * p.kv_stride * 2);
  auto issue = [&](int kv0, bf16_t* kn, bf16_t* vn) {   // rows past kv_end: zeros, no traffic
    const uint32_t row = (uint32_t)(kv0 / BKV) * tile_bytes;
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, MLLM_LDS_VOID(kn + (wave * PER_WAVE + i) * 512), 16,
                                               (int)kv_off[i], (int)row, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, MLLM_LDS_VOID(vn + (wave * PER_WAVE + i) * 512), 16,
                                               (int)kv_off[i], (int)row, 0, 0);
    }
  };
  auto tile = [&](const bf16_t* Ks, const bf16_t* Vs, bf16_t* Kn, bf16_t* Vn, int kv0, bool live) {
    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < BKV / 32; b++) {
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; v++) { s[v] = 0.f; dp[v] = 0.f; }
      // Scores and dP: the LDS reads run AHEAD fragments in front of their MFMAs.  At head_dim 128 the
      // kernel stands at the 256 registers that two wavefronts per SIMD allow, and a request for four
      // fragments ahead is not refused but dropped as a whole: every MFMA then waits for a read
      // issued right in front of it (measured 4 % slower than two ahead, which fits).
      constexpr int AHEAD = HD == 128 ? 2 : 4;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < NC; c++) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<HD>(Ks, 32 * b, c, lane), qf[c], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<HD>(Vs, 32 * b, c, lane), dof[c], dp, 0, 0, 0);
      }
      if (b == 0) {
        // the next tile's loads go out one behind each of the first MFMAs (see the forward kernel)
        issue(kv0 + BKV, Kn, Vn);
        static_assert(2 * NC >= AHEAD + 2 * PER_WAVE, "a slot behind an MFMA for every load");
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
        reads_and_loads_behind_mfmas(std::make_integer_sequence<int, 2 * PER_WAVE>{});
        reads_behind_mfmas<1>(std::make_integer_sequence<int, 2 * NC - AHEAD - 2 * PER_WAVE>{});
        __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
      } else {
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
        reads_behind_mfmas<1>(std::make_integer_sequence<int, 2 * NC - AHEAD>{});
        __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // a tile past the end or wholly above this wavefront's diagonal: only the loads were wanted
      if (b == 0 && (!live || (t.causal && kv0 > wave_last_q))) return;
      // First K^T fragment of the dQ product: its LDS latency runs under the vector work.
      bf16x8 fk = frag_cols_permuted<HD>(Ks, 32 * b, 0, lane);
      __builtin_amdgcn_sched_barrier(0);
      const bool need_mask = (kv0 + 32 * b + 32 > t.seg_len) || (t.causal && kv0 + 32 * b + 31 > wave_first_q);
      if (need_mask) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int kv = kv0 + 32 * b + acc_row(v, h);
          const bool vis = kv < t.seg_len && (!t.causal || kv <= qrow);
          s[v] = vis ? s[v] : -INFINITY;
        }
      }
#pragma unroll
      for (int v = 0; v < 16; v++) s[v] = fast_exp2(fmaf(s[v], p.scale_log2e, -lse2)) * (dp[v] - delta);   // dS^T
      bf16x8 dsf[2];
#pragma unroll
      for (int cc = 0; cc < 2; cc++) dsf[cc] = acc_to_frag(s, cc);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int NDQ = 2 * ND;
#pragma unroll
      for (int i = 0; i < NDQ; i++) {
        bf16x8 nk = fk;
        if (i + 1 < NDQ) nk = frag_cols_permuted<HD>(Ks, 32 * b + 16 * ((i + 1) / ND), 32 * ((i + 1) % ND), lane);
        dqacc[i % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, dsf[i / ND], dqacc[i % ND], 0, 0, 0);
        fk = nk;
      }
      reads_before_mfmas<2>(std::make_integer_sequence<int, NDQ - 1>{});
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  issue(0, Ks0, Vs0);
  for (int kv0 = 0; kv0 < kv_end; kv0 += 2 * BKV) {
    tile(Ks0, Vs0, Ks1, Vs1, kv0, true);
    tile(Ks1, Vs1, Ks0, Vs0, kv0 + BKV, kv0 + BKV < kv_end);
  }
  __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);   // the last enqueued tile (zeros) has landed
  if (!qok) return;
  float out_scale = p.scale;
  if (p.rope_table) {   // the scale rides on the rotation's factors
    rope_unrotate<HD>(dqacc, p.rope_table, qrow, h, p.scale);
    out_scale = 1.f;
  }
  bf16_t* dqp = p.dq + grow * p.q_stride + head * HD;
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      uint2 w;
      w.x = pack_bf16x2(dqacc[d][4 * g4] * out_scale, dqacc[d][4 * g4 + 1] * out_scale);
      w.y = pack_bf16x2(dqacc[d][4 * g4 + 2] * out_scale, dqacc[d][4 * g4 + 3] * out_scale);
      *reinterpret_cast<uint2*>(dqp + 32 * d + 8 * g4 + 4 * h) = w;
    }
}

// ---------------------------------------------------------------------------------------------
// dK/dV pass: one workgroup per (key tile of 128, kv head); each wavefront owns 32 key rows and
// loops over the query heads of the group and the query tiles that can see its keys.
//
// The query-side tiles (Q, dO) are double-buffered in LDS and filled by buffer loads that write
// LDS directly (no staging registers, no LDS store instructions): the loads of tile i+1 are
// enqueued right after the barrier that opens tile i and have all of tile i's MFMAs to land.
// One such instruction moves 64 chunks of 16 bytes into 1 KiB of LDS, lane l to chunk position
// l % CPR of row l / CPR; the lane therefore asks for the global chunk that the XOR swizzle keeps
// at that position.  Rows past the segment are out of the descriptor's range and arrive as zeros.
// ---------------------------------------------------------------------------------------------
// s_waitcnt vmcnt(0) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)

template <int HD>
__global__ __launch_bounds__(256, HD == 64 ? 2 : 1) void attn_bwd_dkv_kernel(AttnParams p) {
  constexpr int NC = HD / 16, ND = HD / 32, TILE = BQ * HD;
  __shared__ __attribute__((aligned(1024))) bf16_t Qs0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t Qs1[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t dOs0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t dOs1[TILE];
  __shared__ float lse_s0[BQ], lse_s1[BQ], delta_s0[BQ], delta_s1[BQ];
  AttnItem t;
  if (!work_item(p.list, t)) return;
  const int kvh = t.head, grp = p.Hq / p.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int krow = t.tile0 + 32 * wave + (lane & 31);
  const bool kok = krow < t.seg_len;
  const int64_t gkrow = t.seg_start + (kok ? krow : 0);
  const bf16_t* kp = p.k + gkrow * p.kv_stride + kvh * HD + 8 * h;
  const bf16_t* vp = p.v + gkrow * p.kv_stride + kvh * HD + 8 * h;
  bf16x8 kf[NC], vf[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) {
    kf[c] = global_frag(kp + 16 * c, kok);
    vf[c] = global_frag(vp + 16 * c, kok);
  }
  f32x16 dkacc[ND], dvacc[ND];
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dkacc[d][v] = 0.f; dvacc[d][v] = 0.f; }

  const int q_begin = t.causal ? (t.tile0 / BQ) * BQ : 0;
  const int wave_first_k = t.tile0 + 32 * wave;
  const int n_it = grp * ((t.seg_len - q_begin + BQ - 1) / BQ);

  constexpr int CPR = HD / 8, RPI = 64 / CPR, PER_WAVE = BQ / RPI / 4;
  uint32_t q_off[PER_WAVE], do_off[PER_WAVE];
#pragma unroll
  for (int i = 0; i < PER_WAVE; i++) {
    const int r = (wave * PER_WAVE + i) * RPI + lane / CPR, c = (lane % CPR) ^ swz<HD>(r);
    q_off[i] = (uint32_t)((r * p.q_stride + 8 * c) * 2);
    do_off[i] = (uint32_t)((r * p.o_stride + 8 * c) * 2);
  }
  const uint32_t q_bytes = (uint32_t)(((int64_t)(t.seg_len - 1) * p.q_stride + HD) * 2);
  const uint32_t do_bytes = (uint32_t)(((int64_t)(t.seg_len - 1) * p.o_stride + HD) * 2);

  // The tile to be loaded next: query head nj of the group, query rows from nq0.  Past the last
  // tile the descriptors are empty and the loads write zeros.
  int nj = 0, nq0 = q_begin;
  float r_lse = 0.f, r_delta = 0.f;   // statistics of the tile in flight, one row per thread (tid < BQ)
  bool r_ok = false;
  auto issue = [&](bf16_t* qs, bf16_t* dos) {
    const bool valid = nj < grp;
    const int head = kvh * grp + (valid ? nj : 0);
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.q + (int64_t)t.seg_start * p.q_stride + head * HD), 0, valid ? (int)q_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rdo = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.d_o + (int64_t)t.seg_start * p.o_stride + head * HD), 0, valid ? (int)do_bytes : 0, 0x00020000);
    const uint32_t qrow = (uint32_t)nq0 * (uint32_t)(p.q_stride * 2), dorow = (uint32_t)nq0 * (uint32_t)(p.o_stride * 2);
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rq, MLLM_LDS_VOID(qs + (wave * PER_WAVE + i) * 512), 16,
                                               (int)(q_off[i] + qrow), 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdo, MLLM_LDS_VOID(dos + (wave * PER_WAVE + i) * 512), 16,
                                               (int)(do_off[i] + dorow), 0, 0, 0);
    }
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.lse + (int64_t)head * p.T + t.seg_start), 0, valid ? t.seg_len * 4 : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.delta + (int64_t)head * p.T + t.seg_start), 0, valid ? t.seg_len * 4 : 0, 0x00020000);
    const uint32_t so = tid < BQ ? (uint32_t)(nq0 + tid) * 4u : 0xFFFFFFFFu;
    r_lse = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rl, (int)so, 0, 0));
    r_delta = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rd, (int)so, 0, 0));
    r_ok = valid && tid < BQ && nq0 + tid < t.seg_len;
    nq0 += BQ;
    if (nq0 >= t.seg_len) { nq0 = q_begin; nj++; }
  };

  // One tile: publish the statistics of the tile whose loads were enqueued a tile ago, wait for
  // those loads, barrier (every wavefront is now done with the other stage), enqueue the next
  // tile into the other stage, multiply.
  auto tile = [&](const bf16_t* Qs, const bf16_t* dOs, float* lse_s, float* delta_s, bf16_t* Qn, bf16_t* dOn,
                  int q0, bool live) {
    if (tid < BQ) {
      lse_s[tid] = r_ok ? r_lse * LOG2E : INFINITY;   // +inf: probabilities of rows past the segment are 0
      delta_s[tid] = r_ok ? r_delta : 0.f;
    }
    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);
    __syncthreads();
    issue(Qn, dOn);
    __builtin_amdgcn_sched_barrier(0);
    if (!live || (t.causal && q0 + BQ - 1 < wave_first_k)) return;  // no query here sees this wave's keys
#pragma unroll
    for (int b = 0; b < BQ / 32; b++) {
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; v++) { s[v] = 0.f; dp[v] = 0.f; }
      // Scores: 2 NC MFMAs, their LDS reads issued four ahead (left alone, the scheduler reads
      // each fragment into the same registers right before its MFMA and waits for it every time).
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < NC; c++) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<HD>(Qs, 32 * b, c, lane), kf[c], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<HD>(dOs, 32 * b, c, lane), vf[c], dp, 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
      reads_behind_mfmas<1>(std::make_integer_sequence<int, 2 * NC - 4>{});
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_sched_barrier(0);
      // First fragments of the dV / dK products: their LDS latency runs under the vector work.
      constexpr int NPV = 2 * ND;            // (cc, d) pairs, two MFMAs each
      bf16x8 fdo = frag_cols_permuted<HD>(dOs, 32 * b, 0, lane), fq = frag_cols_permuted<HD>(Qs, 32 * b, 0, lane);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 pr;
      // The scores are consumed by the vector ALU: keep them out of the accumulation registers
      // (with the whole register file available the allocator otherwise parks them there and
      // copies every value back and forth).
#pragma unroll
      for (int v = 0; v < 16; v++) {
        float a = s[v], c = dp[v];
        asm volatile("" : "+v"(a), "+v"(c));
        s[v] = a;
        dp[v] = c;
      }
      if (t.causal && q0 + 32 * b <= wave_first_k + 31) {   // block touches the diagonal
#pragma unroll
        for (int v = 0; v < 16; v++) s[v] = (krow <= q0 + 32 * b + acc_row(v, h)) ? s[v] : -INFINITY;
      }
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int qi = 32 * b + acc_row(v, h);
        pr[v] = fast_exp2(fmaf(s[v], p.scale_log2e, -lse_s[qi]));
        s[v] = pr[v] * (dp[v] - delta_s[qi]);   // dS
      }
      bf16x8 pf[2], dsf[2];
#pragma unroll
      for (int cc = 0; cc < 2; cc++) { pf[cc] = acc_to_frag(pr, cc); dsf[cc] = acc_to_frag(s, cc); }
      __builtin_amdgcn_sched_barrier(0);
      // dV, dK: every pair of MFMAs is preceded by the four LDS reads of the next pair's fragments.
#pragma unroll
      for (int i = 0; i < NPV; i++) {
        const int cc = i / ND, d = i % ND;
        bf16x8 ndo = fdo, nq = fq;
        if (i + 1 < NPV) {
          const int cc1 = (i + 1) / ND, d1 = (i + 1) % ND;
          ndo = frag_cols_permuted<HD>(dOs, 32 * b + 16 * cc1, 32 * d1, lane);
          nq = frag_cols_permuted<HD>(Qs, 32 * b + 16 * cc1, 32 * d1, lane);
        }
        dvacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fdo, pf[cc], dvacc[d], 0, 0, 0);
        dkacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq, dsf[cc], dkacc[d], 0, 0, 0);
        fdo = ndo;
        fq = nq;
      }
      reads_before_mfma_pairs(std::make_integer_sequence<int, NPV - 1>{});
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  issue(Qs0, dOs0);
  int q0 = q_begin;
  auto advance = [&]() { q0 += BQ; if (q0 >= t.seg_len) q0 = q_begin; };
  for (int it = 0; it < n_it; it += 2) {
    tile(Qs0, dOs0, lse_s0, delta_s0, Qs1, dOs1, q0, true);
    advance();
    tile(Qs1, dOs1, lse_s1, delta_s1, Qs0, dOs0, q0, it + 1 < n_it);
    advance();
  }
  // the last enqueued loads (an empty tile: zeros) must have landed before this workgroup's LDS
  // can be handed to another one
  __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_0);
  if (!kok) return;
  float out_scale = p.scale;
  if (p.rope_table) {
    rope_unrotate<HD>(dkacc, p.rope_table, krow, h, p.scale);
    out_scale = 1.f;
  }
  bf16_t* dkp = p.dk + gkrow * p.kv_stride + kvh * HD;
  bf16_t* dvp = p.dv + gkrow * p.kv_stride + kvh * HD;
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      uint2 w;
      w.x = pack_bf16x2(dkacc[d][4 * g4] * out_scale, dkacc[d][4 * g4 + 1] * out_scale);
      w.y = pack_bf16x2(dkacc[d][4 * g4 + 2] * out_scale, dkacc[d][4 * g4 + 3] * out_scale);
      *reinterpret_cast<uint2*>(dkp + 32 * d + 8 * g4 + 4 * h) = w;
      w.x = pack_bf16x2(dvacc[d][4 * g4], dvacc[d][4 * g4 + 1]);
      w.y = pack_bf16x2(dvacc[d][4 * g4 + 2], dvacc[d][4 * g4 + 3]);
      *reinterpret_cast<uint2*>(dvp + 32 * d + 8 * g4 + 4 * h) = w;
    }
}

// ---------------------------------------------------------------------------------------------
// dK/dV pass, software-pipelined form.  The work of a block of 32 query rows is a chain: scores and
// dP (MFMA) -> probabilities and dS (vector ALU, 1/4 of it the exponential) -> dV and dK (MFMA).
// Run as a chain, with one wavefront per SIMD at head_dim 128, the matrix pipe idles during the
// vector stage and the vector ALU during the other two.  Here every step works on two blocks: the
// score MFMAs of block n+1 are issued one per slot and the vector work of block n is cut into as
// many slices, one behind each MFMA (the matrix pipe runs an MFMA for 32 clocks while the wavefront
// goes on issuing independent instructions); the dV/dK MFMAs of block n follow, carrying the LDS
// reads of the next steps.  The Q / dO tiles rotate through NST stages of LDS: a tile is still
// being read (dV/dK of its second block) after the barrier that opens the next tile, so the tile
// after that is loaded into a third stage.  The stage base is part of the address registers, which
// are advanced once per tile; block and operand offsets ride in the instructions' offset fields.
// ---------------------------------------------------------------------------------------------
typedef MLLM_LDS const char* lds_cptr;
__device__ __forceinline__ bf16x8 lds_b128(lds_cptr base, uint32_t off) {
  return __builtin_bit_cast(bf16x8, *(MLLM_LDS const u32x4_t*)(base + off));
}
__device__ __forceinline__ s16x4 lds_tr(lds_cptr base, uint32_t off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)(base + off));
}
__device__ __forceinline__ f32x4 lds_f4(lds_cptr base, uint32_t off) { return *(MLLM_LDS const f32x4*)(base + off); }
template <int V> using Int = std::integral_constant<int, V>;
// Loads from global memory straight into LDS, written as assembly so that the compiler does not
// know them for what they are.  Told (through the builtin), it makes LDS reads wait for every such
// load in flight into the same LDS variable, which turns a queue of several tiles on their way
// into one tile at a time; it cannot see that the loads go to a stage nobody reads when the stage
// numbers are run-time values.  The kernel that uses these waits for its loads by count and
// separates writers from readers with barriers, as it has to anyway.
// The 64 lanes' 16 (or 4) bytes land side by side from LDS address `lds_addr` (wavefront-uniform).
// The statements set M0 themselves; M0 is a reserved register that the compiler holds no value in and
// sets anew in front of each of its own uses, so overwriting it here disturbs nothing.
typedef int i32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4_t raw_rsrc(const void* base, uint32_t bytes) {   // untyped buffer over [base, base + bytes)
  const uint64_t b = (uint64_t)base;
  i32x4_t r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(b >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}
__device__ __forceinline__ void load_to_lds_b128(i32x4_t rsrc, uint32_t lds_addr, uint32_t byte_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(byte_off), "s"(rsrc) : "memory");
}
__device__ __forceinline__ void load_to_lds_b32(i32x4_t rsrc, uint32_t lds_addr, uint32_t byte_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(byte_off), "s"(rsrc) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(MLLM_LDS const void* p) { return (uint32_t)(size_t)p; }
// At most N of the loads above still in flight (the compiler does not count them, so neither can its builtin).
template <int N>
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

template <int HD>
__global__ __launch_bounds__(256, HD == 64 ? 2 : 1) void attn_bwd_dkv_pipe_kernel(AttnParams p) {
  constexpr int NC = HD / 16, ND = HD / 32, TILE = BQ * HD, NST = 4;
  constexpr int TILE_B = TILE * 2;                          // a stage: the Q tile, then the dO tile
  constexpr int ROWS32_B = 32 * HD * 2, ROWS16_B = 16 * HD * 2;
  constexpr int STAGE_B = 2 * TILE_B, STAT_STAGE_B = 2 * BQ * 4;
  // NST stages of tiles, then NST stages of row statistics (lse of the tile's rows, then delta).  ONE
  // array on purpose: the compiler tags LDS accesses with the variable they belong to and makes every
  // read of a variable wait for all loads in flight into the same variable; it cannot tell the stages
  // of one array apart when their numbers are run-time values.  With a single variable there is
  // nothing to tag, and the waits below (which know the stages) are the only ones.
  constexpr int STATS_AT = NST * STAGE_B;
  __shared__ __attribute__((aligned(1024))) char lds[NST * STAGE_B + NST * STAT_STAGE_B];
  AttnItem t;
  if (!work_item(p.list, t)) return;
  const int kvh = t.head, grp = p.Hq / p.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int krow = t.tile0 + 32 * wave + (lane & 31);
  const bool kok = krow < t.seg_len;
  const int64_t gkrow = t.seg_start + (kok ? krow : 0);
  const bf16_t* kp = p.k + gkrow * p.kv_stride + kvh * HD + 8 * h;
  const bf16_t* vp = p.v + gkrow * p.kv_stride + kvh * HD + 8 * h;
  bf16x8 kf[NC], vf[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) {
    kf[c] = global_frag(kp + 16 * c, kok);
    vf[c] = global_frag(vp + 16 * c, kok);
  }
  // MFMA operands may sit in accumulation registers: park these 64 there for the whole kernel and
  // leave the vector registers to the values that the vector ALU touches
#pragma unroll
  for (int c = 0; c < NC; c++) asm volatile("" : "+a"(kf[c]), "+a"(vf[c]));
  f32x16 dkacc[ND], dvacc[ND];
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dkacc[d][v] = 0.f; dvacc[d][v] = 0.f; }

  const int q_begin = t.causal ? (t.tile0 / BQ) * BQ : 0;
  const int wave_first_k = t.tile0 + 32 * wave;
  const int n_it = grp * ((t.seg_len - q_begin + BQ - 1) / BQ);
  const float c2 = p.scale_log2e;

  // ---- loads ------------------------------------------------------------------------------------
  constexpr int CPR = HD / 8, RPI = 64 / CPR, PER_WAVE = BQ / RPI / 4;
  constexpr int PT = 2 * PER_WAVE + 1;   // load instructions per wavefront and tile
  uint32_t q_off[PER_WAVE], do_off[PER_WAVE];
#pragma unroll
  for (int i = 0; i < PER_WAVE; i++) {
    const int r = (wave * PER_WAVE + i) * RPI + lane / CPR, c = (lane % CPR) ^ swz<HD>(r);
    q_off[i] = (uint32_t)((r * p.q_stride + 8 * c) * 2);
    do_off[i] = (uint32_t)((r * p.o_stride + 8 * c) * 2);
  }
  const uint32_t q_bytes = (uint32_t)(((int64_t)(t.seg_len - 1) * p.q_stride + HD) * 2);
  const uint32_t do_bytes = (uint32_t)(((int64_t)(t.seg_len - 1) * p.o_stride + HD) * 2);
  int nj = 0, nq0 = q_begin;          // the tile to be loaded next: query head nj of the group, rows from nq0
  // Past the last tile the descriptors are empty and the loads write zeros.
  const uint32_t lds_b = lds_address((MLLM_LDS const void*)lds);
  // A tile's loads are enqueued in PT parts so that they can be spread over the MFMAs of a stage.
  i32x4_t rq, rdo, rst;
  uint32_t qrow, dorow, dst_t, dst_s;
  auto issue_begin = [&](int stage) {
    const bool valid = nj < grp;
    const int head = kvh * grp + (valid ? nj : 0);
    rq = raw_rsrc(p.q + (int64_t)t.seg_start * p.q_stride + head * HD, valid ? q_bytes : 0u);
    rdo = raw_rsrc(p.d_o + (int64_t)t.seg_start * p.o_stride + head * HD, valid ? do_bytes : 0u);
    // lse and delta of the tile's rows, 64 floats each, one instruction each: even wavefronts bring
    // lse, odd ones delta (twice the same bytes, so that every wavefront counts the same loads).
    // Rows past the segment read as zero; their dO rows are zero too, so they add nothing.
    rst = raw_rsrc(((wave & 1) ? p.delta : p.lse) + (int64_t)head * p.T + t.seg_start, valid ? (uint32_t)t.seg_len * 4u : 0u);
    qrow = (uint32_t)nq0 * (uint32_t)(p.q_stride * 2);
    dorow = (uint32_t)nq0 * (uint32_t)(p.o_stride * 2);
    dst_t = lds_b + (uint32_t)(stage * STAGE_B + (wave * PER_WAVE) * 1024);
    dst_s = lds_b + (uint32_t)(STATS_AT + stage * STAT_STAGE_B + (wave & 1) * BQ * 4);
  };
  auto issue_part = [&](int j) {
    if (j < PER_WAVE) load_to_lds_b128(rq, dst_t + j * 1024, q_off[j] + qrow);
    else if (j < 2 * PER_WAVE) load_to_lds_b128(rdo, dst_t + TILE_B + (j - PER_WAVE) * 1024, do_off[j - PER_WAVE] + dorow);
    else load_to_lds_b32(rst, dst_s, (uint32_t)(nq0 + lane) * 4u);
  };
  auto issue_end = [&]() {
    nq0 += BQ;
    if (nq0 >= t.seg_len) { nq0 = q_begin; nj++; }
  };
  auto issue = [&](int stage) {
    issue_begin(stage);
#pragma unroll
    for (int j = 0; j < PT; j++) issue_part(j);
    issue_end();
  };

  // ---- lane parts of the LDS offsets, stage included (advanced once per tile); block and operand ride
  // in the instructions' offset fields ------------------------------------------------------------
  // natural-layout fragment (frag_rows): tile row lane%32 of a 32-row block, 16-byte chunk 2c + h
  // transposed fragment (frag_cols_permuted): rows 4h + i16/4 (+8), columns 32d + 16*(lane/16 % 2) + 4*(i16 % 4)
  uint32_t rows_c[NC], rows_n[NC], cols_c[ND][2];   // _c: stage of the current tile, _n: of the next
  {
    const int r = lane & 31, i16 = lane & 15;
#pragma unroll
    for (int c = 0; c < NC; c++) {
      rows_c[c] = (uint32_t)(r * HD + 8 * ((2 * c + h) ^ swz<HD>(r))) * 2u;
      rows_n[c] = rows_c[c] + STAGE_B;
    }
#pragma unroll
    for (int d = 0; d < ND; d++)
#pragma unroll
      for (int e = 0; e < 2; e++) {
        const int k = 4 * h + (i16 >> 2) + 8 * e;
        const int n = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
        cols_c[d][e] = (uint32_t)(k * HD + 8 * ((n >> 3) ^ swz<HD>(k)) + (n & 7)) * 2u;
      }
  }
  uint32_t sa_c = STATS_AT + 16u * h, sa_n = sa_c + STAT_STAGE_B;
  int st_c = 0;   // stage of the current tile

  // ---- the two stages of a step ------------------------------------------------------------------
  const lds_cptr rt = (lds_cptr)lds, rs = (lds_cptr)lds;
  constexpr int NM = 2 * NC, EPS = 16 / NM, NPV = 2 * ND;
  constexpr int RD = NM < 8 ? NM / 2 : 8;   // score fragments are read RD slots ahead of their MFMA
  constexpr int PD = NPV < 8 ? NPV / 2 : 3;   // dV / dK fragments PD pairs ahead
  constexpr int SP = NPV / 4;               // pairs of the second stage that fetch the next block's statistics
  // carried from stage to stage
  bf16x8 pre[RD];            // the first fragments of the next score stage
  f32x16 s_n, dp_n;          // scores and dP of the block after the current one
  float xs[16], ts[16];      // current block: exponent (s scale - lse) log2 e, and dP - delta
  Frag8 pf[2], dsf[2];       // current block: P and dS as MFMA operands
  Frag8 fdo[NPV], fq[NPV];   // current block: transposed dO and Q fragments
  // transposing reads of pair i of the dV / dK products: rows 32 BC + 16 cc .. +15 of the current tile, columns 32 d .. +31
  auto pair_reads = [&](int BC, int i, int part) {   // part 0: the dO fragment, 1: the Q fragment
    const int cc = i / ND, d = i % ND;
    const uint32_t o = BC * ROWS32_B + cc * ROWS16_B;
    if (part == 0) { fdo[i].h[0] = lds_tr(rt, cols_c[d][0] + o + TILE_B); fdo[i].h[1] = lds_tr(rt, cols_c[d][1] + o + TILE_B); }
    else { fq[i].h[0] = lds_tr(rt, cols_c[d][0] + o); fq[i].h[1] = lds_tr(rt, cols_c[d][1] + o); }
  };
  // Score stage: S and dP of block BN of the tile at offsets rows_x, one MFMA per slot; behind each
  // MFMA a slice of the current block's (BC) vector work, P = exp2(xs), dS = P * ts, packed to bf16.
  // An MFMA has no side effect the compiler must keep in place: left alone, those whose results are
  // needed only later all move to the end of the loop body, out of their slots.  Passing each result
  // through an empty volatile statement ties it between its neighbours.
  auto sx = [&](auto BCt, auto BNt, const uint32_t (&rows_x)[NC]) {
    constexpr int BC = decltype(BCt)::value, BN = decltype(BNt)::value;
    bf16x8 fr[NM];
#pragma unroll
    for (int m = 0; m < RD; m++) fr[m] = pre[m];
    float prv[16], dsv[16];
    f32x16 zero;
#pragma unroll
    for (int v = 0; v < 16; v++) zero[v] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < NM; m++) {
      if (m + RD < NM) {
        fr[m + RD] = lds_b128(rt, rows_x[(m + RD) / 2] + ((m + RD) % 2) * TILE_B + BN * ROWS32_B);
      } else {   // the last 2 PD slots fetch the fragments of the first PD pairs, one fragment per slot
        const int j = m - (NM - 2 * PD);
        if (j >= 0) pair_reads(BC, j / 2, j % 2);
      }
      if (m % 2 == 0) {
        s_n = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[m], kf[m / 2], m == 0 ? zero : s_n, 0, 0, 0);
        asm volatile("" : "+a"(s_n));
      } else {
        dp_n = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[m], vf[m / 2], m == 1 ? zero : dp_n, 0, 0, 0);
        asm volatile("" : "+a"(dp_n));
      }
#pragma unroll
      for (int e = 0; e < EPS; e++) {
        const int v = m * EPS + e;
        prv[v] = fast_exp2(xs[v]);
        dsv[v] = prv[v] * ts[v];
        if (v & 1) {
          pf[v >> 3].w[(v >> 1) & 3] = pack_bf16x2(prv[v - 1], prv[v]);
          dsf[v >> 3].w[(v >> 1) & 3] = pack_bf16x2(dsv[v - 1], dsv[v]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // dV / dK stage of block BC: dV += dO^T.P, dK += Q^T.dS, a pair of MFMAs at a time.  Each pair
  // follows the transposing reads of the pair PD further on; the last pairs carry the first reads
  // of the next score stage instead (from rows_x, block BT).  The first pairs fetch the statistics of
  // the next block (offset sa_x, block BN), the later ones turn them and the fresh scores into xs, ts;
  // with ISSUE, the parts of a tile's loads ride along as well.
  auto dx = [&](auto BCt, auto BNt, auto BTt, auto ISSUEt, const uint32_t (&rows_x)[NC], uint32_t sa_x) {
    constexpr int BC = decltype(BCt)::value, BN = decltype(BNt)::value, BT = decltype(BTt)::value;
    constexpr bool ISSUE = decltype(ISSUEt)::value != 0;
    f32x4 st[8];   // lse of row groups 0..3, delta of row groups 0..3
#pragma unroll
    for (int i = 0; i < NPV; i++) {
      const int cc = i / ND, d = i % ND;
      if (i + PD < NPV) {
        pair_reads(BC, i + PD, 0);
        pair_reads(BC, i + PD, 1);
      } else {
        constexpr int PER = (RD + PD - 1) / PD;
        const int j0 = (i - (NPV - PD)) * PER;
#pragma unroll
        for (int m = j0; m < j0 + PER && m < RD; m++) pre[m] = lds_b128(rt, rows_x[m / 2] + (m % 2) * TILE_B + BT * ROWS32_B);
      }
      if (i < SP) {
#pragma unroll
        for (int g = i * 8 / SP; g < (i + 1) * 8 / SP; g++)
          st[g] = lds_f4(rs, sa_x + (g >= 4 ? BQ * 4 : 0) + (32 * BN + 8 * (g & 3)) * 4);
      } else {
#pragma unroll
        for (int v = (i - SP) * 16 / (NPV - SP); v < (i - SP + 1) * 16 / (NPV - SP); v++) {
          xs[v] = fmaf(s_n[v], c2, -(st[v >> 2][v & 3] * LOG2E));
          ts[v] = dp_n[v] - st[4 + (v >> 2)][v & 3];
        }
      }
      if (ISSUE) {
#pragma unroll
        for (int j = i * PT / NPV; j < (i + 1) * PT / NPV; j++) issue_part(j);
      }
      dvacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fdo[i].v, pf[cc].v, dvacc[d], 0, 0, 0);
      asm volatile("" : "+a"(dvacc[d]));
      dkacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[i].v, dsf[cc].v, dkacc[d], 0, 0, 0);
      asm volatile("" : "+a"(dkacc[d]));
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Causal blocks on or above the diagonal: masked pairs get exponent -inf, i.e. probability zero.
  auto mask_diag = [&](int q0b) {
    if (t.causal && q0b <= wave_first_k + 31) {
#pragma unroll
      for (int v = 0; v < 16; v++) xs[v] = (krow <= q0b + acc_row(v, h)) ? xs[v] : -INFINITY;
    }
  };

  int q0 = q_begin;
  // ---- prologue: tile 0 lands, its first block's scores are formed on their own ----------------
#pragma unroll
  for (int st = 0; st < NST - 1; st++) issue(st);
  wait_loads<(NST - 2) * PT>();
  __syncthreads();
  __builtin_amdgcn_sched_barrier(0);
  {
#pragma unroll
    for (int v = 0; v < 16; v++) { s_n[v] = 0.f; dp_n[v] = 0.f; }
#pragma unroll
    for (int c = 0; c < NC; c++) {
      s_n = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_b128(rt, rows_c[c]), kf[c], s_n, 0, 0, 0);
      dp_n = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_b128(rt, rows_c[c] + TILE_B), vf[c], dp_n, 0, 0, 0);
    }
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const f32x4 x = lds_f4(rs, sa_c + 8 * g * 4), y = lds_f4(rs, sa_c + BQ * 4 + 8 * g * 4);
#pragma unroll
      for (int e = 0; e < 4; e++) {
        xs[4 * g + e] = fmaf(s_n[4 * g + e], c2, -(x[e] * LOG2E));
        ts[4 * g + e] = dp_n[4 * g + e] - y[e];
      }
    }
#pragma unroll
    for (int m = 0; m < RD; m++) pre[m] = lds_b128(rt, rows_c[m / 2] + (m % 2) * TILE_B + ROWS32_B);
  }
  __builtin_amdgcn_sched_barrier(0);

  // One tile per iteration.  Block 0: P, dS against the scores of block 1; then tile it+1 must have
  // landed (the NST-3 tiles enqueued after it may still be on their way) and every wavefront must have
  // left tile it-1, whose stage takes tile it+NST-1, enqueued under dV, dK of block 0.  Block 1: P, dS
  // against the scores of block 0 of tile it+1, then its dV, dK.
  for (int it = 0; it < n_it; it++) {
    mask_diag(q0);
    sx(Int<0>{}, Int<1>{}, rows_c);
    wait_loads<(NST - 3) * PT>();
    __syncthreads();
    issue_begin(st_c == 0 ? NST - 1 : st_c - 1);
    __builtin_amdgcn_sched_barrier(0);
    dx(Int<0>{}, Int<1>{}, Int<0>{}, Int<1>{}, rows_n, sa_c);
    issue_end();
    mask_diag(q0 + 32);
    sx(Int<1>{}, Int<0>{}, rows_n);
    dx(Int<1>{}, Int<0>{}, Int<1>{}, Int<0>{}, rows_n, sa_n);
    // rotate the stages
    q0 += BQ;
    if (q0 >= t.seg_len) q0 = q_begin;
    const int st_n = st_c + 1 == NST ? 0 : st_c + 1, st_nn = st_n + 1 == NST ? 0 : st_n + 1;
    const uint32_t dc = st_n == 0 ? (uint32_t)(-(NST - 1) * STAGE_B) : (uint32_t)STAGE_B;
    const uint32_t dn = st_nn == 0 ? (uint32_t)(-(NST - 1) * STAGE_B) : (uint32_t)STAGE_B;
#pragma unroll
    for (int c = 0; c < NC; c++) { rows_c[c] += dc; rows_n[c] += dn; }
#pragma unroll
    for (int d = 0; d < ND; d++) { cols_c[d][0] += dc; cols_c[d][1] += dc; }
    sa_c += st_n == 0 ? (uint32_t)(-(NST - 1) * STAT_STAGE_B) : (uint32_t)STAT_STAGE_B;
    sa_n += st_nn == 0 ? (uint32_t)(-(NST - 1) * STAT_STAGE_B) : (uint32_t)STAT_STAGE_B;
    st_c = st_n;
  }
  // the loads enqueued last (tiles past the end: zeros) must have landed before this workgroup's LDS
  // can be handed to another one
  wait_loads<0>();
  if (!kok) return;
  float out_scale = p.scale;
  if (p.rope_table) {
    rope_unrotate<HD>(dkacc, p.rope_table, krow, h, p.scale);
    out_scale = 1.f;
  }
  bf16_t* dkp = p.dk + gkrow * p.kv_stride + kvh * HD;
  bf16_t* dvp = p.dv + gkrow * p.kv_stride + kvh * HD;
#pragma unroll
  for (int d = 0; d < ND; d++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      uint2 w;
      w.x = pack_bf16x2(dkacc[d][4 * g4] * out_scale, dkacc[d][4 * g4 + 1] * out_scale);
      w.y = pack_bf16x2(dkacc[d][4 * g4 + 2] * out_scale, dkacc[d][4 * g4 + 3] * out_scale);
      *reinterpret_cast<uint2*>(dkp + 32 * d + 8 * g4 + 4 * h) = w;
      w.x = pack_bf16x2(dvacc[d][4 * g4], dvacc[d][4 * g4 + 1]);
      w.y = pack_bf16x2(dvacc[d][4 * g4 + 2], dvacc[d][4 * g4 + 3]);
      *reinterpret_cast<uint2*>(dvp + 32 * d + 8 * g4 + 4 * h) = w;
    }
}

AttnParams make_params(const AttnArgs& a) {
  AttnParams p;
  p.q = (const bf16_t*)a.q; p.k = (const bf16_t*)a.k; p.v = (const bf16_t*)a.v;
  p.o = (bf16_t*)a.o; p.lse = a.lse; p.d_o = (const bf16_t*)a.d_o;
  p.dq = (bf16_t*)a.dq; p.dk = (bf16_t*)a.dk; p.dv = (bf16_t*)a.dv; p.delta = a.delta;
  p.q_stride = a.q_stride; p.kv_stride = a.kv_stride; p.o_stride = a.o_stride;
  p.T = a.total_tokens; p.Hq = a.n_q_heads; p.Hkv = a.n_kv_heads;
  p.list = nullptr;
  p.scale = 1.0f / sqrtf((float)a.head_dim);
  p.scale_log2e = p.scale * LOG2E;
  p.rope_table = a.rope_table;
  return p;
}

}  // namespace

// The kernels address K, V, Q and dO rows through 32-bit byte offsets from the segment start
// (buffer descriptors whose range ends at the last wanted row); a tile may run up to 255 rows
// past the end before the range check rejects it, so those offsets must not wrap either.
static bool offsets_fit(const AttnArgs& a) {
  const int64_t widest = std::max(a.q_stride, std::max(a.kv_stride, a.o_stride));
  return ((int64_t)a.total_tokens + 256) * widest * 2 < (int64_t)0xFFFFFFFFll;
}

hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s) {
  if (a.q_grid == 0) return hipSuccess;
  if (!offsets_fit(a)) return hipErrorInvalidValue;
  ProfScope prof(PROF_ATTN_FWD, a.fwd_flops, s);
  AttnParams p = make_params(a);
  p.list = (const AttnItem*)a.q_list;
  const dim3 grid((unsigned)a.q_grid), block(256);
  if (a.head_dim == 128) hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, block, 0, s, p);
  else if (a.head_dim == 64) hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, block, 0, s, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s) {
  if (a.q_grid == 0) return hipSuccess;
  if (!offsets_fit(a)) return hipErrorInvalidValue;
  ProfScope prof(PROF_ATTN_BWD, 2.0 * a.fwd_flops, s);
  AttnParams p = make_params(a);
  const dim3 block(256), qgrid((unsigned)a.q_grid), kgrid((unsigned)a.kv_grid);
  // dQ first: it writes delta, which the dK/dV pass reads
  if (a.head_dim == 128) {
    p.list = (const AttnItem*)a.q_list;
    hipLaunchKernelGGL(attn_bwd_dq_kernel<128>, qgrid, block, 0, s, p);
    p.list = (const AttnItem*)a.kv_list;
    hipLaunchKernelGGL(attn_bwd_dkv_pipe_kernel<128>, kgrid, block, 0, s, p);
  } else if (a.head_dim == 64) {
    p.list = (const AttnItem*)a.q_list;
    hipLaunchKernelGGL(attn_bwd_dq_kernel<64>, qgrid, block, 0, s, p);
    p.list = (const AttnItem*)a.kv_list;
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<64>, kgrid, block, 0, s, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace mllm
