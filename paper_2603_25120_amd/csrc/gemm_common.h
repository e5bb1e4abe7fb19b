// Pieces shared by the GEMM kernels: launch parameters, buffer resources, the XCD-aware tile
// order and the LDS-staged epilogue.
#pragma once
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace mllm {

constexpr int BK = 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t OOB = 0xFFFFFFFFu;  // byte offset beyond any buffer these kernels accept (< 4 GiB - 16)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

struct GemmParams {
  const bf16_t* a;
  const bf16_t* b;
  void* c;
  const bf16_t* bias;
  const bf16_t* res;
  int64_t M, N, K, lda, ldb, ldc, ldres;
  uint32_t a_bytes, b_bytes;
  int accumulate;
  int tiles_m, tiles_n;
  int kt_per_split;         // k-tiles handled by one workgroup row (gridDim.y splits of the K loop)
  int64_t c_split_stride;   // elements between the partial outputs of consecutive splits
  bf16_t* act;              // fused SwiGLU: silu(gate) * up, [M, N / 2]
  const bf16_t* pre;        // fused SwiGLU gradient: [gate | up], [M, 2 N]
  bf16_t* dpre;             //                        [d gate | d up], [M, 2 N]
  const float* rope_table;  // fused rotary positions: [positions, head_dim] fp32, cos then sin
  const int32_t* rope_pos;  //                         position of every row of C
  int64_t rope_cols;        //                         leading columns of C that are rotated heads
};

inline GemmParams make_gemm_params(const GemmArgs& g, int bm, int bn) {
  GemmParams p;
  p.a = (const bf16_t*)g.a; p.b = (const bf16_t*)g.b; p.c = g.c;
  p.bias = (const bf16_t*)g.bias; p.res = (const bf16_t*)g.residual;
  p.M = g.m; p.N = g.n; p.K = g.k; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldres = g.ldres;
  p.accumulate = g.accumulate;
  p.a_bytes = (uint32_t)((g.a_layout ? g.k : g.m) * g.lda * 2);
  p.b_bytes = (uint32_t)((g.b_layout ? g.n : g.k) * g.ldb * 2);
  p.tiles_m = (int)((g.m + bm - 1) / bm);
  p.tiles_n = (int)((g.n + bn - 1) / bn);
  p.kt_per_split = (int)((g.k + BK - 1) / BK);
  p.c_split_stride = 0;
  p.act = (bf16_t*)g.swiglu_act;
  p.pre = (const bf16_t*)g.swiglu_pre;
  p.dpre = (bf16_t*)g.swiglu_dpre;
  p.rope_table = g.rope_table;
  p.rope_pos = g.rope_pos;
  p.rope_cols = g.rope_cols;
  return p;
}

constexpr int GROUP_M = 8;

// Workgroups are dealt round-robin to the 8 XCDs.  Renumber so that each XCD gets a contiguous
// range of tile ids, then walk the tile grid in panels of GROUP_M tile-rows.
__device__ __forceinline__ void tile_of_block(int pid, int nblk, int tiles_m, int tiles_n,
                                              int& tm, int& tn) {
  const int per = (nblk + 7) >> 3, r = nblk & 7;
  const int x = pid & 7, local = pid >> 3;
  int off = (r == 0 || x <= r) ? x * per : r * per + (x - r) * (per - 1);
  int t = off + local;
  const int in_group = GROUP_M * tiles_n;
  const int gid = t / in_group;
  const int first_m = gid * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  tm = first_m + (t % in_group) % gsz;
  tn = (t % in_group) / gsz;
}

// Epilogue.  The MFMAs are issued with the operands swapped, so an accumulator block holds C
// transposed: a lane owns C row (lane%32) and acc[v] is column 8*(v/4) + 4*(lane/32) + v%4, i.e.
// runs of four consecutive columns.  One 32-row band at a time goes through a per-wavefront fp32
// staging area in LDS (32 x (WN+4) floats at `stage`) and leaves as 16-byte chunks (256 or 512
// contiguous bytes per row), with bias / residual / accumulate applied in fp32 and a single
// rounding on the way out.  Every wavefront of the workgroup must call it (it synchronises: once
// with WAVE_LOCAL, which is valid when each wavefront passes a staging area of its own).
template <int TM, int TN, bool OUT_F32, bool WAVE_LOCAL = false>
__device__ __forceinline__ void store_tile(const GemmParams& p, f32x16 (&acc)[TM][TN], float* stage,
                                           int64_t row0, int64_t col0, int lane) {
  constexpr int WN = 32 * TN, ST_STRIDE = WN + 4;
  const int h = lane >> 5, cl = lane & 31;
  constexpr int EPC = OUT_F32 ? 4 : 8;  // output elements per 16-byte chunk
  constexpr int ESIZE = OUT_F32 ? 4 : 2;
  constexpr int CHUNKS_PER_ROW = WN / EPC, CHUNKS = 32 * CHUNKS_PER_ROW, PER_BAND = CHUNKS / 64;
  static_assert(64 % CHUNKS_PER_ROW == 0, "a lane keeps its columns from chunk to chunk");
  // chunk t of a band: row rr0 + t * ROWS_PER_PASS of the band, columns [cc, cc + EPC) for every t
  constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
  const int rr0 = lane / CHUNKS_PER_ROW, cc = (lane % CHUNKS_PER_ROW) * EPC;
  const int64_t col = col0 + cc;
  const bool col_ok = col < p.N;
  // Addresses: a wavefront-uniform 64-bit base per matrix (the sub-tile's first element) plus a
  // 32-bit offset of the lane's first chunk plus a uniform multiple of the row pitch (a sub-tile
  // spans at most 128 rows: the host keeps 128 row pitches below 4 GiB).
  const int rows_left = (int)min((int64_t)(32 * TM), p.M - row0);   // rows of this sub-tile inside C
  char* const c_base = reinterpret_cast<char*>(p.c) + (row0 * p.ldc + col0) * ESIZE;
  const uint32_t c_pitch = (uint32_t)(p.ldc * ESIZE), c_lane = (uint32_t)rr0 * c_pitch + (uint32_t)(cc * ESIZE);
  const char* const r_base = reinterpret_cast<const char*>(p.res) + (row0 * p.ldres + col0) * 2;
  const uint32_t r_pitch = (uint32_t)(p.ldres * 2), r_lane = (uint32_t)rr0 * r_pitch + (uint32_t)(cc * 2);
  // the bias of this lane's columns, once for the whole tile
  float bias_f[EPC];
#pragma unroll
  for (int q = 0; q < EPC; q++) bias_f[q] = 0.f;
  if (p.bias && col_ok) {
#pragma unroll
    for (int q = 0; q < EPC / 2; q++) {
      const uint32_t bb = *reinterpret_cast<const uint32_t*>(p.bias + col + 2 * q);
      bias_f[2 * q] = bf16lo(bb);
      bias_f[2 * q + 1] = bf16hi(bb);
    }
  }
  // FULL: the whole sub-tile lies inside C (wavefront-uniform), no per-chunk predicate.
  auto emit = [&](auto full_c) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_c)::value;
    // WAVE_LOCAL callers have registers to spare: the residual of the whole tile is requested up
    // front, so one memory latency is exposed instead of one per band
    constexpr bool RES_AHEAD = WAVE_LOCAL && !OUT_F32;
    uint4 res_ahead[RES_AHEAD ? TM * PER_BAND : 1];
    if constexpr (RES_AHEAD) {
      if (p.res) {
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int t = 0; t < PER_BAND; t++) {
            const int r = 32 * i + t * ROWS_PER_PASS;   // + rr0: the lane's row inside the sub-tile
            const bool ok = FULL || (r + rr0 < rows_left && col_ok);
            res_ahead[i * PER_BAND + t] =
                ok ? *reinterpret_cast<const uint4*>(r_base + (r_lane + (uint32_t)r * r_pitch)) : make_uint4(0, 0, 0, 0);
          }
      }
    }
#pragma unroll
    for (int i = 0; i < TM; i++) {
      // the band staged before (or the last tile's fragments) has been read; a wavefront's own
      // LDS accesses execute in order, so after the first band only its own order matters
      if (!WAVE_LOCAL || i == 0) __syncthreads();
      else __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int g4 = 0; g4 < 4; g4++)
          *reinterpret_cast<float4*>(stage + cl * ST_STRIDE + 32 * j + 8 * g4 + 4 * h) =
              make_float4(acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]);
      if (!WAVE_LOCAL) __syncthreads();
      else __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int t = 0; t < PER_BAND; t++) {
        const int rr = rr0 + t * ROWS_PER_PASS;
        const int r = 32 * i + t * ROWS_PER_PASS;
        if (!FULL && !(r + rr0 < rows_left && col_ok)) continue;
        float f[EPC];
#pragma unroll
        for (int q = 0; q < EPC / 4; q++) {
          const float4 v = *reinterpret_cast<const float4*>(stage + rr * ST_STRIDE + cc + 4 * q);
          f[4 * q] = v.x; f[4 * q + 1] = v.y; f[4 * q + 2] = v.z; f[4 * q + 3] = v.w;
        }
        if (p.bias) {
#pragma unroll
          for (int q = 0; q < EPC; q++) f[q] += bias_f[q];
        }
        char* const dst_b = c_base + (c_lane + (uint32_t)r * c_pitch);
        if constexpr (OUT_F32) {
          float4* dst = reinterpret_cast<float4*>(dst_b);
          if (p.accumulate) {
            const float4 old = *dst;
            f[0] += old.x; f[1] += old.y; f[2] += old.z; f[3] += old.w;
          }
          *dst = make_float4(f[0], f[1], f[2], f[3]);
        } else {
          if (p.res) {
            uint4 rv;
            if constexpr (RES_AHEAD) rv = res_ahead[i * PER_BAND + t];
            else rv = *reinterpret_cast<const uint4*>(r_base + (r_lane + (uint32_t)r * r_pitch));
            f[0] += bf16lo(rv.x); f[1] += bf16hi(rv.x); f[2] += bf16lo(rv.y); f[3] += bf16hi(rv.y);
            f[4] += bf16lo(rv.z); f[5] += bf16hi(rv.z); f[6] += bf16lo(rv.w); f[7] += bf16hi(rv.w);
          }
          *reinterpret_cast<uint4*>(dst_b) =
              make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
        }
      }
    }
  };
  if (rows_left >= 32 * TM && col0 + WN <= p.N) emit(std::true_type{});
  else emit(std::false_type{});
}

// Rotary positions on a wavefront's 32*TM x 128 sub-tile while it is still in the accumulators
// (rows from row0, columns from col0, a multiple of 128, so the sub-tile holds whole heads of HD =
// 128 or 64).  A lane owns row lane%32 of every band, so the row's position and its angles are the
// lane's own, and the half-split partner of column c, c + HD/2, lies HD/64 accumulator blocks
// further in the same lane: the rotation needs no exchange.  With a bias the rotation applies to
// x.W + b, so the bias is added here (the caller then stores without it).  Sub-tiles past
// rope_cols (the v columns) are left alone; the branch is wavefront-uniform.
template <int TM, int HD>
__device__ __forceinline__ bool rope_rotate_tile(const GemmParams& p, f32x16 (&acc)[TM][4], int64_t row0,
                                                 int64_t col0, int lane) {
  static_assert(HD == 128 || HD == 64, "heads of 64 or 128");
  if (col0 >= p.rope_cols) return false;
  constexpr int HALF = HD / 2, STEP = HD / 64;      // partner block = block + STEP
  const int h = lane >> 5, cl = lane & 31;
  if (p.bias) {
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++) {
        const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + col0 + 32 * j + 8 * g4 + 4 * h);
        const float b0 = bf16lo(bb.x), b1 = bf16hi(bb.x), b2 = bf16lo(bb.y), b3 = bf16hi(bb.y);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][j][4 * g4] += b0; acc[i][j][4 * g4 + 1] += b1; acc[i][j][4 * g4 + 2] += b2; acc[i][j][4 * g4 + 3] += b3;
        }
      }
  }
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int64_t row = row0 + 32 * i + cl;
    const int pos = row < p.M ? p.rope_pos[row] : 0;
    const float* trow = p.rope_table + (int64_t)pos * HD;
#pragma unroll
    for (int jj = 0; jj < 2; jj++) {
      // HD = 128: blocks (0, 2) and (1, 3), frequencies 32 jj + ...; HD = 64: blocks (0, 1) and (2, 3), two heads
      const int j1 = HD == 128 ? jj : 2 * jj, j2 = j1 + STEP;
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++) {
        const int f0 = (HD == 128 ? 32 * jj : 0) + 8 * g4 + 4 * h;
        const float4 c = *reinterpret_cast<const float4*>(trow + f0);
        const float4 sn = *reinterpret_cast<const float4*>(trow + HALF + f0);
        const float cs[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const float x1 = acc[i][j1][4 * g4 + e], x2 = acc[i][j2][4 * g4 + e];
          acc[i][j1][4 * g4 + e] = x1 * cs[e] - x2 * ss[e];
          acc[i][j2][4 * g4 + e] = x2 * cs[e] + x1 * ss[e];
        }
      }
    }
  }
  return true;
}

// Epilogue of the fused SwiGLU product.  The wavefront's 32*TM x 128 sub-tile holds 64 gate
// columns (accumulator blocks 0, 1) and the 64 up columns of the same indices (blocks 2, 3):
// columns gcol0 .. gcol0 + 63 of gate and of up.  Each band of 32 rows is staged through LDS
// like in store_tile; a lane then takes a gate chunk of 8 columns and its up chunk of the same
// row and writes three 16-byte pieces: gate and up into C = [gate | up] ([M, N], up at column
// N / 2 + gcol) and silu(gate) * up into act ([M, N / 2]).  The sub-tile's columns all exist
// (N / 2 is a multiple of 128); rows past M are skipped.
template <int TM>
__device__ __forceinline__ void store_tile_swiglu(const GemmParams& p, f32x16 (&acc)[TM][4], float* stage,
                                                  int64_t row0, int64_t gcol0, int lane) {
  constexpr int ST_STRIDE = 128 + 4;
  const int h = lane >> 5, cl = lane & 31;
  const int rr0 = lane >> 3, cc = (lane & 7) * 8;          // 8 rows per pass, 8 gate chunks per row
  const int64_t half = p.N >> 1;
  const int rows_left = (int)min((int64_t)(32 * TM), p.M - row0);
  char* const c_base = reinterpret_cast<char*>(p.c) + (row0 * p.ldc + gcol0) * 2;
  char* const a_base = reinterpret_cast<char*>(p.act) + (row0 * half + gcol0) * 2;
  const uint32_t c_pitch = (uint32_t)(p.ldc * 2), a_pitch = (uint32_t)(half * 2);
  const uint32_t up_off = (uint32_t)(half * 2);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    if (i == 0) __syncthreads();
    else __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++)
        *reinterpret_cast<float4*>(stage + cl * ST_STRIDE + 32 * j + 8 * g4 + 4 * h) =
            make_float4(acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int t = 0; t < 4; t++) {
      const int rr = rr0 + 8 * t, r = 32 * i + rr;
      if (r >= rows_left) continue;
      float g[8], u[8], a[8];
#pragma unroll
      for (int q = 0; q < 2; q++) {
        const float4 vg = *reinterpret_cast<const float4*>(stage + rr * ST_STRIDE + cc + 4 * q);
        const float4 vu = *reinterpret_cast<const float4*>(stage + rr * ST_STRIDE + 64 + cc + 4 * q);
        g[4 * q] = vg.x; g[4 * q + 1] = vg.y; g[4 * q + 2] = vg.z; g[4 * q + 3] = vg.w;
        u[4 * q] = vu.x; u[4 * q + 1] = vu.y; u[4 * q + 2] = vu.z; u[4 * q + 3] = vu.w;
      }
#pragma unroll
      for (int e = 0; e < 8; e++)   // silu through the hardware exp2 and reciprocal (1 ulp each; the result is rounded to bf16)
        a[e] = g[e] * u[e] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(g[e] * -1.44269504088896340736f));
      char* const dst = c_base + ((uint32_t)r * c_pitch + (uint32_t)(cc * 2));
      *reinterpret_cast<uint4*>(dst) = make_uint4(pack_bf16x2(g[0], g[1]), pack_bf16x2(g[2], g[3]),
                                                  pack_bf16x2(g[4], g[5]), pack_bf16x2(g[6], g[7]));
      *reinterpret_cast<uint4*>(dst + up_off) = make_uint4(pack_bf16x2(u[0], u[1]), pack_bf16x2(u[2], u[3]),
                                                           pack_bf16x2(u[4], u[5]), pack_bf16x2(u[6], u[7]));
      *reinterpret_cast<uint4*>(a_base + ((uint32_t)r * a_pitch + (uint32_t)(cc * 2))) =
          make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
    }
  }
}

// Epilogue of dA = dY.W_d^T with SwiGLU's gradient: the sub-tile of dA (32*TM x 128, columns from
// col0) never reaches memory.  Band by band it is staged through LDS like in store_tile; a lane
// takes a chunk of 8 columns of dA, the gate and up chunks of the same row and columns from
// pre = [gate | up] ([M, 2N], requested for the whole band before the staging), and writes
//   d gate = dA * up * s * (1 + gate * (1 - s)),  d up = dA * gate * s,  s = sigmoid(gate)
// to dpre = [d gate | d up] ([M, 2N]).  Rows past M and columns past N are skipped.
template <int TM>
__device__ __forceinline__ void store_tile_swiglu_bwd(const GemmParams& p, f32x16 (&acc)[TM][4], float* stage,
                                                      int64_t row0, int64_t col0, int lane) {
  constexpr int ST_STRIDE = 128 + 4, PER_BAND = 8, ROWS_PER_PASS = 4;
  const int h = lane >> 5, cl = lane & 31;
  const int rr0 = lane >> 4, cc = (lane & 15) * 8;
  const bool col_ok = col0 + cc < p.N;
  const int rows_left = (int)min((int64_t)(32 * TM), p.M - row0);
  const uint32_t pitch = (uint32_t)(p.N * 4), up_off = (uint32_t)(p.N * 2);   // bytes: a row of [M, 2N] bf16; the up half
  const char* const pre_base = reinterpret_cast<const char*>(p.pre) + (row0 * 2 * p.N + col0) * 2;
  char* const dpre_base = reinterpret_cast<char*>(p.dpre) + (row0 * 2 * p.N + col0) * 2;
  const uint32_t lane_off = (uint32_t)rr0 * pitch + (uint32_t)(cc * 2);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    uint4 gq[PER_BAND], uq[PER_BAND];
#pragma unroll
    for (int t = 0; t < PER_BAND; t++) {
      const int r = 32 * i + t * ROWS_PER_PASS;
      const bool ok = r + rr0 < rows_left && col_ok;
      const char* src = pre_base + (lane_off + (uint32_t)r * pitch);
      gq[t] = ok ? *reinterpret_cast<const uint4*>(src) : make_uint4(0, 0, 0, 0);
      uq[t] = ok ? *reinterpret_cast<const uint4*>(src + up_off) : make_uint4(0, 0, 0, 0);
    }
    if (i == 0) __syncthreads();
    else __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++)
        *reinterpret_cast<float4*>(stage + cl * ST_STRIDE + 32 * j + 8 * g4 + 4 * h) =
            make_float4(acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int t = 0; t < PER_BAND; t++) {
      const int rr = rr0 + t * ROWS_PER_PASS, r = 32 * i + t * ROWS_PER_PASS;
      if (!(r + rr0 < rows_left && col_ok)) continue;
      float d[8], g[8], u[8], og[8], ou[8];
#pragma unroll
      for (int q = 0; q < 2; q++) {
        const float4 v = *reinterpret_cast<const float4*>(stage + rr * ST_STRIDE + cc + 4 * q);
        d[4 * q] = v.x; d[4 * q + 1] = v.y; d[4 * q + 2] = v.z; d[4 * q + 3] = v.w;
      }
      g[0] = bf16lo(gq[t].x); g[1] = bf16hi(gq[t].x); g[2] = bf16lo(gq[t].y); g[3] = bf16hi(gq[t].y);
      g[4] = bf16lo(gq[t].z); g[5] = bf16hi(gq[t].z); g[6] = bf16lo(gq[t].w); g[7] = bf16hi(gq[t].w);
      u[0] = bf16lo(uq[t].x); u[1] = bf16hi(uq[t].x); u[2] = bf16lo(uq[t].y); u[3] = bf16hi(uq[t].y);
      u[4] = bf16lo(uq[t].z); u[5] = bf16hi(uq[t].z); u[6] = bf16lo(uq[t].w); u[7] = bf16hi(uq[t].w);
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float s = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(g[e] * -1.44269504088896340736f));
        const float gs = g[e] * s;
        og[e] = d[e] * u[e] * (s + gs * (1.f - s));
        ou[e] = d[e] * gs;
      }
      char* const dst = dpre_base + (lane_off + (uint32_t)r * pitch);
      *reinterpret_cast<uint4*>(dst) = make_uint4(pack_bf16x2(og[0], og[1]), pack_bf16x2(og[2], og[3]),
                                                  pack_bf16x2(og[4], og[5]), pack_bf16x2(og[6], og[7]));
      *reinterpret_cast<uint4*>(dst + up_off) = make_uint4(pack_bf16x2(ou[0], ou[1]), pack_bf16x2(ou[2], ou[3]),
                                                           pack_bf16x2(ou[4], ou[5]), pack_bf16x2(ou[6], ou[7]));
    }
  }
}

}  // namespace mllm
