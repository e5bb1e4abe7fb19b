// bf16 MFMA GEMM for gfx950: C[M,N] = op(A) . op(B) (+ bias) (+ residual), fp32 accumulate.
//
// These are the linear operations of the stage, applied to the whole packed sequence at once
// (Model Profiler, "Throughput Profiling"): QKV / output / MLP projections and the connector,
// their input gradients (dX = dY.W^T) and their weight gradients (dW = X^T.dY).
//
// Layout handling.  v_mfma_f32_32x32x16_bf16 wants, per lane, eight consecutive values along
// the contraction index.  Operands whose contraction index is contiguous in memory are staged
// in LDS as [row][k] and fetched with one 16-byte read; operands whose contraction index is the
// strided one (W in Y = X.W, both operands of dW = X^T.dY) are staged as they lie in memory,
// [k][row], and fetched with the LDS transposing read (two ds_read_b64_tr_b16 per fragment), so
// no operand is ever transposed in global memory or in registers.
//
// Tiling.  One workgroup computes a BM x BN tile with NW = (BM/WM)*(BN/WN) wavefronts, each
// owning a WM x WN sub-tile of 32x32 MFMA blocks.  The K loop moves BK = 64 at a time:
// global -> registers (prefetch of the next tile, issued before the MFMAs of the current one)
// -> LDS.  Tiles are visited in an order that keeps the workgroups resident on one XCD (they
// share that XCD's L2) on neighbouring tiles of a GROUP_M-tall panel.
#include "common.h"
#include "kernels.h"

namespace mllm {

namespace {

constexpr int BK = 64;
constexpr int PAD = 8;  // elements; keeps 16-byte alignment and staggers LDS banks

template <int ROWS, int COLS, int NT>
struct TileLoader {
  static constexpr int VEC_PER_ROW = COLS / 8;
  static constexpr int NVEC = ROWS * COLS / 8;
  static constexpr int PER_THREAD = NVEC / NT;
  static_assert(NVEC % NT == 0, "tile must divide among threads");
  uint4 r[PER_THREAD];

  __device__ __forceinline__ void load(const bf16_t* __restrict__ g, int64_t ld, int64_t row0,
                                       int64_t col0, int64_t nrows, int64_t ncols, int tid) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; i++) {
      int v = tid + i * NT;
      int rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
      int64_t gr = row0 + rr, gc = col0 + cc;
      if (gr < nrows && gc < ncols) {
        r[i] = *reinterpret_cast<const uint4*>(g + gr * ld + gc);
      } else {
        r[i] = make_uint4(0, 0, 0, 0);
      }
    }
  }
  __device__ __forceinline__ void store(bf16_t* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < PER_THREAD; i++) {
      int v = tid + i * NT;
      int rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
      *reinterpret_cast<uint4*>(lds + rr * (COLS + PAD) + cc) = r[i];
    }
  }
};

// Fragment of 8 contraction values for row (r0 + lane%32), k = kk*16 + 8*(lane/32) ...
template <bool TRANSPOSED, int STRIDE>
__device__ __forceinline__ bf16x8 fetch_frag(const bf16_t* tile, int r0, int kk, int lane) {
  Frag8 f;
  const int h = lane >> 5;
  if constexpr (!TRANSPOSED) {
    f.u = *reinterpret_cast<const uint4*>(tile + (r0 + (lane & 31)) * STRIDE + kk * 16 + 8 * h);
  } else {
    const int n0 = r0 + 16 * ((lane >> 4) & 1);
    f.h[0] = lds_read_tr4(tile, STRIDE, kk * 16 + 8 * h, n0, lane & 15);
    f.h[1] = lds_read_tr4(tile, STRIDE, kk * 16 + 8 * h + 4, n0, lane & 15);
  }
  return f.v;
}

struct GemmParams {
  const bf16_t* a;
  const bf16_t* b;
  void* c;
  const bf16_t* bias;
  const bf16_t* res;
  int64_t M, N, K, lda, ldb, ldc, ldres;
  int accumulate;
  int tiles_m, tiles_n;
};

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

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T, bool OUT_F32>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_kernel(GemmParams p) {
  constexpr int NWM = BM / WM, NWN = BN / WN, NT = 64 * NWM * NWN;
  constexpr int TM = WM / 32, TN = WN / 32;
  // A tile: [BM][BK] (contraction contiguous) or [BK][BM] (as stored, transposing reads)
  constexpr int A_ROWS = A_T ? BK : BM, A_COLS = A_T ? BM : BK;
  constexpr int B_ROWS = B_T ? BK : BN, B_COLS = B_T ? BN : BK;
  constexpr int A_STRIDE = A_COLS + PAD, B_STRIDE = B_COLS + PAD;
  __shared__ __attribute__((aligned(16))) bf16_t As[A_ROWS * A_STRIDE];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[B_ROWS * B_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  TileLoader<A_ROWS, A_COLS, NT> la;
  TileLoader<B_ROWS, B_COLS, NT> lb;
  auto gload = [&](int64_t k0) {
    if constexpr (A_T) la.load(p.a, p.lda, k0, m0, p.K, p.M, tid);
    else la.load(p.a, p.lda, m0, k0, p.M, p.K, tid);
    if constexpr (B_T) lb.load(p.b, p.ldb, k0, n0, p.K, p.N, tid);
    else lb.load(p.b, p.ldb, n0, k0, p.N, p.K, tid);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  const int nk = (int)((p.K + BK - 1) / BK);
  gload(0);
  la.store(As, tid);
  lb.store(Bs, tid);
  __syncthreads();
  for (int kt = 0; kt < nk; kt++) {
    if (kt + 1 < nk) gload((int64_t)(kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; i++) af[i] = fetch_frag<A_T, A_STRIDE>(As, wm * WM + 32 * i, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; j++) bfr[j] = fetch_frag<B_T, B_STRIDE>(Bs, wn * WN + 32 * j, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
    if (kt + 1 < nk) {
      la.store(As, tid);
      lb.store(Bs, tid);
      __syncthreads();
    }
  }

  // Epilogue: acc[v] of a 32x32 block is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
  const int h = lane >> 5, cl = lane & 31;
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int64_t col = n0 + wn * WN + 32 * j + cl;
    if (col >= p.N) continue;
    const float bias = p.bias ? bf16_to_f32(p.bias[col]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; i++) {
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int64_t row = m0 + wm * WM + 32 * i + 8 * (v >> 2) + 4 * h + (v & 3);
        if (row >= p.M) continue;
        float val = acc[i][j][v] + bias;
        if constexpr (OUT_F32) {
          float* c = reinterpret_cast<float*>(p.c) + row * p.ldc + col;
          if (p.accumulate) val += *c;
          *c = val;
        } else {
          if (p.res) val += bf16_to_f32(p.res[row * p.ldres + col]);
          reinterpret_cast<bf16_t*>(p.c)[row * p.ldc + col] = f32_to_bf16(val);
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_tile(const GemmArgs& g, hipStream_t s) {
  GemmParams p;
  p.a = (const bf16_t*)g.a; p.b = (const bf16_t*)g.b; p.c = g.c;
  p.bias = (const bf16_t*)g.bias; p.res = (const bf16_t*)g.residual;
  p.M = g.m; p.N = g.n; p.K = g.k; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldres = g.ldres;
  p.accumulate = g.accumulate;
  p.tiles_m = (int)((g.m + BM - 1) / BM);
  p.tiles_n = (int)((g.n + BN - 1) / BN);
  dim3 grid((unsigned)(p.tiles_m * p.tiles_n)), block(64 * (BM / WM) * (BN / WN));
  const bool at = g.a_layout != 0, bt = g.b_layout == 0;  // b_layout 0 = [K,N] = transposing reads
#define MLLM_GEMM_CASE(AT, BT, F32)                                                      \
  if (at == AT && bt == BT && (g.out_fp32 != 0) == F32) {                                \
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, AT, BT, F32>), grid, block, 0, s, p); \
    return hipGetLastError();                                                            \
  }
  MLLM_GEMM_CASE(false, true, false)   // Y = X.W
  MLLM_GEMM_CASE(false, false, false)  // dX = dY.W^T (W stored [K_out.., ] as [N,K])
  MLLM_GEMM_CASE(true, true, true)     // dW = X^T.dY, fp32
  MLLM_GEMM_CASE(false, true, true)
  MLLM_GEMM_CASE(false, false, true)
  MLLM_GEMM_CASE(true, true, false)
  MLLM_GEMM_CASE(true, false, false)
  MLLM_GEMM_CASE(true, false, true)
#undef MLLM_GEMM_CASE
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.m <= 0 || g.n <= 0) return hipSuccess;
  const int cls = g.a_layout ? PROF_GEMM_DW : (g.b_layout ? PROF_GEMM_DX : PROF_GEMM_FWD);
  ProfScope prof(cls, 2.0 * (double)g.m * (double)g.n * (double)g.k, s);
  return launch_tile<128, 128, 64, 64>(g, s);
}

}  // namespace mllm
