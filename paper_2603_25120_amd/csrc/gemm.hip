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
//
// Two kernels.  gemm4_kernel: 256x256 tiles on four wavefronts of 128x128 with a hand-placed
// k-loop, for every problem that fills the chip with such tiles and whose K is a multiple of 64
// (also with 192x256 tiles, when those need fewer rounds of one-per-CU workgroups).
// gemm_kernel: the general template (128x128 tiles on four wavefronts of 64x64 for small
// problems, 256x256 tiles on eight wavefronts of 128x64 when K has a ragged tail).
#include <algorithm>
#include <utility>

#include "gemm_common.h"

namespace mllm {

namespace {

// Row padding (elements).  LDS has 64 banks of 4 bytes.  k-contiguous tiles: rows 144 B apart put
// the 16-byte reads of any 16 consecutive rows on distinct banks.  Tiles read with the transposing
// load: 32 lanes of one read touch 4 rows x 64 B, so the row stride must be 16 dwords mod 64
// (576 B for 256 columns, 320 B for 128): the four rows then fill the 64 banks exactly (measured:
// no bank-conflict cycles in any layout).
constexpr int PAD_K = 8;
constexpr int PAD_T = 32;

// Global -> register -> LDS staging of one operand tile through buffer loads: an out-of-range
// offset returns zeros, so ragged edges need no branches.  K_ROWS: the tile's rows run along the
// contraction index (operand stored [K, rows]); otherwise its columns do (stored [rows, K]).
template <int ROWS, int COLS, int PADC, int NT, bool K_ROWS, int BKT>
struct TileLoader {
  static constexpr int VEC_PER_ROW = COLS / 8;
  static constexpr int NVEC = ROWS * COLS / 8;
  static constexpr int PER_THREAD = NVEC / NT;
  static constexpr int STRIDE = COLS + PADC;
  static_assert(NVEC % NT == 0 && NT % VEC_PER_ROW == 0, "tile must divide among threads");
  u32x4 r[PER_THREAD];
  uint32_t off[PER_THREAD];   // byte offset of this thread's vectors at k0 = 0, OOB if never valid
  int klim[PER_THREAD];       // vector i is inside the matrix while k0 < klim[i]
  uint32_t kstep;             // bytes per BK step

  __device__ __forceinline__ void init(int64_t ld, int64_t fixed0, int64_t nfixed, int64_t K, int tid) {
    kstep = (uint32_t)(K_ROWS ? BKT * ld * 2 : BKT * 2);
#pragma unroll
    for (int i = 0; i < PER_THREAD; i++) {
      const int v = tid + i * NT, rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
      const int64_t fx = fixed0 + (K_ROWS ? cc : rr);
      const int64_t lin = K_ROWS ? (int64_t)rr * ld + fx : fx * ld + cc;
      off[i] = fx < nfixed ? (uint32_t)(lin * 2) : OOB;
      klim[i] = (int)(K - (K_ROWS ? rr : cc));
    }
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, int kt) { load_part<0, PER_THREAD>(rsrc, kt); }
  __device__ __forceinline__ void store(bf16_t* lds, int tid) const { store_part<0, PER_THREAD>(lds, tid); }
  template <int I0, int I1>
  __device__ __forceinline__ void load_part(__amdgpu_buffer_rsrc_t rsrc, int kt) {
    const int k0 = kt * BKT;
#pragma unroll
    for (int i = I0; i < I1; i++) {
      const uint32_t o = (off[i] != OOB && k0 < klim[i]) ? off[i] + (uint32_t)kt * kstep : OOB;
      r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)o, 0, 0);
    }
  }
  template <int I0, int I1>
  __device__ __forceinline__ void store_part(bf16_t* lds, int tid) const {
#pragma unroll
    for (int i = I0; i < I1; i++) {
      const int v = tid + i * NT, rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
      *reinterpret_cast<u32x4*>(lds + rr * STRIDE + cc) = r[i];
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

// Scheduling pattern of one k-step: MFMA slot M is preceded by up to PER LDS reads while any
// of the N_READS remain.
template <int PER, int N_READS, int M>
__device__ __forceinline__ void interleave_slot() {
  if constexpr (M * PER < N_READS)
    __builtin_amdgcn_sched_group_barrier(0x100, (M + 1) * PER <= N_READS ? PER : N_READS - M * PER, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
}
template <int PER, int N_READS, int... Ms>
__device__ __forceinline__ void interleave_reads(std::integer_sequence<int, Ms...>) {
  (interleave_slot<PER, N_READS, Ms>(), ...);
}

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T, bool OUT_F32, int BKT>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_kernel(GemmParams p) {
  constexpr int NWM = BM / WM, NWN = BN / WN, NT = 64 * NWM * NWN;
  constexpr int TM = WM / 32, TN = WN / 32;
  // A tile: [BM][BK] (contraction contiguous) or [BK][BM] (as stored, transposing reads)
  constexpr int A_ROWS = A_T ? BKT : BM, A_COLS = A_T ? BM : BKT, A_PAD = A_T ? PAD_T : PAD_K;
  constexpr int B_ROWS = B_T ? BKT : BN, B_COLS = B_T ? BN : BKT, B_PAD = B_T ? PAD_T : PAD_K;
  constexpr int A_STRIDE = A_COLS + A_PAD, B_STRIDE = B_COLS + B_PAD;
  constexpr int A_SIZE = A_ROWS * A_STRIDE, B_SIZE = B_ROWS * B_STRIDE;
  // two LDS stages: tile kt+1 is written while tile kt is being multiplied
  __shared__ __attribute__((aligned(16))) bf16_t As[2 * A_SIZE];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2 * B_SIZE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  TileLoader<A_ROWS, A_COLS, A_PAD, NT, A_T, BKT> la;
  TileLoader<B_ROWS, B_COLS, B_PAD, NT, B_T, BKT> lb;
  la.init(p.lda, m0, p.M, p.K, tid);
  lb.init(p.ldb, n0, p.N, p.K, tid);
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(p.a, p.a_bytes), rb = make_rsrc(p.b, p.b_bytes);
  auto gload = [&](int kt) {
    la.load(ra, kt);
    lb.load(rb, kt);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // Split-K: workgroup row blockIdx.y owns k-tiles [kt0, kt0 + nk) and writes its own partial C.
  const int kt0 = blockIdx.y * p.kt_per_split;
  const int nk = min(p.kt_per_split, (int)((p.K + BKT - 1) / BKT) - kt0);
  gload(kt0);
  la.store(As, tid);
  lb.store(Bs, tid);
  gload(kt0 + 1);
  __syncthreads();

  // Fragments are double-buffered in registers: those of step kk+1 are fetched from LDS while
  // the 16 MFMAs of step kk run; step 0 of the next tile is fetched right after the barrier.
  bf16x8 af[2][TM], bfr[2][TN];
  auto fetch = [&](int buf, const bf16_t* at, const bf16_t* bt, int kk) {
#pragma unroll
    for (int i = 0; i < TM; i++) af[buf][i] = fetch_frag<A_T, A_STRIDE>(at, wm * WM + 32 * i, kk, lane);
#pragma unroll
    for (int j = 0; j < TN; j++) bfr[buf][j] = fetch_frag<B_T, B_STRIDE>(bt, wn * WN + 32 * j, kk, lane);
  };
  fetch(0, As, Bs, 0);
  constexpr int STEPS = BKT / 16;
  using LA = TileLoader<A_ROWS, A_COLS, A_PAD, NT, A_T, BKT>;
  using LB = TileLoader<B_ROWS, B_COLS, B_PAD, NT, B_T, BKT>;
  // EARLY (four k-steps per tile): the tile is moved in the first half of the k-steps and the
  // barrier sits before the last step's MFMAs, so the next tile's first fragments are fetched
  // under them.  Otherwise the move is spread over all k-steps and the barrier closes the
  // iteration.
  constexpr bool EARLY = STEPS == 4;
  constexpr int MOVE_STEPS = EARLY ? STEPS / 2 : STEPS;
  constexpr int A_PER = LA::PER_THREAD / MOVE_STEPS, B_PER = LB::PER_THREAD / MOVE_STEPS;
  static_assert(A_PER * MOVE_STEPS == LA::PER_THREAD && B_PER * MOVE_STEPS == LB::PER_THREAD && A_PER >= 1 && B_PER >= 1,
                "the moving k-steps must split the tile evenly");
  static_assert(STEPS == 2 || STEPS == 4, "two or four k-steps per tile");
  for (int kt = 0; kt < nk; kt++) {
    const int cur = kt & 1;
    bf16_t* an = As + (cur ^ 1) * A_SIZE;
    bf16_t* bn = Bs + (cur ^ 1) * B_SIZE;
    const bf16_t* at = As + cur * A_SIZE;
    const bf16_t* bt = Bs + cur * B_SIZE;
    // Branch-free body.  The moving k-steps each put a share of tile kt+1 from the staging
    // registers into the other LDS stage and at once refill those registers with the same share
    // of tile kt+2 (every prefetch has a whole iteration to land); every step but the last
    // fetches the next step's fragments before issuing its MFMAs.  With EARLY the barrier comes
    // before the last step's MFMAs: by then every fragment of this stage is in registers and
    // every store to the other stage has been issued.  Past the end the prefetch offsets are out
    // of range (zeros, no traffic) and the stored stage is never read.
    auto step = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      if constexpr (kk < MOVE_STEPS) {
        la.template store_part<kk * A_PER, (kk + 1) * A_PER>(an, tid);
        lb.template store_part<kk * B_PER, (kk + 1) * B_PER>(bn, tid);
        la.template load_part<kk * A_PER, (kk + 1) * A_PER>(ra, kt0 + kt + 2);
        lb.template load_part<kk * B_PER, (kk + 1) * B_PER>(rb, kt0 + kt + 2);
      }
      if constexpr (kk + 1 < STEPS) {
        fetch((kk + 1) & 1, at, bt, kk + 1);
      } else if constexpr (EARLY) {
        __syncthreads();
        fetch(0, an, bn, 0);
      }
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
      // Issue order inside the step: the LDS reads of the next fragments go out one per MFMA from
      // the step's start (left alone, the scheduler puts them after the MFMAs and the wavefront
      // then waits on LDS with nothing queued behind it).
      if constexpr (kk + 1 < STEPS || EARLY) {
        constexpr int N_READS = TM * (A_T ? 2 : 1) + TN * (B_T ? 2 : 1), N_MFMA = TM * TN;
        constexpr int PER = (N_READS + N_MFMA - 1) / N_MFMA;     // reads per MFMA slot
        interleave_reads<PER, N_READS>(std::make_integer_sequence<int, N_MFMA>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    if constexpr (STEPS == 4) {
      step(std::integral_constant<int, 2>{});
      step(std::integral_constant<int, 3>{});
    }
    if constexpr (!EARLY) {
      __syncthreads();
      fetch(0, an, bn, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  constexpr int ST_STRIDE = WN + 4;  // floats
  static_assert(NWM * NWN * 32 * ST_STRIDE * 4 <= 2 * A_SIZE * 2, "staging must fit in the A stages");
  if constexpr (OUT_F32) p.c = reinterpret_cast<float*>(p.c) + blockIdx.y * p.c_split_stride;
  store_tile<TM, TN, OUT_F32>(p, acc, reinterpret_cast<float*>(As) + wave * 32 * ST_STRIDE,
                              m0 + wm * WM, n0 + wn * WN, lane);
}

// ---------------------------------------------------------------------------------------------
// 256x256x64 tiles on four wavefronts (one per SIMD), each owning 128x128 = 4x4 MFMA blocks with
// the accumulators in AGPRs: a third fewer LDS fragment reads per MFMA than 128x64 sub-tiles.
// With a single wavefront per SIMD nothing else hides a stall, so the k-loop is written slot by
// slot: every MFMA slot names the LDS read, LDS store and global load that issue in front of it and
// a scheduling barrier after every slot keeps that order.  Two sets of staging registers: a
// global load has two whole iterations to land.  The k-advance of the global loads is a scalar
// offset (no per-load address arithmetic), clamped to the last tile so that no address leaves the
// operand; that needs K to be a multiple of 64, except in the ragged-K form for operands stored
// [K, .], which sends the last tile's advance through the range-checked lane offsets.
template <class F, int... Is>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  for_each_index(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

template <int ROWS, int COLS, int PADC, int NT, bool K_ROWS>
struct ScalarStepLoader {
  static constexpr int VEC_PER_ROW = COLS / 8;
  static constexpr int NVEC = ROWS * COLS / 8;
  static constexpr int PER_THREAD = NVEC / NT;
  static constexpr int STRIDE = COLS + PADC;
  static_assert(NVEC % NT == 0 && NT % VEC_PER_ROW == 0, "tile must divide among threads");
  u32x4 r[2][PER_THREAD];
  uint32_t off[PER_THREAD];   // byte offset of this thread's vectors in k-tile 0, OOB if never valid
  uint32_t kstep;             // bytes per k-tile

  // pair_half > 0 (operands stored [K, N] only): the tile's 256 columns are, in blocks of 64,
  // columns [c, c + 64) of the left half of the matrix, the same columns of the right half
  // (+ pair_half), then [c + 64, c + 128) of the left half and of the right half, with
  // c = fixed0 / 2: each wavefront's 128 columns then hold matching gate and up columns.
  __device__ __forceinline__ void init(int64_t ld, int64_t fixed0, int64_t nfixed, int tid, int64_t pair_half = 0) {
    kstep = (uint32_t)(K_ROWS ? BK * ld * 2 : BK * 2);
#pragma unroll
    for (int i = 0; i < PER_THREAD; i++) {
      const int v = tid + i * NT, rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
      int64_t fx = fixed0 + (K_ROWS ? cc : rr);
      if (K_ROWS && pair_half > 0) {
        const int blk = cc >> 6;
        fx = (blk & 1) * pair_half + (fixed0 >> 1) + 64 * (blk >> 1) + (cc & 63);
      }
      const int64_t lin = K_ROWS ? (int64_t)rr * ld + fx : fx * ld + cc;
      off[i] = fx < nfixed ? (uint32_t)(lin * 2) : OOB;
    }
  }
  template <int S, int I>
  __device__ __forceinline__ void load1(__amdgpu_buffer_rsrc_t rsrc, uint32_t soff) {
    r[S][I] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off[I], (int)soff, 0);
  }
  // The same with part of the k-advance in the lane's own offset, which the buffer's range check
  // sees (the scalar offset it does not): rows past the operand's end then read as zeros.
  template <int S, int I>
  __device__ __forceinline__ void load1_checked(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_adv, uint32_t soff) {
    uint32_t v = off[I] + lane_adv;
    v = v < lane_adv ? OOB : v;   // an offset that is OOB already stays so instead of wrapping
    r[S][I] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)v, (int)soff, 0);
  }
  template <int S, int I>
  __device__ __forceinline__ void store1(bf16_t* lds, int tid) const {
    const int v = tid + I * NT, rr = v / VEC_PER_ROW, cc = (v % VEC_PER_ROW) * 8;
    *reinterpret_cast<u32x4*>(lds + rr * STRIDE + cc) = r[S][I];
  }
};

// k-advance of the loads of k-tile t: all of it in the scalar offset, except (RAGGED_K) for the
// last, partial k-tile, where it goes through the lanes' offsets so that the range check applies.
struct KAdvance { uint32_t lane, scalar; };
template <bool RAGGED_K>
__device__ __forceinline__ KAdvance k_advance(uint32_t t, uint32_t last_tile, uint32_t kstep) {
  if (RAGGED_K && t == last_tile) return {t * kstep, 0u};
  return {0u, t * kstep};
}

// EPI: 0 plain epilogue; 1 SwiGLU forward fused; 2 SwiGLU gradient fused; 3 / 4 rotary positions
// fused for heads of 128 / 64.
template <int TM, bool A_T, bool B_T, bool OUT_F32, bool RAGGED_K, int EPI = 0>
__device__ __forceinline__ void gemm4_tile(GemmParams p) {
  constexpr bool SWIGLU = EPI == 1;
  // TM = 4: 256x256 tiles, wavefronts of 128x128.  TM = 3: 192x256 tiles, wavefronts of 96x128,
  // for problems whose 256-row tiles would leave the last round of workgroups mostly empty.
  static_assert(TM == 4 || (TM == 3 && !A_T), "192-row tiles only for an A operand stored [M, K]");
  // RAGGED_K: K need not be a multiple of 64.  Only when k runs along the rows of both operands:
  // the rows of the last k-tile that lie past K are then past the end of the operand.
  static_assert(!RAGGED_K || (A_T && B_T), "a ragged K needs both operands stored [K, .]");
  // SWIGLU: C = [gate | up]; the epilogue also writes silu(gate) * up (forward layout only).
  static_assert(!SWIGLU || (TM == 4 && !A_T && B_T && !OUT_F32), "fused SwiGLU: Y = X.W with W stored [K, N], bf16");
  static_assert(EPI != 2 || (TM == 4 && !A_T && !B_T && !OUT_F32), "fused SwiGLU gradient: dA = dY.W^T with W stored [N, K], bf16");
  static_assert((EPI != 3 && EPI != 4) || (TM == 4 && !A_T && B_T && !OUT_F32), "fused rotary positions: Y = X.W with W stored [K, N], bf16");
  constexpr int BM = 64 * TM, BN = 256, WM = 32 * TM, WN = 128, NT = 256, TN = 4;
  constexpr int NA = 2 * TM;          // A vectors per thread and k-tile (B: 8)
  constexpr int NU = TM + 4;          // fragment units per k-step
  constexpr int NS = 4 * TM;          // MFMA slots per k-step
  constexpr int Q3 = TM == 4 ? 4 : 3; // vectors moved in the last k-step (into the tile's own stage)
  constexpr int A_ROWS = A_T ? BK : BM, A_COLS = A_T ? BM : BK, A_PAD = A_T ? PAD_T : PAD_K;
  constexpr int B_ROWS = B_T ? BK : BN, B_COLS = B_T ? BN : BK, B_PAD = B_T ? PAD_T : PAD_K;
  constexpr int A_STRIDE = A_COLS + A_PAD, B_STRIDE = B_COLS + B_PAD;
  constexpr int A_SIZE = A_ROWS * A_STRIDE, B_SIZE = B_ROWS * B_STRIDE;
  __shared__ __attribute__((aligned(16))) bf16_t As[2 * A_SIZE];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2 * B_SIZE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  using LA = ScalarStepLoader<A_ROWS, A_COLS, A_PAD, NT, A_T>;
  using LB = ScalarStepLoader<B_ROWS, B_COLS, B_PAD, NT, B_T>;
  static_assert(LA::PER_THREAD == NA && LB::PER_THREAD == 8, "vectors per thread and operand");
  LA la;
  LB lb;
  la.init(p.lda, m0, p.M, tid);
  lb.init(p.ldb, n0, p.N, tid, SWIGLU ? p.N >> 1 : 0);
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(p.a, p.a_bytes), rb = make_rsrc(p.b, p.b_bytes);

  // The accumulators are not cleared: the first k-step of the first k-tile multiplies into a
  // constant zero (256 register writes per lane saved on every output tile).
  f32x16 acc[TM][TN];

  const int kt0 = blockIdx.y * p.kt_per_split;
  const int last_tile = (int)((p.K + BK - 1) / BK) - 1;
  // a split past the end of K (the last ones, when K does not divide evenly) has no k-tiles: zeros
  const int nk = max(0, min(p.kt_per_split, last_tile + 1 - kt0));
  auto load_a = [&](auto s_c, auto i_c, uint32_t t) __attribute__((always_inline)) {
    constexpr int S = decltype(s_c)::value, I = decltype(i_c)::value;
    if constexpr (RAGGED_K) {
      const KAdvance k = k_advance<true>(t, (uint32_t)last_tile, la.kstep);
      la.template load1_checked<S, I>(ra, k.lane, k.scalar);
    } else {
      la.template load1<S, I>(ra, t * la.kstep);
    }
  };
  auto load_b = [&](auto s_c, auto i_c, uint32_t t) __attribute__((always_inline)) {
    constexpr int S = decltype(s_c)::value, I = decltype(i_c)::value;
    if constexpr (RAGGED_K) {
      const KAdvance k = k_advance<true>(t, (uint32_t)last_tile, lb.kstep);
      lb.template load1_checked<S, I>(rb, k.lane, k.scalar);
    } else {
      lb.template load1<S, I>(rb, t * lb.kstep);
    }
  };
  auto load_all = [&](auto s_c, int kt) {
    const uint32_t t = (uint32_t)min(kt, last_tile);
    static_for<NA>([&](auto i) { load_a(s_c, i, t); });
    static_for<8>([&](auto i) { load_b(s_c, i, t); });
  };
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  // Prologue.  Tiles 0 and 1 are requested together (one exposed latency for both); tile 0 goes
  // to stage 0 and its registers take tile 2.  From here on, at k-tile kt of parity P, set P^1
  // holds tile kt+1 and set P tile kt+2.  The first Q3 of tile 1's A vectors are moved here: the
  // k-loop moves those in the last k-step of the tile before.
  load_all(C0{}, kt0);
  load_all(C1{}, kt0 + 1);
  static_for<NA>([&](auto i) { la.template store1<0, decltype(i)::value>(As, tid); });
  static_for<8>([&](auto i) { lb.template store1<0, decltype(i)::value>(Bs, tid); });
  load_all(C0{}, kt0 + 2);
  {
    const uint32_t t = (uint32_t)min(kt0 + 3, last_tile);
    static_for<Q3>([&](auto i) { la.template store1<1, decltype(i)::value>(As + A_SIZE, tid); });
    static_for<Q3>([&](auto i) { load_a(C1{}, i, t); });
  }
  __syncthreads();

  // Fragments, double-buffered: unit u of a k-step, in the order of first use: A0, B0..B3, A1...
  bf16x8 af[2][TM], bfr[2][TN];
  auto fetch_unit = [&](auto u_c, auto buf_c, const bf16_t* at, const bf16_t* bt, auto kk_c) {
    constexpr int u = decltype(u_c)::value, buf = decltype(buf_c)::value, kk = decltype(kk_c)::value;
    if constexpr (u == 0) af[buf][0] = fetch_frag<A_T, A_STRIDE>(at, wm * WM, kk, lane);
    else if constexpr (u <= 4) bfr[buf][u - 1] = fetch_frag<B_T, B_STRIDE>(bt, wn * WN + 32 * (u - 1), kk, lane);
    else af[buf][u - 4] = fetch_frag<A_T, A_STRIDE>(at, wm * WM + 32 * (u - 4), kk, lane);
  };
  static_for<NU>([&](auto u) { fetch_unit(u, C0{}, As, Bs, C0{}); });

  // One k-tile.  P = parity of the tile = its LDS stage = the staging set that holds tile kt+2
  // (the other set holds tile kt+1).
  auto iteration = [&](auto p_c, auto first_c, int kt) __attribute__((always_inline)) {
    constexpr int P = decltype(p_c)::value;
    constexpr bool FIRST = decltype(first_c)::value;
    bf16_t* an = As + (P ^ 1) * A_SIZE;
    bf16_t* bn = Bs + (P ^ 1) * B_SIZE;
    const bf16_t* at = As + P * A_SIZE;
    const bf16_t* bt = Bs + P * B_SIZE;
    const uint32_t t3 = (uint32_t)min(kt0 + kt + 3, last_tile), t4 = (uint32_t)min(kt0 + kt + 4, last_tile);
    // The tile move, vector q of NA + 8 (A vectors, then B vectors).  k-steps 0..2 move vectors
    // Q3.. of tile kt+1 (set P^1 -> the other stage, refilled with tile kt+3); k-step 3, once the
    // barrier has freed this tile's own stage, vectors 0..Q3-1 of tile kt+2 (set P -> this stage,
    // refilled with tile kt+4).
    auto move_store = [&](auto kk_c, auto q_c) __attribute__((always_inline)) {
      constexpr int kk = decltype(kk_c)::value, q = decltype(q_c)::value, S = kk == 3 ? P : (P ^ 1);
      if constexpr (q < NA) la.template store1<S, q>(kk == 3 ? const_cast<bf16_t*>(at) : an, tid);
      else lb.template store1<S, q - NA>(kk == 3 ? const_cast<bf16_t*>(bt) : bn, tid);
    };
    auto move_load = [&](auto kk_c, auto q_c) __attribute__((always_inline)) {
      constexpr int kk = decltype(kk_c)::value, q = decltype(q_c)::value, S = kk == 3 ? P : (P ^ 1);
      using SC = std::integral_constant<int, S>;
      if constexpr (q < NA) load_a(SC{}, q_c, kk == 3 ? t4 : t3);
      else load_b(SC{}, std::integral_constant<int, q - NA>{}, kk == 3 ? t4 : t3);
    };
    // slot m of k-step kk: MFMA block (m / 4, m % 4), preceded by one memory operation.
    //   TM = 4 (16 slots): even m reads fragment unit m/2 of the next k-step (in the last k-step,
    //     after the barrier, of the next tile's first k-step); odd m does half a vector move,
    //     alternately the store to LDS and the refill of the register.
    //   TM = 3 (12 slots): m = 0, 2, .., 10 and 11 read the seven fragment units; m = 1, 3, .., 9
    //     each move one whole vector (store, then refill) while vectors remain.
    auto slot = [&](auto kk_c, auto m_c) __attribute__((always_inline)) {
      constexpr int kk = decltype(kk_c)::value, m = decltype(m_c)::value;
      if constexpr (kk == 3 && m == 0) __syncthreads();
      constexpr int unit = (m % 2 == 0) ? m / 2 : ((TM == 3 && m == 11) ? 6 : -1);
      if constexpr (unit >= 0) {
        using U = std::integral_constant<int, unit>;
        if constexpr (kk < 3)
          fetch_unit(U{}, std::integral_constant<int, (kk + 1) & 1>{}, at, bt, std::integral_constant<int, kk + 1>{});
        else
          fetch_unit(U{}, C0{}, an, bn, C0{});
      } else if constexpr (TM == 4) {
        constexpr int o = (m - 1) / 2;                          // 0..7 within the k-step
        using Q = std::integral_constant<int, (kk == 3 ? 0 : 4 + 4 * kk) + o / 2>;
        if constexpr (o % 2 == 0) move_store(kk_c, Q{});
        else move_load(kk_c, Q{});
      } else {
        constexpr int o = (m - 1) / 2;                          // 0..4 within the k-step
        constexpr int q = kk == 3 ? o : Q3 + 5 * kk + o;
        if constexpr (kk == 3 ? (o < Q3) : (q < NA + 8)) {
          move_store(kk_c, std::integral_constant<int, q>{});
          move_load(kk_c, std::integral_constant<int, q>{});
        }
      }
      constexpr int i = m / 4, j = m % 4;
      if constexpr (FIRST && kk == 0) {
        constexpr f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[0][j], af[0][i], zero, 0, 0, 0);
      } else {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    auto step = [&](auto kk_c) __attribute__((always_inline)) {
      static_for<NS>([&](auto m) __attribute__((always_inline)) { slot(kk_c, m); });
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
  };
  if (nk >= 1) {
    iteration(C0{}, std::true_type{}, 0);
  } else {   // a split without k-tiles writes zeros
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
  }
  for (int kt = 1; kt + 1 < nk; kt += 2) {
    iteration(C1{}, std::false_type{}, kt);
    iteration(C0{}, std::false_type{}, kt + 1);
  }
  if (nk >= 2 && !(nk & 1)) iteration(C1{}, std::false_type{}, nk - 1);

  // the epilogue stages through the B stages (large enough for either tile height)
  constexpr int ST_STRIDE = WN + 4;  // floats
  static_assert(4 * 32 * ST_STRIDE * 4 <= 2 * B_SIZE * 2, "staging must fit in the B stages");
  if constexpr (OUT_F32) p.c = reinterpret_cast<float*>(p.c) + blockIdx.y * p.c_split_stride;
  if constexpr (SWIGLU)
    store_tile_swiglu<TM>(p, acc, reinterpret_cast<float*>(Bs) + wave * 32 * ST_STRIDE, m0 + wm * WM,
                          (n0 >> 1) + 64 * wn, lane);
  else if constexpr (EPI == 2)
    store_tile_swiglu_bwd<TM>(p, acc, reinterpret_cast<float*>(Bs) + wave * 32 * ST_STRIDE, m0 + wm * WM,
                              n0 + wn * WN, lane);
  else {
    if constexpr (EPI == 3 || EPI == 4) {
      if (rope_rotate_tile<TM, EPI == 3 ? 128 : 64>(p, acc, m0 + wm * WM, n0 + wn * WN, lane)) p.bias = nullptr;
    }
    store_tile<TM, TN, OUT_F32, true>(p, acc, reinterpret_cast<float*>(Bs) + wave * 32 * ST_STRIDE,
                                      m0 + wm * WM, n0 + wn * WN, lane);
  }
}

template <int TM, bool A_T, bool B_T, bool OUT_F32>
__global__ __launch_bounds__(256) void gemm4_kernel(GemmParams p) {
  gemm4_tile<TM, A_T, B_T, OUT_F32, false>(p);
}
// Weight gradients over a token count that is no multiple of 64.
template <bool OUT_F32>
__global__ __launch_bounds__(256) void gemm4_ragged_k_kernel(GemmParams p) {
  gemm4_tile<4, true, true, OUT_F32, true>(p);
}

// Y = [gate | up] = X.W and silu(gate) * up in one pass (the decoder's MLP up-projection).
__global__ __launch_bounds__(256) void gemm4_swiglu_kernel(GemmParams p) {
  gemm4_tile<4, false, true, false, false, 1>(p);
}
// dA = dY.W_d^T kept in registers; [d gate | d up] written (the decoder's MLP down-projection, backward).
__global__ __launch_bounds__(256) void gemm4_swiglu_bwd_kernel(GemmParams p) {
  gemm4_tile<4, false, false, false, false, 2>(p);
}

// Y = X.W (+ b) with the rotary positions applied to the q and k heads in the epilogue.
template <int HD>
__global__ __launch_bounds__(256) void gemm4_rope_kernel(GemmParams p) {
  gemm4_tile<4, false, true, false, false, HD == 128 ? 3 : 4>(p);
}

// The four-wavefront kernel takes a problem tiled 256 x 256 when K is a positive multiple of 64,
// or any K >= 64 when k runs along the rows of both operands (the weight-gradient layout).
bool takes_gemm4(const GemmArgs& g) {
  return g.k >= BK && (g.k % BK == 0 || (g.a_layout != 0 && g.b_layout == 0));
}
// Its 192-row form when that saves rounds of one-per-CU workgroups.  A round of 192-row tiles
// has three quarters of the MFMA work but the same prologue and epilogue: measured at 0.9 of a
// round of 256-row tiles for K = 1024..4096.  Only for A stored [M, K] and unsplit problems.
bool takes_rows192(const GemmArgs& g, int splits) {
  if (!takes_gemm4(g) || g.a_layout != 0 || splits != 1) return false;
  const int64_t tn = (g.n + 255) / 256, t192 = ((g.m + 191) / 192) * tn, t256 = ((g.m + 255) / 256) * tn;
  return 9 * ((t192 + 255) / 256) < 10 * ((t256 + 255) / 256);
}

template <int BM, int BN, int WM, int WN, int BKT = 64>
hipError_t launch_tile(const GemmArgs& g, hipStream_t s, int splits = 1) {
  GemmParams p = make_gemm_params(g, BM, BN);
  p.kt_per_split = (int)((g.k + BKT - 1) / BKT);
  if (splits > 1) {
    p.kt_per_split = (p.kt_per_split + splits - 1) / splits;
    p.c_split_stride = g.m * g.n;
  }
  dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)splits), block(64 * (BM / WM) * (BN / WN));
  const bool at = g.a_layout != 0, bt = g.b_layout == 0;  // b_layout 0 = [K,N] = transposing reads
  if (BM == 256 && BN == 256 && takes_gemm4(g)) {
    const dim3 block4(256);
    if (g.swiglu_act) {   // launch_gemm has checked gemm_swiglu_fusable()
      hipLaunchKernelGGL(gemm4_swiglu_kernel, grid, block4, 0, s, p);
      return hipGetLastError();
    }
    if (g.swiglu_dpre) {
      hipLaunchKernelGGL(gemm4_swiglu_bwd_kernel, grid, block4, 0, s, p);
      return hipGetLastError();
    }
    if (g.rope_table) {   // launch_gemm has checked gemm_rope_fusable()
      if (g.rope_head_dim == 128) hipLaunchKernelGGL(gemm4_rope_kernel<128>, grid, block4, 0, s, p);
      else hipLaunchKernelGGL(gemm4_rope_kernel<64>, grid, block4, 0, s, p);
      return hipGetLastError();
    }
    const bool rows192 = takes_rows192(g, splits);
    if (rows192) {
      p.tiles_m = (int)((g.m + 191) / 192);
      grid.x = (unsigned)(p.tiles_m * p.tiles_n);
    }
#define MLLM_GEMM4_CASE(AT, BT, F32)                                                     \
  if (at == AT && bt == BT && (g.out_fp32 != 0) == F32) {                                \
    if constexpr (!AT) {                                                                 \
      if (rows192) {                                                                     \
        hipLaunchKernelGGL((gemm4_kernel<3, AT, BT, F32>), grid, block4, 0, s, p);       \
        return hipGetLastError();                                                        \
      }                                                                                  \
    }                                                                                    \
    if constexpr (AT && BT) {                                                            \
      if (g.k % BK != 0) {                                                               \
        hipLaunchKernelGGL((gemm4_ragged_k_kernel<F32>), grid, block4, 0, s, p);         \
        return hipGetLastError();                                                        \
      }                                                                                  \
    }                                                                                    \
    hipLaunchKernelGGL((gemm4_kernel<4, AT, BT, F32>), grid, block4, 0, s, p);           \
    return hipGetLastError();                                                            \
  }
    MLLM_GEMM4_CASE(false, true, false)
    MLLM_GEMM4_CASE(false, false, false)
    MLLM_GEMM4_CASE(true, true, true)
    MLLM_GEMM4_CASE(false, true, true)
    MLLM_GEMM4_CASE(false, false, true)
    MLLM_GEMM4_CASE(true, true, false)
    MLLM_GEMM4_CASE(true, false, false)
    MLLM_GEMM4_CASE(true, false, true)
#undef MLLM_GEMM4_CASE
  }
#define MLLM_GEMM_CASE(AT, BT, F32)                                                      \
  if (at == AT && bt == BT && (g.out_fp32 != 0) == F32) {                                \
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, AT, BT, F32, BKT>), grid, block, 0, s, p); \
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

// Weight-gradient GEMMs of narrow layers (M x N small, K = tokens large) have too few output tiles
// to fill 256 CUs.  They are cut along K into `splits` partial products (fp32, in a scratch
// buffer), summed afterwards in a fixed order.  Returns 1 when the plain launch is used.
namespace {
struct SplitPlan { int splits; bool big_tile; };
SplitPlan plan_split(int64_t m, int64_t n, int64_t k) {
  const int64_t t256 = ((m + 255) / 256) * ((n + 255) / 256), t128 = ((m + 127) / 128) * ((n + 127) / 128);
  const int64_t nk = (k + BK - 1) / BK;
  if (t256 >= 200) {
    // Enough tiles to fill the chip, but a last partial round of workgroups can leave most CUs
    // idle (1.5 rounds cost 2).  Cutting K in S parts makes S times as many, S times shorter
    // workgroups: pick the S <= 4 with the fewest rounds per unit of work, charging the
    // reduction pass about a twentieth of a round.
    int best = 1;
    double best_cost = (double)((t256 + 255) / 256);
    for (int sp = 2; sp <= 4 && nk / sp >= 64; sp++) {
      const double cost = (double)((t256 * sp + 255) / 256) / sp + 0.05 * sp;
      if (cost < best_cost - 1e-9) { best_cost = cost; best = sp; }
    }
    return {best, true};
  }
  const bool big = t256 >= 24;
  const int64_t cap = std::max<int64_t>(1, std::min<int64_t>(16, nk / 8));   // at least 8 k-tiles per split
  if (big) {
    // One 256x256 workgroup per CU: S splits make t256 * S workgroups that run in
    // ceil(t256 * S / 256) rounds of 1/S of the K loop each; a split also costs its partial
    // product's trip through memory, about a hundredth of a full K loop.
    int best = 1;
    double best_cost = 1e30;
    for (int sp = 1; sp <= cap; sp++) {
      const double cost = (double)((t256 * sp + 255) / 256) / sp + 0.01 * sp;
      if (cost < best_cost - 1e-9) { best_cost = cost; best = sp; }
    }
    return {best, true};
  }
  const int64_t want = std::min<int64_t>((512 + t128 - 1) / t128, cap);
  return {(int)std::max<int64_t>(want, 1), false};
}
}  // namespace

size_t gemm_splitk_ws_bytes(int64_t m, int64_t n, int64_t k) {
  const SplitPlan sp = plan_split(m, n, k);
  return sp.splits > 1 ? (size_t)sp.splits * (size_t)m * (size_t)n * 4 : 0;
}

bool gemm_swiglu_fusable(int64_t m, int64_t n, int64_t k) {
  const int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
  return big_tiles >= 200 && n % 256 == 0 && k >= BK && k % BK == 0;
}

bool gemm_swiglu_bwd_fusable(int64_t m, int64_t n, int64_t k) {
  const int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
  return big_tiles >= 200 && n % 8 == 0 && k >= BK && k % BK == 0;
}

bool gemm_rope_fusable(int64_t m, int64_t n, int64_t k, int32_t head_dim) {
  const int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
  return big_tiles >= 200 && (head_dim == 64 || head_dim == 128) && n % 8 == 0 && k >= BK && k % BK == 0;
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.m <= 0 || g.n <= 0) return hipSuccess;
  if (g.rope_table && (!g.rope_pos || !gemm_rope_fusable(g.m, g.n, g.k, g.rope_head_dim) || g.a_layout != 0 ||
                       g.b_layout != 0 || g.out_fp32 || g.residual || g.swiglu_act || g.swiglu_dpre || g.ldc != g.n ||
                       g.rope_cols % 128 != 0 || g.rope_cols > g.n))
    return hipErrorInvalidValue;
  if ((g.swiglu_dpre || g.swiglu_pre) &&
      (!g.swiglu_dpre || !g.swiglu_pre || g.swiglu_act || !gemm_swiglu_bwd_fusable(g.m, g.n, g.k) || g.a_layout != 0 ||
       g.b_layout != 1 || g.out_fp32 || g.bias || g.residual || g.ldc != 2 * g.n))
    return hipErrorInvalidValue;
  if (g.swiglu_act && (!gemm_swiglu_fusable(g.m, g.n, g.k) || g.a_layout != 0 || g.b_layout != 0 || g.out_fp32 ||
                       g.bias || g.residual || g.ldc != g.n))
    return hipErrorInvalidValue;
  // operands are addressed through 32-bit buffer offsets
  if ((g.a_layout ? g.k : g.m) * g.lda * 2 > GEMM_MAX_OPERAND_BYTES || (g.b_layout ? g.n : g.k) * g.ldb * 2 > GEMM_MAX_OPERAND_BYTES)
    return hipErrorInvalidValue;
  // the epilogue addresses a sub-tile of up to 128 rows with 32-bit offsets from its first element
  if (g.ldc * (g.out_fp32 ? 4 : 2) * 128 > 0xFFFFFFFFll || (g.residual && g.ldres * 2 * 128 > 0xFFFFFFFFll))
    return hipErrorInvalidValue;
  const int64_t big_tiles = ((g.m + 255) / 256) * ((g.n + 255) / 256);
  const SplitPlan sp = plan_split(g.m, g.n, g.k);
  const bool split = sp.splits > 1 && g.out_fp32 && !g.bias && g.ldc == g.n && g.splitk_ws &&
                     g.splitk_ws_bytes >= (size_t)sp.splits * g.m * g.n * 4;
  const bool large = big_tiles >= 200 || (split && sp.big_tile);
  // timing classes: the three layouts of the 256x256 kernel, its 192-row form, and the 128x128 kernel
  const int cls = !large ? PROF_GEMM_SMALL : (!split && !g.swiglu_act && !g.swiglu_dpre && !g.rope_table && takes_rows192(g, 1)) ? PROF_GEMM_ROWS192
                  : g.a_layout ? PROF_GEMM_DW : (g.b_layout ? PROF_GEMM_DX : PROF_GEMM_FWD);
  const double flops = 2.0 * (double)g.m * (double)g.n * (double)g.k;
  // 256x256 tiles (8 wavefronts of 128x64) once they fill the chip; smaller problems keep
  // 128x128 tiles so that more workgroups exist.
  if (!split) {
    ProfScope prof(cls, flops, s);
    return big_tiles >= 200 ? launch_tile<256, 256, 128, 64>(g, s) : launch_tile<128, 128, 64, 64>(g, s);
  }
  GemmArgs part = g;
  part.c = g.splitk_ws;
  part.accumulate = 0;
  hipError_t e;
  {
    ProfScope prof(cls, flops, s);
    e = sp.big_tile ? launch_tile<256, 256, 128, 64>(part, s, sp.splits)
                    : launch_tile<128, 128, 64, 64>(part, s, sp.splits);
  }
  if (e != hipSuccess) return e;
  return launch_splitk_reduce((const float*)g.splitk_ws, (float*)g.c, sp.splits, g.m * g.n, g.accumulate, s);
}

}  // namespace mllm
