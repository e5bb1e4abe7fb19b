// bf16 MFMA GEMM, 256x256x64 tiles fed by direct-to-LDS buffer loads (gfx950).
//
// Same contraction and layouts as gemm.hip (the linear operations over the whole packed sequence,
// Model Profiler, "Throughput Profiling"), but the operand tiles go from global memory straight
// into LDS (`buffer_load_dwordx4 ... lds`): no staging registers, no LDS store instructions, and
// a wavefront never stalls on a global load in the middle of its MFMA stream.
//
// LDS layout.  A direct-to-LDS load writes lane l's 16 bytes at (uniform base) + 16*l, so one
// wavefront instruction fills 1 KiB contiguously and rows cannot be padded.  Bank conflicts are
// avoided by permuting WHICH global 16-byte chunk a lane fetches: chunk c of row r lives at
// position c ^ swz(r) of that row.
//   * operand stored [rows, K] (contraction contiguous): tile [rows][64], 128 B rows, 8 rows per
//     instruction, swz(r) = (r >> 1) & 7; fragments are read with one ds_read_b128 per lane.
//   * operand stored [K, cols]: tile [64][cols], rows of 2*cols bytes as they lie in memory,
//     swz(k) = 4 * (k & 3); fragments are read with the LDS transposing read.
// Two stages per operand in separate LDS arrays; the K loop is unrolled by two so that every
// access names its stage statically.
#include <cstdlib>

#include "gemm_common.h"

namespace mllm {

namespace {

#define MLLM_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int PF_DIST = 2;  // tiles between an L2 prefetch and the load it serves
// s_waitcnt immediate: vmcnt <= 2, no wait on expcnt / lgkmcnt (gfx9 field layout)
constexpr int WAIT_VMCNT_2 = 2 | (0x7 << 4) | (0xF << 8);

// One operand tile.  ROWS x ROWELEMS elements in LDS; K_ROWS: rows run along the contraction.
template <int ROWS, int ROWELEMS, bool K_ROWS, int NW>
struct DmaTile {
  static constexpr int CHUNKS_PER_ROW = ROWELEMS / 8;
  static constexpr int ROWS_PER_INSTR = 64 / CHUNKS_PER_ROW;
  static constexpr int N_INSTR = ROWS / ROWS_PER_INSTR;
  static constexpr int PER_WAVE = N_INSTR / NW;
  static constexpr int SIZE = ROWS * ROWELEMS;  // elements
  static_assert(64 % CHUNKS_PER_ROW == 0 && N_INSTR % NW == 0 && PER_WAVE >= 1, "tile shape");
  uint32_t off[PER_WAVE];  // byte offset of this lane's chunk at k0 = 0, OOB if never valid
  int klim[PER_WAVE];      // chunk is inside the matrix while k0 < klim
  uint32_t kstep;
  uint32_t pf_off;         // L2 prefetch: byte offset of the 128-byte line this lane touches
  int pf_klim;

  // LDS serves 256 B per clock (64 banks): a 16-byte read is processed 16 lanes at a time, an
  // 8-byte transposing read 32 lanes at a time.  16 consecutive 128-byte rows must therefore put
  // their chunk on 16 different 16-byte slots of a 256-byte window ((r&1, pos) distinct), and the
  // 4 rows x 64 B that 32 lanes of a transposing read touch on the 4 quarters of a window.
  __device__ __forceinline__ static int swz(int r) { return K_ROWS ? 4 * (r & 3) : ((r >> 1) & 7); }

  __device__ __forceinline__ void init(int64_t ld, int64_t fixed0, int64_t nfixed, int64_t K, int wave, int lane) {
    kstep = (uint32_t)(K_ROWS ? BK * ld * 2 : BK * 2);
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      const int q = wave * PER_WAVE + i;
      const int r = q * ROWS_PER_INSTR + lane / CHUNKS_PER_ROW;
      const int c = (lane % CHUNKS_PER_ROW) ^ swz(r);
      const int64_t fx = fixed0 + (K_ROWS ? 8 * c : r);
      const int64_t lin = K_ROWS ? (int64_t)r * ld + fx : fx * ld + 8 * c;
      off[i] = fx < nfixed ? (uint32_t)(lin * 2) : OOB;
      klim[i] = (int)(K - (K_ROWS ? r : 8 * c));
    }
    // One lane per 128-byte line of the tile: ROWS * ROWELEMS * 2 / 128 lines = 64 * NW lanes.
    constexpr int LINES_PER_ROW = ROWELEMS * 2 / 128, N_LINES = ROWS * LINES_PER_ROW;
    static_assert(N_LINES <= 64 * NW, "at most one prefetch instruction per wavefront");
    const int line = wave * 64 + lane, r = line / LINES_PER_ROW, e = (line % LINES_PER_ROW) * 64;
    const int64_t fx = fixed0 + (K_ROWS ? e : r);
    pf_off = (fx < nfixed && line < N_LINES) ? (uint32_t)((K_ROWS ? (int64_t)r * ld + fx : fx * ld + e) * 2) : OOB;
    pf_klim = (int)(K - (K_ROWS ? r : e));
  }
  // Touch every line of tile kt so that it is in L2 by the time the real load asks for it.  The
  // four bytes per lane land in a scratch area nobody reads.
  __device__ __forceinline__ void prefetch(__amdgpu_buffer_rsrc_t rsrc, void* scratch, int kt) const {
    const uint32_t o = (pf_off != OOB && kt * BK < pf_klim) ? pf_off + (uint32_t)kt * kstep : OOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, MLLM_LDS_PTR(scratch), 4, (int)o, 0, 0, 0);
  }
  // Enqueue this wavefront's share of tile kt into the stage at `lds` (wave-uniform pointer).
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, bf16_t* lds, int kt, int wave) const {
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < PER_WAVE; i++) {
      const uint32_t o = (off[i] != OOB && k0 < klim[i]) ? off[i] + (uint32_t)kt * kstep : OOB;
      bf16_t* dst = lds + (wave * PER_WAVE + i) * 512;  // 1 KiB per instruction
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, MLLM_LDS_PTR(dst), 16, (int)o, 0, 0, 0);
    }
  }
  // Eight contraction values k = 16*kk + 8*(lane/32) .. +7 of tile row/column (r0 + lane%32).
  __device__ __forceinline__ static bf16x8 frag(const bf16_t* tile, int r0, int kk, int lane) {
    Frag8 f;
    const int h = lane >> 5;
    if constexpr (!K_ROWS) {
      const int r = r0 + (lane & 31), c = 2 * kk + h;
      f.u = *reinterpret_cast<const uint4*>(tile + r * ROWELEMS + 8 * (c ^ swz(r)));
    } else {
      const int i16 = lane & 15, g = (lane >> 4) & 1;
      const int n = r0 + 16 * g + 4 * (i16 & 3);       // first of this lane's 4 columns
      const int k = 16 * kk + 8 * h + (i16 >> 2);       // row of the first read; second read is k + 4
      const int pos = (n >> 3) ^ swz(k);                // swz(k) == swz(k + 4)
      const bf16_t* p0 = tile + k * ROWELEMS + 8 * pos + (n & 7);
      f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)p0);
      f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)(p0 + 4 * ROWELEMS));
    }
    return f.v;
  }
};

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T, bool OUT_F32>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_dma_kernel(GemmParams p) {
  constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN;
  constexpr int TM = WM / 32, TN = WN / 32, STEPS = BK / 16;
  using TA = DmaTile<A_T ? BK : BM, A_T ? BM : BK, A_T, NW>;
  using TB = DmaTile<B_T ? BK : BN, B_T ? BN : BK, B_T, NW>;
  __shared__ __attribute__((aligned(1024))) bf16_t As0[TA::SIZE];
  __shared__ __attribute__((aligned(1024))) bf16_t As1[TA::SIZE];
  __shared__ __attribute__((aligned(1024))) bf16_t Bs0[TB::SIZE];
  __shared__ __attribute__((aligned(1024))) bf16_t Bs1[TB::SIZE];
  __shared__ __attribute__((aligned(256))) uint32_t pf_scratch[NW * 64];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / NWN, wn = wave % NWN;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  TA la;
  TB lb;
  la.init(p.lda, m0, p.M, p.K, wave, lane);
  lb.init(p.ldb, n0, p.N, p.K, wave, lane);
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(p.a, p.a_bytes), rb = make_rsrc(p.b, p.b_bytes);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  bf16x8 af[2][TM], bfr[2][TN];
  auto fetch = [&](int buf, const bf16_t* at, const bf16_t* bt, int kk) {
#pragma unroll
    for (int i = 0; i < TM; i++) af[buf][i] = TA::frag(at, wm * WM + 32 * i, kk, lane);
#pragma unroll
    for (int j = 0; j < TN; j++) bfr[buf][j] = TB::frag(bt, wn * WN + 32 * j, kk, lane);
  };
  // One tile: enqueue the loads of the next tile into the other stage, then four k-steps of
  // (fetch next step's fragments, TM*TN MFMAs), then the barrier that also waits for the loads.
  auto tile_step = [&](const bf16_t* at, const bf16_t* bt, bf16_t* an, bf16_t* bn, int kt_next) {
    la.issue(ra, an, kt_next, wave);
    lb.issue(rb, bn, kt_next, wave);
    la.prefetch(ra, pf_scratch + wave * 64, kt_next + PF_DIST);
    lb.prefetch(rb, pf_scratch + wave * 64, kt_next + PF_DIST);
    __builtin_amdgcn_sched_barrier(0);  // the loads go out before the MFMA stream, not after it
#pragma unroll
    for (int kk = 0; kk < STEPS; kk++) {
      if (kk + 1 < STEPS) fetch((kk + 1) & 1, at, bt, kk + 1);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
    }
    // Loads return in order: letting the two youngest (the L2 prefetches) stay in flight still
    // guarantees that this wavefront's share of (an, bn) has landed.  The fragment reads of
    // (at, bt) completed before the MFMAs that used them were issued.
    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT_2);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    fetch(0, an, bn, 0);
  };

  const int nk = (int)((p.K + BK - 1) / BK);
  la.issue(ra, As0, 0, wave);
  lb.issue(rb, Bs0, 0, wave);
  __syncthreads();
  fetch(0, As0, Bs0, 0);
  // Tiles past the end load zeros (out-of-range offsets) and add nothing, so an odd tile count
  // simply runs one empty half-iteration.
  for (int kt = 0; kt < nk; kt += 2) {
    tile_step(As0, Bs0, As1, Bs1, kt + 1);
    tile_step(As1, Bs1, As0, Bs0, kt + 2);
  }

  // Epilogue staging: 32 x (WN+4) floats per wavefront, carved out of the four stage arrays.
  constexpr int ST_BYTES = 32 * (WN + 4) * 4;
  constexpr int PER_ARRAY = NW / 4;
  static_assert(NW % 4 == 0 && PER_ARRAY * ST_BYTES <= TA::SIZE * 2 && PER_ARRAY * ST_BYTES <= TB::SIZE * 2, "staging fits");
  bf16_t* arr = (wave / PER_ARRAY) == 0 ? As0 : (wave / PER_ARRAY) == 1 ? As1 : (wave / PER_ARRAY) == 2 ? Bs0 : Bs1;
  float* stage = reinterpret_cast<float*>(arr) + (wave % PER_ARRAY) * (ST_BYTES / 4);
  store_tile<TM, TN, OUT_F32>(p, acc, stage, m0 + wm * WM, n0 + wn * WN, lane);
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_dma_tile(const GemmArgs& g, hipStream_t s) {
  GemmParams p = make_gemm_params(g, BM, BN);
  dim3 grid((unsigned)(p.tiles_m * p.tiles_n)), block(64 * (BM / WM) * (BN / WN));
  const bool at = g.a_layout != 0, bt = g.b_layout == 0;  // b_layout 0 = stored [K,N]
#define MLLM_GEMM_CASE(AT, BT, F32)                                                          \
  if (at == AT && bt == BT && (g.out_fp32 != 0) == F32) {                                    \
    hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WM, WN, AT, BT, F32>), grid, block, 0, s, p); \
    return hipGetLastError();                                                                \
  }
  MLLM_GEMM_CASE(false, true, false)
  MLLM_GEMM_CASE(false, false, false)
  MLLM_GEMM_CASE(true, true, true)
  MLLM_GEMM_CASE(false, true, true)
  MLLM_GEMM_CASE(false, false, true)
  MLLM_GEMM_CASE(true, true, false)
  MLLM_GEMM_CASE(true, false, false)
  MLLM_GEMM_CASE(true, false, true)
#undef MLLM_GEMM_CASE
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_dma(const GemmArgs& g, hipStream_t s) {
  static const char* impl = getenv("MLLM_GEMM_IMPL");
  if (impl && impl[0] == '8') return launch_dma_tile<256, 256, 128, 64>(g, s);
  return launch_dma_tile<256, 256, 128, 128>(g, s);
}

}  // namespace mllm
