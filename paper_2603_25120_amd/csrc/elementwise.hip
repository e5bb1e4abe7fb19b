// HBM-bound kernels of the stage: LayerNorm / RMSNorm forward and backward (one wavefront per
// row, wavefront reductions), rotary positions, GELU / SwiGLU forward and backward, bias-gradient
// column sums, row scatter / gather for the connector.  All math in fp32 on bf16 storage, 16-byte
// accesses, no atomics: every cross-row reduction is two deterministic stages.
#include "common.h"
#include "kernels.h"

namespace mllm {

namespace {

constexpr int ROWS_PER_BLOCK = 4;  // 4 wavefronts, one row each

__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = bf16lo(u.x); f[1] = bf16hi(u.x); f[2] = bf16lo(u.y); f[3] = bf16hi(u.y);
  f[4] = bf16lo(u.z); f[5] = bf16hi(u.z); f[6] = bf16lo(u.w); f[7] = bf16hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                    pack_bf16x2(f[6], f[7]));
}

// ---------------------------------------------------------------------------------------------
// normalisation forward: y = (x - mean) * rstd * gamma + beta   (LayerNorm, KIND 0)
//                        y = x * rstd * gamma                   (RMSNorm,   KIND 1)
// NV = 16-byte vectors per lane; the row lives in registers between the passes.  Rows of x and y
// are ld elements apart (ld = d for a dense matrix, more for a column slice of a wider one).
// ---------------------------------------------------------------------------------------------
template <int KIND, int NV>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const bf16_t* __restrict__ x,
                                                       const bf16_t* __restrict__ gamma,
                                                       const bf16_t* __restrict__ beta,
                                                       bf16_t* __restrict__ y, float* __restrict__ stats,
                                                       int64_t T, int d, int64_t ld, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
  if (row >= T) return;
  const int nvec = d >> 3;
  float v[NV][8];
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < NV; j++) {
    int c = lane + 64 * j;
    if (c < nvec) {
      uint4 u = *reinterpret_cast<const uint4*>(x + row * ld + 8 * c);
      unpack8(u, v[j]);
#pragma unroll
      for (int e = 0; e < 8; e++) sum += v[j][e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; e++) v[j][e] = 0.f;
    }
  }
  float mean = 0.f;
  if (KIND == 0) mean = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < NV; j++) {
    int c = lane + 64 * j;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < 8; e++) {
        float t = v[j][e] - mean;
        sq += t * t;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
  if (lane == 0) {
    stats[row] = rstd;
    stats[T + row] = mean;
  }
#pragma unroll
  for (int j = 0; j < NV; j++) {
    int c = lane + 64 * j;
    if (c < nvec) {
      float g[8], b[8], o[8];
      unpack8(*reinterpret_cast<const uint4*>(gamma + 8 * c), g);
      if (KIND == 0) unpack8(*reinterpret_cast<const uint4*>(beta + 8 * c), b);
#pragma unroll
      for (int e = 0; e < 8; e++) {
        o[e] = (v[j][e] - mean) * rstd * g[e];
        if (KIND == 0) o[e] += b[e];
      }
      *reinterpret_cast<uint4*>(y + row * ld + 8 * c) = pack8(o);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// normalisation backward.  With xhat = (x - mean) * rstd and dxh = dy * gamma:
//   LayerNorm: dx = (dxh - mean(dxh) - xhat * mean(dxh * xhat)) * rstd
//   RMSNorm:   dx = (dxh - xhat * mean(dxh * xhat)) * rstd
// plus the residual branch's gradient dres.  Rows of dy, x, dres and dx are ld elements apart.
// A workgroup of 256 threads owns one row at a time
// (rows b, b + B, ...); a thread keeps NV 16-byte vectors of the row and its own column sums of
// dy * xhat (and of dy) in registers; they go to partial[b][*] at the end.
// ---------------------------------------------------------------------------------------------
template <int KIND, int NV>
__global__ __launch_bounds__(256) void norm_bwd_kernel(
    const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
    const float* __restrict__ stats, const bf16_t* __restrict__ dres, bf16_t* __restrict__ dx,
    float* __restrict__ partial, int64_t T, int d, int64_t ld) {
  __shared__ float red[2][2][4];  // [row parity][which sum][wavefront]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int B = gridDim.x, b = blockIdx.x;
  const int nvec = d >> 3;
  float g[NV][8], dg[NV][8], db[NV][8];
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int c = tid + 256 * j;
    if (c < nvec) unpack8(*reinterpret_cast<const uint4*>(gamma + 8 * c), g[j]);
#pragma unroll
    for (int e = 0; e < 8; e++) { dg[j][e] = 0.f; db[j][e] = 0.f; if (c >= nvec) g[j][e] = 0.f; }
  }
  int parity = 0;
  for (int64_t row = b; row < T; row += B, parity ^= 1) {
    const float rstd = stats[row];
    const float mean = KIND == 0 ? stats[T + row] : 0.f;
    float xh[NV][8], dxh[NV][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int c = tid + 256 * j;
      if (c < nvec) {
        float xv[8], dv[8];
        unpack8(*reinterpret_cast<const uint4*>(x + row * ld + 8 * c), xv);
        unpack8(*reinterpret_cast<const uint4*>(dy + row * ld + 8 * c), dv);
#pragma unroll
        for (int e = 0; e < 8; e++) {
          xh[j][e] = (xv[e] - mean) * rstd;
          dxh[j][e] = dv[e] * g[j][e];
          s1 += dxh[j][e];
          s2 += dxh[j][e] * xh[j][e];
          dg[j][e] += dv[e] * xh[j][e];
          db[j][e] += dv[e];
        }
      }
    }
    s2 = wave_sum(s2);
    if (KIND == 0) s1 = wave_sum(s1);
    if (lane == 0) { red[parity][0][wave] = s1; red[parity][1][wave] = s2; }
    __syncthreads();  // one barrier per row: the two parities alternate, so a slot is rewritten
                      // only after every wavefront has passed the barrier of the row in between
    const float m2 = (red[parity][1][0] + red[parity][1][1] + red[parity][1][2] + red[parity][1][3]) / (float)d;
    const float m1 = KIND == 0 ? (red[parity][0][0] + red[parity][0][1] + red[parity][0][2] + red[parity][0][3]) / (float)d : 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int c = tid + 256 * j;
      if (c < nvec) {
        float o[8], r[8];
        if (dres) unpack8(*reinterpret_cast<const uint4*>(dres + row * ld + 8 * c), r);
#pragma unroll
        for (int e = 0; e < 8; e++) {
          o[e] = (dxh[j][e] - m1 - xh[j][e] * m2) * rstd;
          if (dres) o[e] += r[e];
        }
        *reinterpret_cast<uint4*>(dx + row * ld + 8 * c) = pack8(o);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int c = tid + 256 * j;
    if (c < nvec) {
      float* pg = partial + (int64_t)b * d + 8 * c;
      *reinterpret_cast<float4*>(pg) = make_float4(dg[j][0], dg[j][1], dg[j][2], dg[j][3]);
      *reinterpret_cast<float4*>(pg + 4) = make_float4(dg[j][4], dg[j][5], dg[j][6], dg[j][7]);
      if (KIND == 0) {
        float* pb = partial + (int64_t)(B + b) * d + 8 * c;
        *reinterpret_cast<float4*>(pb) = make_float4(db[j][0], db[j][1], db[j][2], db[j][3]);
        *reinterpret_cast<float4*>(pb + 4) = make_float4(db[j][4], db[j][5], db[j][6], db[j][7]);
      }
    }
  }
}

// out[c] (+)= sum_p partial[p][c].  A workgroup owns 8 columns: 128 row slices x 2 float4 column
// groups; slice s adds rows s, s+128, ... in order (four loads in flight), then the slice sums are
// added pairwise (s with s+64, then s with s+32, ...): a fixed association, so the result is
// bitwise reproducible.
constexpr int RED_COLS = 8, RED_SLICES = 128;
// blockIdx.y = 1, 2 (when launched with two or three rows of workgroups) reduce a second and third
// set of partial sums, P * n and 2 P * n floats further on, into out1 and out2: a norm's gradients go
// in one launch.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial,
                                                              float* __restrict__ out, int P,
                                                              int64_t n, int accumulate,
                                                              float* __restrict__ out1 = nullptr,
                                                              float* __restrict__ out2 = nullptr) {
  __shared__ float4 part[RED_SLICES][RED_COLS / 4];
  if (blockIdx.y == 1) { partial += (int64_t)P * n; out = out1; }
  if (blockIdx.y == 2) { partial += 2 * (int64_t)P * n; out = out2; }
  if (!out) return;   // a set that this launch does not carry
  const int cg = threadIdx.x & 1, slice = threadIdx.x >> 1;
  const int64_t c = ((int64_t)blockIdx.x * (RED_COLS / 4) + cg) * 4;
  const bool valid = c < n;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (valid) {
    const float* col = partial + c;
    int p = slice;
    for (; p + 3 * RED_SLICES < P; p += 4 * RED_SLICES) {
      const float4 v0 = *reinterpret_cast<const float4*>(col + (int64_t)p * n);
      const float4 v1 = *reinterpret_cast<const float4*>(col + (int64_t)(p + RED_SLICES) * n);
      const float4 v2 = *reinterpret_cast<const float4*>(col + (int64_t)(p + 2 * RED_SLICES) * n);
      const float4 v3 = *reinterpret_cast<const float4*>(col + (int64_t)(p + 3 * RED_SLICES) * n);
      s.x += (v0.x + v1.x) + (v2.x + v3.x); s.y += (v0.y + v1.y) + (v2.y + v3.y);
      s.z += (v0.z + v1.z) + (v2.z + v3.z); s.w += (v0.w + v1.w) + (v2.w + v3.w);
    }
    for (; p < P; p += RED_SLICES) {
      const float4 v = *reinterpret_cast<const float4*>(col + (int64_t)p * n);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  part[slice][cg] = s;
  __syncthreads();
#pragma unroll
  for (int half = RED_SLICES / 2; half >= 1; half >>= 1) {
    if (slice < half) {
      const float4 a = part[slice][cg], b = part[slice + half][cg];
      part[slice][cg] = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
    }
    __syncthreads();
  }
  if (slice == 0 && valid) {
    float4 t = part[0][cg];
    float4* o = reinterpret_cast<float4*>(out + c);
    if (accumulate) {
      const float4 old = *o;
      t.x += old.x; t.y += old.y; t.z += old.z; t.w += old.w;
    }
    *o = t;
  }
}

// ---------------------------------------------------------------------------------------------
// rotary positions, in place, half-split pairs (i, i + hd/2); angle = pos * base^(-2i/hd).
// One thread: one token, eight consecutive i, all heads.  Angles in fp64 so that positions in
// the ten-thousands keep full fp32-accurate sines.
// ---------------------------------------------------------------------------------------------
__global__ void rope_kernel(bf16_t* __restrict__ qk, const int32_t* __restrict__ pos, int64_t T,
                            int64_t row_stride, int64_t col0, int n_heads, int hd, double log2_base,
                            int inverse) {
  const int per_tok = hd >> 4;  // threads per token
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t t = gid / per_tok;
  if (t >= T) return;
  const int i0 = (int)(gid % per_tok) * 8;
  const double p = (double)pos[t];
  float cs[8], sn[8];
#pragma unroll
  for (int e = 0; e < 8; e++) {
    double inv = exp2(-2.0 * (double)(i0 + e) / (double)hd * log2_base);
    double s, c;
    sincos(p * inv, &s, &c);
    cs[e] = (float)c;
    sn[e] = inverse ? -(float)s : (float)s;
  }
  bf16_t* base = qk + t * row_stride + col0 + i0;
  const int half = hd >> 1;
  for (int h = 0; h < n_heads; h++) {
    bf16_t* p1 = base + h * hd;
    float a[8], b[8], oa[8], ob[8];
    unpack8(*reinterpret_cast<const uint4*>(p1), a);
    unpack8(*reinterpret_cast<const uint4*>(p1 + half), b);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      oa[e] = a[e] * cs[e] - b[e] * sn[e];
      ob[e] = b[e] * cs[e] + a[e] * sn[e];
    }
    *reinterpret_cast<uint4*>(p1) = pack8(oa);
    *reinterpret_cast<uint4*>(p1 + half) = pack8(ob);
  }
}

// Table of the rotary angles for the kernels that rotate in their own epilogue: row `pos` holds
// cos(pos * base^(-2i/hd)) for i < hd/2, then the sines (fp32; angles and sincos in fp64, as in
// rope_kernel, so both forms of the rotation use the same factors).
__global__ void rope_table_kernel(float* __restrict__ table, int64_t n_pos, int hd, double log2_base) {
  const int half = hd >> 1;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= n_pos * half) return;
  const int64_t pos = gid / half;
  const int i = (int)(gid % half);
  const double inv = exp2(-2.0 * (double)i / (double)hd * log2_base);
  double sn, cs;
  sincos((double)pos * inv, &sn, &cs);
  table[pos * hd + i] = (float)cs;
  table[pos * hd + half + i] = (float)sn;
}

// ---------------------------------------------------------------------------------------------
// activations
// ---------------------------------------------------------------------------------------------
__global__ void gelu_fwd_kernel(int act, const bf16_t* __restrict__ h, bf16_t* __restrict__ a, int64_t nvec) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float z[8], o[8];
  unpack8(reinterpret_cast<const uint4*>(h)[i], z);
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = gelu_f(act, z[e]);
  reinterpret_cast<uint4*>(a)[i] = pack8(o);
}
__global__ void gelu_bwd_kernel(int act, const bf16_t* __restrict__ da, const bf16_t* __restrict__ h,
                                bf16_t* __restrict__ dh, int64_t nvec) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float z[8], g[8], o[8];
  unpack8(reinterpret_cast<const uint4*>(h)[i], z);
  unpack8(reinterpret_cast<const uint4*>(da)[i], g);
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = g[e] * gelu_grad_f(act, z[e]);
  reinterpret_cast<uint4*>(dh)[i] = pack8(o);
}
// The same with the column sums of dh (the gradient of the bias in front of the activation) formed
// on the way: workgroup (bx, by) owns columns [512 bx, 512 bx + 512) and rows by*4 + wave + k*4*gridDim.y;
// a lane keeps eight columns, the four wavefronts' sums are added through LDS in a fixed order and
// land in row by of `partial` ([gridDim.y, f] fp32), which reduce_partials_kernel then sums.
// da and dh may be the same buffer (a lane reads its eight values of a row before it writes them).
__global__ __launch_bounds__(256) void gelu_bwd_colsum_kernel(int act, const bf16_t* da,
                                                              const bf16_t* __restrict__ h, bf16_t* dh,
                                                              float* __restrict__ partial, int64_t T, int64_t f) {
  __shared__ float red[3][64][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = ((int64_t)blockIdx.x * 64 + lane) * 8;
  const bool valid = c < f;
  const int64_t step = (int64_t)gridDim.y * 4;
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (valid) {
    int64_t r = (int64_t)blockIdx.y * 4 + wave;
    uint4 zq, gq;
    if (r < T) { zq = *reinterpret_cast<const uint4*>(h + r * f + c); gq = *reinterpret_cast<const uint4*>(da + r * f + c); }
    for (; r < T; r += step) {
      float z[8], g[8], o[8];
      unpack8(zq, z);
      unpack8(gq, g);
      if (r + step < T) {   // the next row's loads go out before this row's arithmetic
        zq = *reinterpret_cast<const uint4*>(h + (r + step) * f + c);
        gq = *reinterpret_cast<const uint4*>(da + (r + step) * f + c);
      }
#pragma unroll
      for (int e = 0; e < 8; e++) { o[e] = g[e] * gelu_grad_f(act, z[e]); s[e] += o[e]; }
      *reinterpret_cast<uint4*>(dh + r * f + c) = pack8(o);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) red[wave - 1][lane][e] = s[e];
  }
  __syncthreads();
  if (wave == 0 && valid) {
#pragma unroll
    for (int e = 0; e < 8; e++) s[e] = (s[e] + red[0][lane][e]) + (red[1][lane][e] + red[2][lane][e]);
    float* p = partial + (int64_t)blockIdx.y * f + c;
    *reinterpret_cast<float4*>(p) = make_float4(s[0], s[1], s[2], s[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(s[4], s[5], s[6], s[7]);
  }
}
// gu = [g | u], [T, 2f];  a = g * sigmoid(g) * u
__global__ void swiglu_fwd_kernel(const bf16_t* __restrict__ gu, bf16_t* __restrict__ a, int64_t T, int64_t f) {
  const int64_t vec_per_row = f >> 3;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * vec_per_row) return;
  const int64_t t = i / vec_per_row, c = (i % vec_per_row) * 8;
  float g[8], u[8], o[8];
  unpack8(*reinterpret_cast<const uint4*>(gu + t * 2 * f + c), g);
  unpack8(*reinterpret_cast<const uint4*>(gu + t * 2 * f + f + c), u);
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = g[e] / (1.f + expf(-g[e])) * u[e];
  *reinterpret_cast<uint4*>(a + t * f + c) = pack8(o);
}
__global__ void swiglu_bwd_kernel(const bf16_t* __restrict__ da, const bf16_t* __restrict__ gu,
                                  bf16_t* __restrict__ dgu, int64_t T, int64_t f) {
  const int64_t vec_per_row = f >> 3;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * vec_per_row) return;
  const int64_t t = i / vec_per_row, c = (i % vec_per_row) * 8;
  float g[8], u[8], d[8], og[8], ou[8];
  unpack8(*reinterpret_cast<const uint4*>(gu + t * 2 * f + c), g);
  unpack8(*reinterpret_cast<const uint4*>(gu + t * 2 * f + f + c), u);
  unpack8(*reinterpret_cast<const uint4*>(da + t * f + c), d);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    float s = 1.f / (1.f + expf(-g[e]));
    og[e] = d[e] * u[e] * (s + g[e] * s * (1.f - s));
    ou[e] = d[e] * g[e] * s;
  }
  *reinterpret_cast<uint4*>(dgu + t * 2 * f + c) = pack8(og);
  *reinterpret_cast<uint4*>(dgu + t * 2 * f + f + c) = pack8(ou);
}

// ---------------------------------------------------------------------------------------------
// column sums (bias gradients), stage 1: a workgroup owns 512 columns (8 per lane) and row chunk
// blockIdx.y; its four wavefronts take every fourth row of the chunk, four loads in flight each,
// and their sums are added through LDS in a fixed order.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ x, int64_t ldx,
                                                             float* __restrict__ partial, int64_t T,
                                                             int64_t n) {
  __shared__ float red[3][64][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = ((int64_t)blockIdx.x * 64 + lane) * 8;
  const bool valid = c < n;
  const int64_t step = (int64_t)gridDim.y * 4;
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (valid) {
    const bf16_t* col = x + c;
    int64_t r = (int64_t)blockIdx.y * 4 + wave;
    for (; r + 3 * step < T; r += 4 * step) {
      const uint4 u0 = *reinterpret_cast<const uint4*>(col + r * ldx);
      const uint4 u1 = *reinterpret_cast<const uint4*>(col + (r + step) * ldx);
      const uint4 u2 = *reinterpret_cast<const uint4*>(col + (r + 2 * step) * ldx);
      const uint4 u3 = *reinterpret_cast<const uint4*>(col + (r + 3 * step) * ldx);
      float v0[8], v1[8], v2[8], v3[8];
      unpack8(u0, v0); unpack8(u1, v1); unpack8(u2, v2); unpack8(u3, v3);
#pragma unroll
      for (int e = 0; e < 8; e++) s[e] += (v0[e] + v1[e]) + (v2[e] + v3[e]);
    }
    for (; r < T; r += step) {
      float v[8];
      unpack8(*reinterpret_cast<const uint4*>(col + r * ldx), v);
#pragma unroll
      for (int e = 0; e < 8; e++) s[e] += v[e];
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) red[wave - 1][lane][e] = s[e];
  }
  __syncthreads();
  if (wave == 0 && valid) {
#pragma unroll
    for (int e = 0; e < 8; e++) s[e] = (s[e] + red[0][lane][e]) + (red[1][lane][e] + red[2][lane][e]);
    float* p = partial + (int64_t)blockIdx.y * n + c;
    *reinterpret_cast<float4*>(p) = make_float4(s[0], s[1], s[2], s[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(s[4], s[5], s[6], s[7]);
  }
}

__global__ void scatter_rows_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                    const int32_t* __restrict__ rows, int64_t n_rows, int64_t vec_per_row,
                                    int gather) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows * vec_per_row) return;
  const int64_t r = i / vec_per_row, c = i % vec_per_row;
  const int64_t other = rows[r];
  if (gather) reinterpret_cast<uint4*>(dst)[r * vec_per_row + c] = reinterpret_cast<const uint4*>(src)[other * vec_per_row + c];
  else reinterpret_cast<uint4*>(dst)[other * vec_per_row + c] = reinterpret_cast<const uint4*>(src)[r * vec_per_row + c];
}
// Average pooling at the end of the encoder (Evaluation, audio modality) and its gradient.
__global__ void pool_rows_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                 const int32_t* __restrict__ first, const int32_t* __restrict__ count,
                                 int64_t n_out, int64_t vec_per_row) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_out * vec_per_row) return;
  const int64_t j = i / vec_per_row, c = i % vec_per_row;
  const int64_t r0 = first[j];
  const int n = count[j];
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = 0; r < n; r++) {
    float v[8];
    unpack8(reinterpret_cast<const uint4*>(src)[(r0 + r) * vec_per_row + c], v);
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] += v[e];
  }
  const float inv = 1.f / (float)n;
#pragma unroll
  for (int e = 0; e < 8; e++) acc[e] *= inv;
  reinterpret_cast<uint4*>(dst)[j * vec_per_row + c] = pack8(acc);
}
__global__ void unpool_rows_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                   const int32_t* __restrict__ window, const int32_t* __restrict__ count,
                                   int64_t n_rows, int64_t vec_per_row) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows * vec_per_row) return;
  const int64_t r = i / vec_per_row, c = i % vec_per_row;
  const int64_t j = window[r];
  float v[8];
  unpack8(reinterpret_cast<const uint4*>(src)[j * vec_per_row + c], v);
  const float inv = 1.f / (float)count[j];
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] *= inv;
  reinterpret_cast<uint4*>(dst)[r * vec_per_row + c] = pack8(v);
}
__global__ void zero_rows_kernel(bf16_t* __restrict__ dst, const int32_t* __restrict__ rows,
                                 int64_t n_rows, int64_t vec_per_row) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows * vec_per_row) return;
  const int64_t r = rows[i / vec_per_row], c = i % vec_per_row;
  reinterpret_cast<uint4*>(dst)[r * vec_per_row + c] = make_uint4(0, 0, 0, 0);
}
__global__ void splitk_reduce_kernel(const float4* __restrict__ partial, float4* __restrict__ out,
                                     int splits, int64_t nvec, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  // the parts are added in their order; four of their loads are in flight at a time
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  if (accumulate) o = out[i];
  float4 t = partial[i];
  int sp = 1;
  for (; sp + 3 < splits; sp += 4) {
    const float4 a = partial[(int64_t)sp * nvec + i], b = partial[(int64_t)(sp + 1) * nvec + i];
    const float4 c = partial[(int64_t)(sp + 2) * nvec + i], d = partial[(int64_t)(sp + 3) * nvec + i];
    t.x += a.x; t.y += a.y; t.z += a.z; t.w += a.w;
    t.x += b.x; t.y += b.y; t.z += b.z; t.w += b.w;
    t.x += c.x; t.y += c.y; t.z += c.z; t.w += c.w;
    t.x += d.x; t.y += d.y; t.z += d.z; t.w += d.w;
  }
  for (; sp < splits; sp++) {
    const float4 v = partial[(int64_t)sp * nvec + i];
    t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
  }
  t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
  out[i] = t;
}
__global__ void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t nvec) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nvec) dst[i] = src[i];
}

inline unsigned blocks_for(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

#define MLLM_NV_DISPATCH(NVEC, CALL)          \
  if ((NVEC) <= 64) { CALL(1) }               \
  else if ((NVEC) <= 128) { CALL(2) }         \
  else if ((NVEC) <= 256) { CALL(4) }         \
  else if ((NVEC) <= 512) { CALL(8) }         \
  else { CALL(16) }

hipError_t launch_norm_fwd(int kind, const void* x, const void* gamma, const void* beta, void* y,
                           float* stats, int64_t t, int64_t d, int64_t ld, float eps, hipStream_t s) {
  if (t == 0) return hipSuccess;
  if (d % 8 != 0 || d > 8192 || ld < d || ld % 8 != 0) return hipErrorInvalidValue;
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)t * (double)d, s);
  dim3 grid(blocks_for(t, ROWS_PER_BLOCK)), block(256);
#define CALL(NV)                                                                                  \
  if (kind == 0) hipLaunchKernelGGL((norm_fwd_kernel<0, NV>), grid, block, 0, s, (const bf16_t*)x, \
      (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, stats, t, (int)d, ld, eps);              \
  else hipLaunchKernelGGL((norm_fwd_kernel<1, NV>), grid, block, 0, s, (const bf16_t*)x,           \
      (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, stats, t, (int)d, ld, eps);
  MLLM_NV_DISPATCH(d / 8, CALL)
#undef CALL
  return hipGetLastError();
}

// Narrow rows (d <= 1024): a wavefront owns a row, so there is no barrier per row and all 256
// threads have data; the four wavefronts' column sums are added through LDS once at the end.
// CS: the column sums of dx (as computed, before rounding to bf16) come out as a third set of
// partial sums: dx is the gradient of a linear map's output whenever the layer below or the
// attention block above the norm ends in one, and those sums are that map's bias gradient.
template <int KIND, int NV, bool CS>
__global__ __launch_bounds__(256, 3) void norm_bwd_wave_kernel(
    const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
    const float* __restrict__ stats, const bf16_t* __restrict__ dres, bf16_t* __restrict__ dx,
    float* __restrict__ partial, int64_t T, int d, int64_t ld) {
  __shared__ float red[CS ? 3 : 2][4][1024];  // [d gamma | d beta | column sums of dx][wavefront][column]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int B = gridDim.x, b = blockIdx.x;
  const int nvec = d >> 3;
  float g[NV][8], dg[NV][8], db[NV][8], dc[CS ? NV : 1][8];
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int c = lane + 64 * j;
    if (c < nvec) unpack8(*reinterpret_cast<const uint4*>(gamma + 8 * c), g[j]);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      dg[j][e] = 0.f; db[j][e] = 0.f; if (c >= nvec) g[j][e] = 0.f;
      if (CS) dc[j][e] = 0.f;
    }
  }
  // The next row's loads are issued before this row's arithmetic: two rows in flight per wavefront.
  uint4 nx[NV], ndy[NV], nres[NV];
  auto fetch = [&](int64_t row) {
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int c = lane + 64 * j;
      if (c < nvec) {
        nx[j] = *reinterpret_cast<const uint4*>(x + row * ld + 8 * c);
        ndy[j] = *reinterpret_cast<const uint4*>(dy + row * ld + 8 * c);
        if (dres) nres[j] = *reinterpret_cast<const uint4*>(dres + row * ld + 8 * c);
      }
    }
  };
  const int64_t row0 = (int64_t)b * 4 + wave, row_step = (int64_t)4 * B;
  if (row0 < T) fetch(row0);
  for (int64_t row = row0; row < T; row += row_step) {
    const float rstd = stats[row];
    const float mean = KIND == 0 ? stats[T + row] : 0.f;
    float xh[NV][8], dxh[NV][8], r[NV][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int c = lane + 64 * j;
#pragma unroll
      for (int e = 0; e < 8; e++) { xh[j][e] = 0.f; dxh[j][e] = 0.f; r[j][e] = 0.f; }
      if (c < nvec) {
        float xv[8], dv[8];
        unpack8(nx[j], xv);
        unpack8(ndy[j], dv);
        if (dres) unpack8(nres[j], r[j]);
#pragma unroll
        for (int e = 0; e < 8; e++) {
          xh[j][e] = (xv[e] - mean) * rstd;
          dxh[j][e] = dv[e] * g[j][e];
          s1 += dxh[j][e];
          s2 += dxh[j][e] * xh[j][e];
          dg[j][e] += dv[e] * xh[j][e];
          db[j][e] += dv[e];
        }
      }
    }
    if (row + row_step < T) fetch(row + row_step);
    const float m2 = wave_sum(s2) / (float)d;
    const float m1 = KIND == 0 ? wave_sum(s1) / (float)d : 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int c = lane + 64 * j;
      if (c < nvec) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
          o[e] = (dxh[j][e] - m1 - xh[j][e] * m2) * rstd + r[j][e];
          if (CS) dc[j][e] += o[e];
        }
        *reinterpret_cast<uint4*>(dx + row * ld + 8 * c) = pack8(o);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int c = lane + 64 * j;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < 8; e++) {
        red[0][wave][8 * c + e] = dg[j][e];
        red[1][wave][8 * c + e] = db[j][e];
        if (CS) red[2][wave][8 * c + e] = dc[j][e];
      }
    }
  }
  __syncthreads();
  for (int col = tid; col < d; col += 256) {
    partial[(int64_t)b * d + col] = (red[0][0][col] + red[0][1][col]) + (red[0][2][col] + red[0][3][col]);
    if (KIND == 0)
      partial[(int64_t)(B + b) * d + col] = (red[1][0][col] + red[1][1][col]) + (red[1][2][col] + red[1][3][col]);
    if (CS)
      partial[(int64_t)(2 * B + b) * d + col] = (red[2][0][col] + red[2][1][col]) + (red[2][2][col] + red[2][3][col]);
  }
}

bool norm_bwd_colsum_fusable(int64_t d) { return d % 8 == 0 && d / 8 <= 128; }

int64_t norm_bwd_partial_rows(int64_t t) {
  return t < 1 ? 1 : (t > 1024 ? 1024 : t);
}

hipError_t launch_norm_bwd(int kind, const void* dy, const void* x, const void* gamma,
                           const float* stats, const void* dres, void* dx, float* dgamma,
                           float* dbeta, int accumulate, float* partial, int64_t t, int64_t d,
                           int64_t ld, hipStream_t s, float* dx_colsum) {
  if (d % 8 != 0 || d > 8192 || ld < d || ld % 8 != 0) return hipErrorInvalidValue;
  if (dx_colsum && !norm_bwd_colsum_fusable(d)) return hipErrorInvalidValue;
  const int64_t nvec = d / 8;
  // Workgroups (= rows of partial sums).  The wavefront-per-row kernel with two vectors per lane
  // keeps three workgroups per CU resident: a grid of 768 runs in one round.
  int64_t W = norm_bwd_partial_rows(t);
  if (nvec > 64 && nvec <= 128) W = std::min<int64_t>(W, 768);
  ProfScope prof(PROF_ELEMENTWISE, (dres ? 8.0 : 6.0) * (double)t * (double)d, s);
  dim3 grid((unsigned)W), block(256);
#define CALL(NV)                                                                                   \
  if (kind == 0) hipLaunchKernelGGL((norm_bwd_kernel<0, NV>), grid, block, 0, s, (const bf16_t*)dy, \
      (const bf16_t*)x, (const bf16_t*)gamma, stats, (const bf16_t*)dres, (bf16_t*)dx, partial, t, (int)d, ld); \
  else hipLaunchKernelGGL((norm_bwd_kernel<1, NV>), grid, block, 0, s, (const bf16_t*)dy,           \
      (const bf16_t*)x, (const bf16_t*)gamma, stats, (const bf16_t*)dres, (bf16_t*)dx, partial, t, (int)d, ld);
#define CALL_WAVE_CS(KIND, NV, CS)                                                                          \
  hipLaunchKernelGGL((norm_bwd_wave_kernel<KIND, NV, CS>), grid, block, 0, s, (const bf16_t*)dy,             \
      (const bf16_t*)x, (const bf16_t*)gamma, stats, (const bf16_t*)dres, (bf16_t*)dx, partial, t, (int)d, ld);
#define CALL_WAVE(NV)                                                                       \
  if (kind == 0) { if (dx_colsum) { CALL_WAVE_CS(0, NV, true) } else { CALL_WAVE_CS(0, NV, false) } } \
  else { if (dx_colsum) { CALL_WAVE_CS(1, NV, true) } else { CALL_WAVE_CS(1, NV, false) } }
  if (nvec <= 64) { CALL_WAVE(1) } else if (nvec <= 128) { CALL_WAVE(2) }
  else if (nvec <= 256) { CALL(1) } else if (nvec <= 512) { CALL(2) } else { CALL(4) }
#undef CALL_WAVE
#undef CALL_WAVE_CS
#undef CALL
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks_for(d, RED_COLS), dx_colsum ? 3 : (kind == 0 ? 2 : 1)), dim3(256), 0, s,
                     partial, dgamma, (int)W, d, accumulate, kind == 0 ? dbeta : nullptr, dx_colsum);
  return hipGetLastError();
}

hipError_t launch_rope(void* qk, const int32_t* pos, int64_t t, int64_t row_stride, int64_t col0,
                       int32_t n_heads, int32_t head_dim, float rope_base, int inverse,
                       hipStream_t s) {
  if (t == 0 || n_heads == 0) return hipSuccess;
  if (head_dim % 16 != 0 || row_stride % 8 != 0 || col0 % 8 != 0) return hipErrorInvalidValue;
  const int64_t n = t * (head_dim / 16);
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)t * (double)n_heads * (double)head_dim, s);
  hipLaunchKernelGGL(rope_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, (bf16_t*)qk, pos, t,
                     row_stride, col0, (int)n_heads, (int)head_dim, log2((double)rope_base), inverse);
  return hipGetLastError();
}

hipError_t launch_rope_table(float* table, int64_t n_pos, int32_t head_dim, float rope_base, hipStream_t s) {
  if (n_pos == 0) return hipSuccess;
  if (head_dim % 16 != 0) return hipErrorInvalidValue;
  const int64_t n = n_pos * (head_dim / 2);
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)n_pos * (double)head_dim, s);
  hipLaunchKernelGGL(rope_table_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, table, n_pos, (int)head_dim,
                     log2((double)rope_base));
  return hipGetLastError();
}

hipError_t launch_act_fwd(int act, const void* pre, void* a, int64_t t, int64_t f, hipStream_t s) {
  if (t == 0) return hipSuccess;
  if (f % 8 != 0) return hipErrorInvalidValue;
  const int64_t nvec = t * f / 8;
  ProfScope prof(PROF_ELEMENTWISE, (act == 2 ? 6.0 : 4.0) * (double)t * (double)f, s);
  if (act == 2)
    hipLaunchKernelGGL(swiglu_fwd_kernel, dim3(blocks_for(nvec, 256)), dim3(256), 0, s,
                       (const bf16_t*)pre, (bf16_t*)a, t, f);
  else
    hipLaunchKernelGGL(gelu_fwd_kernel, dim3(blocks_for(nvec, 256)), dim3(256), 0, s, act,
                       (const bf16_t*)pre, (bf16_t*)a, nvec);
  return hipGetLastError();
}

hipError_t launch_act_bwd(int act, const void* da, const void* pre, void* dpre, int64_t t,
                          int64_t f, hipStream_t s) {
  if (t == 0) return hipSuccess;
  if (f % 8 != 0) return hipErrorInvalidValue;
  const int64_t nvec = t * f / 8;
  ProfScope prof(PROF_ELEMENTWISE, (act == 2 ? 10.0 : 6.0) * (double)t * (double)f, s);
  if (act == 2)
    hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(blocks_for(nvec, 256)), dim3(256), 0, s,
                       (const bf16_t*)da, (const bf16_t*)pre, (bf16_t*)dpre, t, f);
  else
    hipLaunchKernelGGL(gelu_bwd_kernel, dim3(blocks_for(nvec, 256)), dim3(256), 0, s, act,
                       (const bf16_t*)da, (const bf16_t*)pre, (bf16_t*)dpre, nvec);
  return hipGetLastError();
}

hipError_t launch_gelu_bwd_colsum(int act, const void* da, const void* pre, void* dpre, float* colsum,
                                  int accumulate, float* partial, int64_t t, int64_t f, hipStream_t s) {
  if (f % 8 != 0 || (act != 0 && act != 1)) return hipErrorInvalidValue;
  const int64_t P = colsum_partial_rows(t);
  ProfScope prof(PROF_ELEMENTWISE, 6.0 * (double)t * (double)f, s);
  hipLaunchKernelGGL(gelu_bwd_colsum_kernel, dim3(blocks_for(f, 512), (unsigned)P), dim3(256), 0, s, act,
                     (const bf16_t*)da, (const bf16_t*)pre, (bf16_t*)dpre, partial, t, f);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks_for(f, RED_COLS)), dim3(256), 0, s, partial, colsum, (int)P,
                     f, accumulate);
  return hipGetLastError();
}

int64_t colsum_partial_rows(int64_t t) {   // row chunks of (at least) four rows, at most 512
  if (t < 4) return 1;
  return t < 2048 ? t / 4 : 512;
}

hipError_t launch_colsum(const void* x, int64_t ldx, float* out, int accumulate, float* partial,
                         int64_t t, int64_t n, hipStream_t s) {
  if (n % 8 != 0 || ldx % 8 != 0) return hipErrorInvalidValue;
  const int64_t P = colsum_partial_rows(t);
  ProfScope prof(PROF_ELEMENTWISE, 2.0 * (double)t * (double)n, s);
  hipLaunchKernelGGL(colsum_partial_kernel, dim3(blocks_for(n, 512), (unsigned)P), dim3(256), 0, s,
                     (const bf16_t*)x, ldx, partial, t, n);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks_for(n, RED_COLS)), dim3(256), 0, s, partial,
                     out, (int)P, n, accumulate);
  return hipGetLastError();
}

hipError_t launch_scatter_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows,
                               int64_t d, int gather, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (d % 8 != 0) return hipErrorInvalidValue;
  const int64_t n = n_rows * (d / 8);
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)n_rows * (double)d, s);
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s,
                     (const bf16_t*)src, (bf16_t*)dst, rows, n_rows, d / 8, gather);
  return hipGetLastError();
}

hipError_t launch_pool_rows(const void* src, void* dst, const int32_t* first, const int32_t* count,
                            int64_t n_out, int64_t d, hipStream_t s) {
  if (n_out == 0) return hipSuccess;
  if (d % 8 != 0) return hipErrorInvalidValue;
  const int64_t n = n_out * (d / 8);
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)n_out * (double)d, s);
  hipLaunchKernelGGL(pool_rows_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, (const bf16_t*)src,
                     (bf16_t*)dst, first, count, n_out, d / 8);
  return hipGetLastError();
}

hipError_t launch_unpool_rows(const void* src, void* dst, const int32_t* window, const int32_t* count,
                              int64_t n_rows, int64_t d, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (d % 8 != 0) return hipErrorInvalidValue;
  const int64_t n = n_rows * (d / 8);
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)n_rows * (double)d, s);
  hipLaunchKernelGGL(unpool_rows_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, (const bf16_t*)src,
                     (bf16_t*)dst, window, count, n_rows, d / 8);
  return hipGetLastError();
}

hipError_t launch_zero_rows(void* dst, const int32_t* rows, int64_t n_rows, int64_t d,
                            hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (d % 8 != 0) return hipErrorInvalidValue;
  const int64_t n = n_rows * (d / 8);
  hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, (bf16_t*)dst,
                     rows, n_rows, d / 8);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* partial, float* out, int splits, int64_t n, int accumulate,
                                hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (n % 4 != 0) return hipErrorInvalidValue;
  ProfScope prof(PROF_ELEMENTWISE, 4.0 * (double)n * (splits + 1 + (accumulate ? 1 : 0)), s);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks_for(n / 4, 256)), dim3(256), 0, s,
                     (const float4*)partial, (float4*)out, splits, n / 4, accumulate);
  return hipGetLastError();
}

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16 != 0) return hipErrorInvalidValue;
  const int64_t nvec = (int64_t)(bytes / 16);
  ProfScope prof(PROF_ELEMENTWISE, 2.0 * (double)bytes, s);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks_for(nvec, 256)), dim3(256), 0, s, (const uint4*)src,
                     (uint4*)dst, nvec);
  return hipGetLastError();
}

}  // namespace mllm
