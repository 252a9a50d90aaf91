// fp32 variant of the dense steps (plain FMA, 64 x 64 tiles through LDS).
// It exists for exactness checks on small shapes, not for speed: operands are
// addressed through generic strides so one kernel serves all three
// contractions without transposed copies.
#pragma once

#include "common.hip.h"
#include "rng.hip.h"

namespace oapl {

// element (row, k) of an operand is p[row * s_row + k * s_k]
struct F32Operand {
  const float* p;
  int64_t s_row, s_k;
};

// C[m][n] = sum_k A(m, k) * B(n, k) for one 64 x 64 tile; 256 threads, each a
// 4 x 4 micro-tile: rows 4*ty .. 4*ty+3, columns 4*tx .. 4*tx+3 with
// tx = tid % 16 (16 consecutive lanes share a row group).
template <class Epi>
__global__ void __launch_bounds__(256)
k_gemm_f32(F32Operand A, F32Operand B, int64_t M, int64_t N, int64_t K, Epi epi) {
  __shared__ float As[16][65], Bs[16][65];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256, row = e >> 4, kk = e & 15;
      const int64_t k = k0 + kk;
      As[kk][row] = (m0 + row < M && k < K) ? A.p[(m0 + row) * A.s_row + k * A.s_k] : 0.f;
      Bs[kk][row] = (n0 + row < N && k < K) ? B.p[(n0 + row) * B.s_row + k * B.s_k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  epi(acc, m0 + ty * 4, n0 + tx * 4, M, N);
}

// Forward: M = tokens, N = vocabulary.  Per token row and 64-column tile the
// pair (m, s) = (max_v z, sum_v exp(z - m)); parts[tile][t].
struct EpiLseF32 {
  float2* parts;
  int64_t T;
  float* upart;  // optional third partial u = sum_v exp(z - m) * z (for the entropy), or nullptr
  __device__ void operator()(float (&acc)[4][4], int64_t m, int64_t n, int64_t M, int64_t N) const {
    const int64_t part = n >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float mx = -__builtin_inff();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (n + j >= N) acc[i][j] = -__builtin_inff();
        mx = fmaxf(mx, acc[i][j]);
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      const float ref = fmaxf(mx, kNegHuge);
      float s = 0.f, u = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float e = expf(acc[i][j] - ref);
        s += e;
        u += e > 0.f ? e * acc[i][j] : 0.f;
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) { s += __shfl_xor(s, o, 64); u += __shfl_xor(u, o, 64); }
      if ((threadIdx.x & 15) == 0 && m + i < M) {
        parts[part * T + m + i] = make_float2(ref, s);
        if (upart) upart[part * T + m + i] = u;
      }
    }
  }
};

// Sampling: M = tokens, N = vocabulary.  Per token row and 64-column tile the best perturbed logit
// z / temperature + Gumbel(Philox(seed; v / 4, t)) and its vocabulary index; parts[tile][t].
struct EpiSampleF32 {
  float2* parts;
  int64_t T;
  float inv_temperature;
  uint32_t seed_lo, seed_hi;
  __device__ void operator()(float (&acc)[4][4], int64_t m, int64_t n, int64_t M, int64_t N) const {
    const int64_t part = n >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t t = m + i;
      uint32_t x[4];
      philox4x32_10((uint32_t)(n >> 2), (uint32_t)t, (uint32_t)(t >> 32), 0u, seed_lo, seed_hi, x);
      float best = -__builtin_inff();
      int arg = 0x7FFFFFFF;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float sc = __builtin_fmaf(acc[i][j], inv_temperature, gumbel_from_bits(x[j]));
        if (n + j < N && sc > best) { best = sc; arg = (int)(n + j); }
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) {
        const float so = __shfl_xor(best, o, 64);
        const int io = __shfl_xor(arg, o, 64);
        if (better(so, io, best, arg)) { best = so; arg = io; }
      }
      if ((threadIdx.x & 15) == 0 && t < M) parts[part * T + t] = make_float2(best, __int_as_float(arg));
    }
  }
};

// Backward step 1: dZ[t][v] = c_t (1[v == y_t] - exp(z - lse_t)), fp32, panel-local rows.
struct EpiDzF32 {
  const int32_t* tokens;
  const float* lse;
  const float* coef;
  float* dZ;
  int64_t ld;
  __device__ void operator()(float (&acc)[4][4], int64_t m, int64_t n, int64_t M, int64_t N) const {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (m + i >= M) continue;
      const float c = coef[m + i], l = lse[m + i];
      const int64_t y = tokens[m + i];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (n + j < N) dZ[(m + i) * ld + n + j] = c * ((n + j == y ? 1.f : 0.f) - expf(acc[i][j] - l));
    }
  }
};

// Plain store or read-add-store of the tile into C[m][n].
struct EpiStoreF32 {
  float* C;
  int64_t ld;
  int accumulate;
  __device__ void operator()(float (&acc)[4][4], int64_t m, int64_t n, int64_t M, int64_t N) const {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (m + i < M && n + j < N) {
          float* p = C + (m + i) * ld + n + j;
          *p = accumulate ? *p + acc[i][j] : acc[i][j];
        }
  }
};

}  // namespace oapl
