// bf16 MFMA contractions of the OAPL loss head, hand-written for gfx950.
//
// One main loop serves all four dense steps of the path.  It computes a
// BM x BN tile of  C[m][n] = sum_k A[m][k] * B[n][k]  with both operands
// K-contiguous ("NT" form), fp32 accumulation in v_mfma_f32_32x32x16_bf16,
// operands streamed HBM/L2 -> LDS by direct-to-LDS buffer loads (no VGPR
// staging) into a two-stage, XOR-swizzled LDS ring.
//
// In the accumulator of a 32x32 MFMA block a lane owns ONE column n (lane%32)
// and 16 rows m: m = 8*(r/4) + 4*(lane/32) + r%4 for register r.  Every
// epilogue is built around that:
//   * forward (logits^T tile, M = vocabulary, N = tokens): the soft-max
//     reduction over the vocabulary is lane-local, so the streaming max / sum
//     needs no cross-lane traffic until the very end;
//   * outputs that are row-major in n with m contiguous (dZ[t][v], dH[t][j],
//     dW[v][j]) get 4 consecutive m per lane.
#pragma once

#include "common.hip.h"

namespace oapl {

template <int WM_, int WN_, int TM_, int TN_>
struct TileCfg {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
  static constexpr int NW = WM * WN;            // waves per workgroup
  static constexpr int NT = NW * 64;            // threads per workgroup
  static constexpr int BM = WM * TM * 32;
  static constexpr int BN = WN * TN * 32;
  static constexpr int BK = 64;                 // k-extent of one LDS stage
  static constexpr int ROW_BYTES = BK * 2;      // 128 B = 8 chunks of 16 B
  static constexpr int A_STAGE = BM * ROW_BYTES;
  static constexpr int B_STAGE = BN * ROW_BYTES;
  static constexpr int B_OFF = 2 * A_STAGE;
  static constexpr int MAIN_BYTES = 2 * (A_STAGE + B_STAGE);
  static constexpr int NIA = BM / (8 * NW);     // direct loads per wave and stage, A
  static constexpr int NIB = BN / (8 * NW);
  // bf16 staging tiles used by epilogues (16 B of padding per row).
  static constexpr int PITCH_NM = BM * 2 + 16;  // tile stored [n][m]
  static constexpr int PITCH_MN = BN * 2 + 16;  // tile stored [m][n]
  static constexpr int STAGE_NM = BN * PITCH_NM;
  static constexpr int STAGE_MN = BM * PITCH_MN;
  static constexpr int RED_BYTES = WM * BN * 8;
  static constexpr int LDS_BYTES =
      MAIN_BYTES > STAGE_NM ? (MAIN_BYTES > STAGE_MN ? MAIN_BYTES : STAGE_MN)
                            : (STAGE_NM > STAGE_MN ? STAGE_NM : STAGE_MN);
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split over waves");
  static_assert(RED_BYTES <= LDS_BYTES, "reduction scratch must fit");
};

typedef __attribute__((address_space(3))) char* lds_char_ptr;

// 16-byte chunk c of LDS row `row` lives at physical chunk c ^ ((row >> 1) & 7):
// 16 consecutive rows read at one logical chunk then hit 16 distinct 16-byte
// bank groups (rows alternate between the two 128-byte halves of the 256-byte
// bank line, and the XOR spreads each half over its 8 groups).
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

template <class C>
struct Mainloop {
  __amdgpu_buffer_rsrc_t ra, rb;
  int voffA[C::NIA], voffB[C::NIB];   // per-lane byte offsets of this lane's chunk in the A / B tile
  int chunkA[C::NIA], chunkB[C::NIB]; // logical 16-byte chunk index (0..7) the lane fetches
  int rdA[4], rdB[4];                 // LDS byte offsets of this lane's operand fragment for k-step 0..3
  int wave, lane;

  // lda / ldb in elements.  Offsets depend only on the leading dimensions and
  // the lane, so one setup serves every tile of a kernel.
  __device__ __forceinline__ void setup(int64_t lda, int64_t ldb) {
    const int tid = threadIdx.x;
    // the wave index feeds LDS base addresses that must live in scalar registers
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    lane = tid & 63;
    const int wm = wave / C::WN, wn = wave % C::WN;
#pragma unroll
    for (int i = 0; i < C::NIA; ++i) {
      const int row = (i * C::NW + wave) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz(row);
      chunkA[i] = c;
      voffA[i] = (int)(row * lda * 2 + c * 16);
    }
#pragma unroll
    for (int i = 0; i < C::NIB; ++i) {
      const int row = (i * C::NW + wave) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz(row);
      chunkB[i] = c;
      voffB[i] = (int)(row * ldb * 2 + c * 16);
    }
    const int rowA = wm * C::TM * 32 + (lane & 31);
    const int rowB = wn * C::TN * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = 2 * ks + (lane >> 5);
      rdA[ks] = rowA * C::ROW_BYTES + ((c ^ swz(rowA)) << 4);
      rdB[ks] = C::B_OFF + rowB * C::ROW_BYTES + ((c ^ swz(rowB)) << 4);
    }
  }

  // A tile: rows [0, rows_valid) of a row-major matrix starting at `base`
  // (already moved to the tile's first row, k = 0).  Rows past rows_valid and
  // anything past the buffer read as zero (buffer range check).
  __device__ __forceinline__ void set_a(const bf16_t* base, int64_t rows_valid, int64_t lda) {
    const int64_t rv = rows_valid < C::BM ? (rows_valid < 0 ? 0 : rows_valid) : C::BM;
    // num_records must sit in scalar registers (the clamp above may be done on the vector ALU)
    ra = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, __builtin_amdgcn_readfirstlane((int)(rv * lda * 2)), 0x00020000);
  }
  __device__ __forceinline__ void set_b(const bf16_t* base, int64_t rows_valid, int64_t ldb) {
    const int64_t rv = rows_valid < C::BN ? (rows_valid < 0 ? 0 : rows_valid) : C::BN;
    rb = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, __builtin_amdgcn_readfirstlane((int)(rv * ldb * 2)), 0x00020000);
  }

  // Starts the direct-to-LDS loads of the k-tile beginning at element k0 into
  // `stage`.  `K` is only looked at when the k-tile is the ragged last one.
  template <int STAGE>
  __device__ __forceinline__ void issue(lds_char_ptr smem, int k0, int K) {
    const int soff = k0 * 2;
    if (k0 + C::BK <= K) {
#pragma unroll
      for (int i = 0; i < C::NIA; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            ra, (lds_void_ptr)(smem + STAGE * C::A_STAGE + (i * C::NW + wave) * 1024), 16, voffA[i], soff, 0, 0);
#pragma unroll
      for (int i = 0; i < C::NIB; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rb, (lds_void_ptr)(smem + C::B_OFF + STAGE * C::B_STAGE + (i * C::NW + wave) * 1024), 16, voffB[i], soff, 0, 0);
    } else {
      // ragged k-tile: chunks at or past K are sent out of range and come back as zeros
#pragma unroll
      for (int i = 0; i < C::NIA; ++i) {
        const int v = (k0 + chunkA[i] * 8 < K) ? voffA[i] : 0x7FFFFF00;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            ra, (lds_void_ptr)(smem + STAGE * C::A_STAGE + (i * C::NW + wave) * 1024), 16, v, soff, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < C::NIB; ++i) {
        const int v = (k0 + chunkB[i] * 8 < K) ? voffB[i] : 0x7FFFFF00;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rb, (lds_void_ptr)(smem + C::B_OFF + STAGE * C::B_STAGE + (i * C::NW + wave) * 1024), 16, v, soff, 0, 0);
      }
    }
  }

  template <int STAGE>
  __device__ __forceinline__ void compute(lds_char_ptr smem, f32x16 (&acc)[C::TM][C::TN]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 a[C::TM], b[C::TN];
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
        a[i] = *(const __attribute__((address_space(3))) bf16x8*)(smem + STAGE * C::A_STAGE + rdA[ks] + i * 32 * C::ROW_BYTES);
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
        b[j] = *(const __attribute__((address_space(3))) bf16x8*)(smem + STAGE * C::B_STAGE + rdB[ks] + j * 32 * C::ROW_BYTES);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  static __device__ __forceinline__ void wait_loads_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's direct-to-LDS loads have landed
    __syncthreads();
  }

  // acc += A_tile * B_tile^T over k in [0, K).  Ends with a barrier: on return
  // every wave is done reading LDS, so the caller may reuse it at once.
  __device__ __forceinline__ void run(lds_char_ptr smem, int K, f32x16 (&acc)[C::TM][C::TN]) {
    const int nk = (K + C::BK - 1) / C::BK;
    issue<0>(smem, 0, K);
    wait_loads_and_sync();
    // Two k-tiles per trip so the stage index is a compile-time constant; an
    // odd last k-tile is peeled off below.  The accumulators flow straight
    // through (no early exit inside the loop).
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
      issue<1>(smem, (kt + 1) * C::BK, K);
      compute<0>(smem, acc);
      wait_loads_and_sync();
      if (kt + 2 < nk) issue<0>(smem, (kt + 2) * C::BK, K);
      compute<1>(smem, acc);
      wait_loads_and_sync();
    }
    if (kt < nk) {
      compute<0>(smem, acc);
      __syncthreads();
    }
  }
};

template <class C>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[C::TM][C::TN]) {
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

// Row offset (within the wave's 32*TM rows, before the lane-half term) of
// accumulator register r of m-block i.
__device__ __forceinline__ constexpr int acc_row(int i, int r) { return i * 32 + 8 * (r >> 2) + (r & 3); }

// ---------------------------------------------------------------------------
// bf16 staging of an accumulator tile through LDS for 16-byte coalesced stores
// ---------------------------------------------------------------------------

// LDS tile [n][m]: each lane writes 4 consecutive m (8 bytes) per step.
template <class C>
__device__ __forceinline__ void stage_nm(lds_char_ptr smem, const f32x16 (&acc)[C::TM][C::TN]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_l = wn * C::TN * 32 + j * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m_l = wm * C::TM * 32 + i * 32 + 8 * q + 4 * h;
        bf16x4 v;
        v[0] = (bf16_t)acc[i][j][4 * q + 0];
        v[1] = (bf16_t)acc[i][j][4 * q + 1];
        v[2] = (bf16_t)acc[i][j][4 * q + 2];
        v[3] = (bf16_t)acc[i][j][4 * q + 3];
        *(__attribute__((address_space(3))) bf16x4*)(smem + n_l * C::PITCH_NM + m_l * 2) = v;
      }
  }
}

// out[n][m] (row pitch ldo elements, pointer already at the tile origin):
// rows n < n_rows, columns m < m_cols (m_cols a multiple of 8).
template <class C>
__device__ __forceinline__ void store_nm(lds_char_ptr smem, bf16_t* out, int64_t ldo, int64_t n_rows, int64_t m_cols) {
  constexpr int CH = C::BM / 8;
  for (int idx = threadIdx.x; idx < C::BN * CH; idx += C::NT) {
    const int n_l = idx / CH, ch = idx % CH;
    if (n_l < n_rows && ch * 8 < m_cols) {
      const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + n_l * C::PITCH_NM + ch * 16);
      *(u32x4*)(out + (int64_t)n_l * ldo + ch * 8) = v;
    }
  }
}

// LDS tile [m][n]: 2-byte writes, consecutive lanes write consecutive n.
template <class C>
__device__ __forceinline__ void stage_mn(lds_char_ptr smem, const f32x16 (&acc)[C::TM][C::TN]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_l = wn * C::TN * 32 + j * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m_l = wm * C::TM * 32 + acc_row(i, r) + 4 * h;
        *(__attribute__((address_space(3))) bf16_t*)(smem + m_l * C::PITCH_MN + n_l * 2) = (bf16_t)acc[i][j][r];
      }
  }
}

template <class C>
__device__ __forceinline__ void store_mn(lds_char_ptr smem, bf16_t* out, int64_t ldo, int64_t m_rows, int64_t n_cols) {
  constexpr int CH = C::BN / 8;
  for (int idx = threadIdx.x; idx < C::BM * CH; idx += C::NT) {
    const int m_l = idx / CH, ch = idx % CH;
    if (m_l < m_rows && ch * 8 < n_cols) {
      const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + m_l * C::PITCH_MN + ch * 16);
      *(u32x4*)(out + (int64_t)m_l * ldo + ch * 8) = v;
    }
  }
}

// Tile coordinates for a logical workgroup id: tiles are walked in strips of
// SN tiles along n, m fastest within a strip row, so that the ~32 workgroups
// resident on one XCD form a (32 / SN) x SN patch and share operand panels.
template <int SN>
__device__ __forceinline__ void strip_tile(int L, int MT, int NTl, int& mt, int& nt) {
  const int per_strip = SN * MT;
  const int strip = L / per_strip;
  const int rem = L - strip * per_strip;
  const int width = (NTl - strip * SN) < SN ? (NTl - strip * SN) : SN;
  mt = rem / width;
  nt = strip * SN + rem % width;
}

// ---------------------------------------------------------------------------
// Forward: logits^T tiles with a streaming (online) log-sum-exp over the
// vocabulary.  The T x V logits never leave registers.
//   A = W [V, d]  (M = vocabulary),  B = H [T, d]  (N = tokens),  K = d.
// One workgroup owns one token tile and walks a contiguous range ("split") of
// vocabulary tiles, carrying per token the running pair
//     m2 = max_v z * log2(e),   s = sum_v 2^(z * log2(e) - m2)
// and merging a new tile by the usual rescaling rule.  It writes one (m2, s)
// pair per token and split; a later kernel merges the splits.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_fwd_lse(const bf16_t* __restrict__ W, const bf16_t* __restrict__ H, int V, int64_t T, int d,
          int n_splits, float2* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;

  const int n_tiles = (int)((T + C::BN - 1) / C::BN);
  const int total = n_tiles * n_splits;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  const int nt = L / n_splits, split = L % n_splits;
  const int MT = (V + C::BM - 1) / C::BM;
  const int mt_begin = (int)((int64_t)split * MT / n_splits);
  const int mt_end = (int)((int64_t)(split + 1) * MT / n_splits);
  const int64_t n0 = (int64_t)nt * C::BN;

  Mainloop<C> ml;
  ml.setup(d, d);
  ml.set_b(H + n0 * d, T - n0, d);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;

  float m2[C::TN], s[C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) { m2[j] = kNegHuge; s[j] = 0.f; }

  f32x16 acc[C::TM][C::TN];
  for (int mt = mt_begin; mt < mt_end; ++mt) {
    const int m0 = mt * C::BM;
    ml.set_a(W + (int64_t)m0 * d, V - m0, d);
    zero_acc<C>(acc);
    ml.run(smem, d, acc);

    if (m0 + C::BM > V) {  // ragged last vocabulary tile: rows >= V do not exist
      const int row0 = m0 + wm * C::TM * 32 + 4 * h;
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (row0 + acc_row(i, r) >= V) {
#pragma unroll
            for (int j = 0; j < C::TN; ++j) acc[i][j][r] = -__builtin_inff();
          }
    }
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      float mx = -__builtin_inff();
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r]);
      const float mnew = fmaxf(m2[j], mx * kLog2e);
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r], kLog2e, -mnew));
      s[j] = s[j] * __builtin_amdgcn_exp2f(m2[j] - mnew) + sum;
      m2[j] = mnew;
    }
  }

  // merge the two lane halves (same token, different vocabulary rows) ...
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const float mo = __shfl_xor(m2[j], 32, 64), so = __shfl_xor(s[j], 32, 64);
    const float M = fmaxf(m2[j], mo);
    s[j] = s[j] * __builtin_amdgcn_exp2f(m2[j] - M) + so * __builtin_amdgcn_exp2f(mo - M);
    m2[j] = M;
  }
  // ... then the WM waves stacked along the vocabulary, through LDS.
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  __attribute__((address_space(3))) f32x2* red = (__attribute__((address_space(3))) f32x2*)smem;
  if (h == 0) {
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
      red[wm * C::BN + wn * C::TN * 32 + j * 32 + lane] = f32x2{m2[j], s[j]};
  }
  __syncthreads();
  for (int n_l = threadIdx.x; n_l < C::BN; n_l += C::NT) {
    if (n0 + n_l < T) {
      f32x2 a = red[n_l];
#pragma unroll
      for (int w = 1; w < C::WM; ++w) {
        const f32x2 b = red[w * C::BN + n_l];
        const float M = fmaxf(a.x, b.x);
        a.y = a.y * __builtin_amdgcn_exp2f(a.x - M) + b.y * __builtin_amdgcn_exp2f(b.x - M);
        a.x = M;
      }
      partials[(int64_t)split * T + n0 + n_l] = make_float2(a.x, a.y);
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, step 1: recompute a logits^T tile and turn it into the gradient
// with respect to the logits.  With p = softmax(z_t) and f_t = c_t (1 - p_{t,y_t}),
//     dL/dz[t][v] = c_t (1[v == y_t] - p[t][v]) = f_t * G[t][v],
//     G[t][y_t] = 1,   G[t][v] = -p[t][v] / (1 - p[t][y_t])  otherwise.
// G is what is rounded to bf16: its one-hot entry is exact, and the remaining
// entries (tiny, with uncorrelated roundings) carry no common factor, so no
// rounding error is shared by all tokens of a rollout.  The fp32 row factor f_t
// is applied by the consumers: dH = diag(f) (G W), dW = G^T (diag(f) H).
// G is written twice, for one panel of Tp token rows:
//     dZ  [Tp][Vp]  (v contiguous)   -> dH
//     dZT [V][Tp]   (t contiguous)   -> dW
// Rows / columns outside the valid ranges are written as zeros so the
// consumers can read whole tiles.
//   A = W [V, d] (M = vocabulary), B = H panel [n_valid, d] (N = tokens).
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dz(const bf16_t* __restrict__ W, const bf16_t* __restrict__ Hp, int V, int64_t n_valid, int d,
         const int32_t* __restrict__ tokens, const float* __restrict__ lse2, const float* __restrict__ inv_omp,
         bf16_t* __restrict__ dZ, int64_t Vp, bf16_t* __restrict__ dZT, int64_t Tp) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;

  const int MT = (V + C::BM - 1) / C::BM;
  const int NTl = (int)((n_valid + C::BN - 1) / C::BN);
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<8>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int64_t n0 = (int64_t)nt * C::BN;

  Mainloop<C> ml;
  ml.setup(d, d);
  ml.set_a(W + (int64_t)m0 * d, V - m0, d);
  ml.set_b(Hp + n0 * d, n_valid - n0, d);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.run(smem, d, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
  const int wave_row0 = m0 + wm * C::TM * 32;      // first vocabulary row of this wave
  const int row0 = wave_row0 + 4 * h;              // ... of this lane

  bool any_hit = false;
  float ninv[C::TN], l2[C::TN];   // -1 / (1 - p_y), lse in the exp2 domain
  int ytok[C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int64_t n = n0 + wn * C::TN * 32 + j * 32 + (lane & 31);
    const bool ok = n < n_valid;
    ninv[j] = ok ? -inv_omp[n] : 0.f;
    l2[j] = ok ? lse2[n] : 0.f;
    ytok[j] = ok ? tokens[n] : -1;
    any_hit |= (unsigned)(ytok[j] - wave_row0) < (unsigned)(C::TM * 32);
  }
#pragma unroll
  for (int j = 0; j < C::TN; ++j)
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r], kLog2e, -l2[j]));
        acc[i][j][r] = p * ninv[j];
      }
  // the one-hot term: at most one element per token over the whole vocabulary,
  // so only waves whose row range contains a sampled token look for it
  if (__builtin_amdgcn_ballot_w64(any_hit) != 0) {
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      const int rel = ytok[j] - row0;
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (rel == acc_row(i, r)) acc[i][j][r] = ninv[j] != 0.f ? 1.f : 0.f;
    }
  }
  if (m0 + C::BM > V) {  // rows past the vocabulary carry exp2(0 - lse2) garbage: clear them
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (row0 + acc_row(i, r) >= V) {
#pragma unroll
          for (int j = 0; j < C::TN; ++j) acc[i][j][r] = 0.f;
        }
  }

  // dZ[t][v]: stage [n][m], then 16-byte row stores
  stage_nm<C>(smem, acc);
  __syncthreads();
  {
    const int64_t rows = n_valid - n0;
    const int64_t cols = Vp - m0;
    store_nm<C>(smem, dZ + n0 * Vp + m0, Vp, rows, cols);
  }
  __syncthreads();
  // dZT[v][t]: stage [m][n]; all BN columns are written (zeros past n_valid)
  stage_mn<C>(smem, acc);
  __syncthreads();
  store_mn<C>(smem, dZT + (int64_t)m0 * Tp + n0, Tp, (int64_t)V - m0, C::BN);
}

// ---------------------------------------------------------------------------
// Backward, step 2: dH[t][j] = f_t * sum_v G[t][v] * W[v][j]
//   A = WT [d][Vp] (M = hidden index j), B = dZ panel [n_valid][Vp] (N = tokens), K = V.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dh(const bf16_t* __restrict__ WT, const bf16_t* __restrict__ dZ, int d, int64_t n_valid, int V, int64_t Vp,
         const float* __restrict__ row_factor /* f_t, panel-local */, bf16_t* __restrict__ dH /* panel's first row */) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;

  const int MT = (d + C::BM - 1) / C::BM;
  const int NTl = (int)((n_valid + C::BN - 1) / C::BN);
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<8>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int64_t n0 = (int64_t)nt * C::BN;

  Mainloop<C> ml;
  ml.setup(Vp, Vp);
  ml.set_a(WT + (int64_t)m0 * Vp, d - m0, Vp);
  ml.set_b(dZ + n0 * Vp, n_valid - n0, Vp);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.run(smem, V, acc);

  {
    const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) % C::WN;
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      const int64_t n = n0 + wn * C::TN * 32 + j * 32 + (lane & 31);
      const float f = n < n_valid ? row_factor[n] : 0.f;
#pragma unroll
      for (int i = 0; i < C::TM; ++i) acc[i][j] *= f;
    }
  }
  stage_nm<C>(smem, acc);
  __syncthreads();
  store_nm<C>(smem, dH + n0 * d + m0, d, n_valid - n0, (int64_t)d - m0);
}

// ---------------------------------------------------------------------------
// Backward, step 3: dW[v][j] (+)= sum_t G[t][v] * (f_t H[t][j])
//   A = HT [d][Tp] = (diag(f) H)^T (M = hidden index j), B = dZT [V][Tp] (N = vocabulary), K = Kt
//   (the panel's token count rounded up to the tile; the padding is zeros).
// fp32 output written straight from the accumulators: 4 consecutive j per lane.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dw(const bf16_t* __restrict__ HT, const bf16_t* __restrict__ dZT, int d, int V, int64_t Tp, int Kt,
         float* __restrict__ dW, int accumulate) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;

  const int MT = (d + C::BM - 1) / C::BM;
  const int NTl = (V + C::BN - 1) / C::BN;
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<8>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int n0 = nt * C::BN;

  Mainloop<C> ml;
  ml.setup(Tp, Tp);
  ml.set_a(HT + (int64_t)m0 * Tp, d - m0, Tp);
  ml.set_b(dZT + (int64_t)n0 * Tp, V - n0, Tp);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.run(smem, Kt, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n = n0 + wn * C::TN * 32 + j * 32 + (lane & 31);
    if (n >= V) continue;
    float* row = dW + (int64_t)n * d;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m = m0 + wm * C::TM * 32 + i * 32 + 8 * q + 4 * h;
        if (m < d) {  // d is a multiple of 8, so the 4 lanes of a quad are in or out together
          f32x4 v;
          v[0] = acc[i][j][4 * q + 0];
          v[1] = acc[i][j][4 * q + 1];
          v[2] = acc[i][j][4 * q + 2];
          v[3] = acc[i][j][4 * q + 3];
          f32x4* p = (f32x4*)(row + m);
          if (accumulate) v += *p;
          *p = v;
        }
      }
  }
}

}  // namespace oapl
