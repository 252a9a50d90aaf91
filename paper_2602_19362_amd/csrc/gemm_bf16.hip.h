// bf16 MFMA contractions of the OAPL loss head, hand-written for gfx950.
//
// One main loop serves all dense steps of the path.  It computes a
// 256 x 384 tile of  C[m][n] = sum_k A[m][k] * B[n][k]  with both operands
// k-contiguous, fp32 accumulation in v_mfma_f32_32x32x16_bf16, operands
// streamed L2 -> LDS by direct-to-LDS buffer loads (no VGPR staging) into a
// two-stage, XOR-swizzled LDS ring that fills the CU's 160 KB, 8 wavefronts
// (two per SIMD, so one wavefront's waits are covered by the other's MFMAs),
// each a 64 x 192 patch (192 accumulator registers per lane).  The tile is as
// large as registers and LDS allow: operand delivery from L2 is what the loop
// waits for, and 256 x 384 needs 17 % fewer operand bytes per flop than 256 x 256.
//
// Operand layout in HBM ("packed"): a matrix with R rows and K columns is
// stored as blocks of RB rows x 64 columns (RB = 256 for the m-side operand,
// 384 for the n-side operand), block (rt, kt) at byte offset
// (rt * n_kt + kt) * RB * 128, row-major inside the block (128 B per row), zero
// padded to whole blocks.  One k-step of one tile is then ONE contiguous 32 / 48 KiB
// read per operand (full 128-byte lines, sequential DRAM pages), instead of
// row fragments spread over a 2 MB .. 80 MB span, and ragged edges need no
// special case in the loads: padding is zeros.  The caller's row-major H and W
// are packed once per call by k_pack_rows / k_pack_transposed; the kernels
// that produce intermediate operands write them packed directly.
//
// In the accumulator of a 32x32 MFMA block a lane owns ONE column n (lane%32)
// and 16 rows m: m = 8*(r/4) + 4*(lane/32) + r%4 for register r.  Every
// epilogue is built around that:
//   * forward (logits^T tile, M = vocabulary, N = tokens): the soft-max
//     reduction over the vocabulary is lane-local, so the streaming max / sum
//     needs no cross-lane traffic until the very end;
//   * outputs with m contiguous (G[t][v], dH[t][j], dW[v][j]) get 4
//     consecutive m per lane.
//
// The bodies of the tile kernels are compiled in the device pass only (__HIP_DEVICE_COMPILE__).
// They use instructions that gfx950 alone has (16-byte direct-to-LDS loads, the 32x32x16 bf16
// MFMA, v_permlane32_swap).  The host pass needs nothing but the signatures, for its launch stubs;
// it checks builtins against a generic target, keeps its complaints about device code to itself,
// and has been seen to drop a kernel's launch stub, or to refuse a launch as "no matching
// function", after an unrelated edit of the main loop.
#pragma once

#include "common.hip.h"
#include "rng.hip.h"

namespace oapl {


template <int WM_, int WN_, int TM_, int TN_, int NS_>
struct TileCfg {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
  static constexpr int NW = WM * WN;            // waves per workgroup
  static constexpr int NT = NW * 64;            // threads per workgroup
  static constexpr int BM = WM * TM * 32;
  static constexpr int BN = WN * TN * 32;
  static constexpr int BK = kPackK;             // k-extent of one LDS stage
  static constexpr int NS = NS_;                // LDS stages in the ring
  static constexpr int KSTEPS = BK / 16;        // MFMA k-steps per stage
  static constexpr int ROW_BYTES = kPackRowBytes;
  static constexpr int STAGE_A = BM * ROW_BYTES;   // one stage of the m-side operand
  static constexpr int STAGE_B = BN * ROW_BYTES;   // ... of the n-side operand
  static constexpr int SLOT = STAGE_A + STAGE_B;   // one ring slot: the m-side block, then the n-side block
  static constexpr int MAIN_BYTES = NS * (STAGE_A + STAGE_B);
  static constexpr int NI_A = BM / (8 * NW);    // direct loads per wave and stage (8 rows each), m-side operand
  static constexpr int NI_B = BN / (8 * NW);    // ... n-side operand
  // bf16 staging tiles used by epilogues (16 B of padding per row).  A whole tile does not fit
  // the LDS, so epilogues stage it in chunks: [n][m] by wave column (BN / WN rows of n at a
  // time), [m][n] by pairs of wave rows (BM / MN_CHUNKS rows of m at a time).
  static constexpr int PITCH_NM = BM * 2 + 16;  // tile stored [n][m]
  static constexpr int PITCH_MN = BN * 2 + 16;  // tile stored [m][n]
  static constexpr int NM_CHUNKS = WN, NM_ROWS = BN / WN;
  static constexpr int MN_CHUNKS = WM >= 2 ? WM / 2 : 1, MN_ROWS = BM / MN_CHUNKS;
  static constexpr int STAGE_NM = NM_ROWS * PITCH_NM;
  static constexpr int STAGE_MN = MN_ROWS * PITCH_MN;
  static constexpr int RED_BYTES = WM * BN * 8;
  static constexpr int LDS_BYTES =
      MAIN_BYTES > STAGE_NM ? (MAIN_BYTES > STAGE_MN ? MAIN_BYTES : STAGE_MN)
                            : (STAGE_NM > STAGE_MN ? STAGE_NM : STAGE_MN);
  static_assert(BM == kPackRowsA, "the m side of a tile is one packed block tall");
  static_assert(NS == 2, "ring size");
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "block rows must split over waves");
  static_assert(RED_BYTES + RED_BYTES / 2 <= LDS_BYTES, "reduction scratch must fit");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
};

typedef __attribute__((address_space(3))) char* lds_char_ptr;

// s_waitcnt immediate for "at most n vector-memory operations still outstanding" (gfx9 encoding:
// vmcnt in bits [3:0] and [15:14]; expcnt and lgkmcnt fields left at their maximum = no wait).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// Workgroup barrier for LDS hand-offs in epilogues: waits for this wave's LDS operations only.
// __syncthreads() also waits for the wave's outstanding global stores (vmcnt(0)), i.e. for a round
// trip to memory at every hand-off; the data of a store that has been issued is already out of the
// registers, so nothing here needs that wait.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0); vmcnt and expcnt fields at their maximum = no wait
  __builtin_amdgcn_s_barrier();
}

template <class C>
struct Mainloop {
  // 16-byte chunk c of LDS row `row` lives at physical chunk c ^ ((row >> 1) & 7).  The operand
  // fetch of 16 consecutive rows at one logical chunk then touches 16 distinct 16-byte bank groups:
  // two consecutive rows fill one 256-byte bank line, and the XOR walks each half's 8 slots.
  static __device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

  __amdgpu_buffer_rsrc_t ra, rb;
  int voff;                           // per-lane byte offset of this lane's chunk inside the first 8 rows a wave loads
  // LDS byte offsets of this lane's operand fragments at k-step 0 of ring slot 0.  K-step ks sits at the
  // same offset with address bits 5..6 flipped by ks (the swizzle is an XOR on the 16-byte chunk index and
  // the k-step is bits 1..2 of that index); deriving it where it is used costs one XOR per operand and
  // k-step and saves six registers over a table.
  int rdA0, rdB0;
  int wave, lane;

  __device__ __forceinline__ void setup() {
    const int tid = threadIdx.x;
    // the wave index feeds LDS base addresses that must live in scalar registers
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    lane = tid & 63;
    const int wm = wave / C::WN, wn = wave % C::WN;
    // One wave-wide load covers 8 block rows; lane l lands at LDS byte l*16 of that 1 KiB.  Load i of
    // a wave takes rows (i * NW + wave) * 8 ..: 8 * NW rows further per i, which leaves the swizzle
    // term unchanged (8 * NW is a multiple of 16), so one lane offset serves every i and both operands;
    // the i term goes into the scalar offset.
    static_assert((8 * C::NW) % 16 == 0, "swizzle must repeat from one load of a wave to the next");
    {
      const int row = wave * 8 + (lane >> 3);
      voff = row * C::ROW_BYTES + (((lane & 7) ^ swz(row)) << 4);
    }
    const int rowA = wm * C::TM * 32 + (lane & 31);
    const int rowB = wn * C::TN * 32 + (lane & 31);
    static_assert(C::KSTEPS == 4, "k-step index = chunk bits 1..2");
    const int c0 = lane >> 5;
    rdA0 = rowA * C::ROW_BYTES + ((c0 ^ swz(rowA)) << 4);
    rdB0 = C::STAGE_A + rowB * C::ROW_BYTES + ((c0 ^ swz(rowB)) << 4);
  }

  // The empty asm keeps the compiler from hoisting the per-k-step addresses out of the loop (back into a table).
  static __device__ __forceinline__ int fresh(int x) {
    asm volatile("" : "+v"(x));
    return x;
  }

  // Operand = one row-tile strip of a packed matrix: n_kt consecutive blocks of 32 KiB (A) / 48 KiB (B).
  __device__ __forceinline__ void set_a(const bf16_t* strip, int n_kt) {
    ra = __builtin_amdgcn_make_buffer_rsrc((void*)strip, 0, n_kt * C::STAGE_A, 0x00020000);
  }
  __device__ __forceinline__ void set_b(const bf16_t* strip, int n_kt) {
    rb = __builtin_amdgcn_make_buffer_rsrc((void*)strip, 0, n_kt * C::STAGE_B, 0x00020000);
  }

  // Starts the direct-to-LDS loads of k-block kt into ring slot STAGE (a literal at the call sites,
  // so the LDS addresses fold to constants once inlined).
  __device__ __forceinline__ void issue(const int STAGE, lds_char_ptr smem, int kt) {
#pragma unroll
    for (int i = 0; i < C::NI_A; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          ra, (lds_void_ptr)(smem + STAGE * C::SLOT + (i * C::NW + wave) * 1024), 16, voff,
          kt * C::STAGE_A + i * C::NW * 1024, 0, 0);
#pragma unroll
    for (int i = 0; i < C::NI_B; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rb, (lds_void_ptr)(smem + STAGE * C::SLOT + C::STAGE_A + (i * C::NW + wave) * 1024), 16, voff,
          kt * C::STAGE_B + i * C::NW * 1024, 0, 0);
  }

  __device__ __forceinline__ void compute(const int STAGE, lds_char_ptr smem, f32x16 (&acc)[C::TM][C::TN]) {
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) {
      bf16x8 a[C::TM], b[C::TN];
      const int ra_ks = fresh(rdA0) ^ (ks << 5), rb_ks = fresh(rdB0) ^ (ks << 5);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
        a[i] = *(const __attribute__((address_space(3))) bf16x8*)(smem + STAGE * C::SLOT + ra_ks + i * 32 * C::ROW_BYTES);
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
        b[j] = *(const __attribute__((address_space(3))) bf16x8*)(smem + STAGE * C::SLOT + rb_ks + j * 32 * C::ROW_BYTES);
      // all reads of a k-step are issued before its first multiplication; the scheduler then overlaps
      // them with the previous k-step's last multiplications instead of starting every k-step by waiting
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // One k-block of the pipeline in ring slot S (a literal at the call sites): wait until the block's
  // loads have landed, barrier (which also tells that every wave is done with the other slot),
  // refill the other slot with the next block, multiply.  Branches are wave-uniform and touch no
  // accumulator.
  __device__ __forceinline__ void step(const int S, lds_char_ptr smem, int kt, int nk, f32x16 (&acc)[C::TM][C::TN]) {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    if (kt + 1 < nk) issue(S ^ 1, smem, kt + 1);
    compute(S, smem, acc);
  }

  // Starts a tile: k-block 0 into slot 0.  Every wave must be past its last LDS read of the
  // previous tile (finish() ends with a barrier).
  __device__ __forceinline__ void start(lds_char_ptr smem) { issue(0, smem, 0); }

  // k-blocks [k0, k1) of a tile with nk k-blocks in all (k0 even, after start() or an earlier steps()).
  // PRELOADED (with k0 = 0): k-block 1 was issued beforehand as well (start(), then issue(1, smem, 1) if the tile
  // has two blocks), by a caller whose work between two tiles leaves the LDS alone.  The first block then issues
  // nothing.  It waits for both blocks: waiting for the first alone (vmcnt = the second block's loads, and a bare
  // s_barrier, since __syncthreads() waits for every outstanding load itself) measured no different.
  template <bool PRELOADED = false>
  __device__ __forceinline__ void steps(lds_char_ptr smem, int k0, int k1, int nk, f32x16 (&acc)[C::TM][C::TN]) {
    int kt = k0;
    if (PRELOADED) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __syncthreads();
      compute(0, smem, acc);
      kt = 1;
      if (kt < k1) {
        step(1, smem, 1, nk, acc);
        kt = 2;
      }
    }
    for (; kt + 2 <= k1; kt += 2) {
      step(0, smem, kt, nk, acc);
      step(1, smem, kt + 1, nk, acc);
    }
    if (kt < k1) step(0, smem, kt, nk, acc);
  }

  // acc += A_tile * B_tile^T over k-blocks [0, nk) after start().  Ends with a barrier: on return
  // every wave is done reading LDS, so the caller may reuse it (or start() the next tile) at once.
  template <bool PRELOADED = false>
  __device__ __forceinline__ void finish(lds_char_ptr smem, int nk, f32x16 (&acc)[C::TM][C::TN]) {
    steps<PRELOADED>(smem, 0, nk, nk, acc);
    __syncthreads();
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
// bf16 staging of an accumulator tile through LDS for 16-byte coalesced stores.
// A whole tile is larger than the LDS, so it goes in chunks (see TileCfg); every
// stage_* call must be followed by a barrier, then the matching store_*, then a
// barrier before the next chunk is staged.
// ---------------------------------------------------------------------------

// LDS chunk [n][m] (n = the BN / WN columns of wave column `chunk`): each lane of those waves
// writes 4 consecutive m (8 bytes) per step.
template <class C>
__device__ __forceinline__ void stage_nm(lds_char_ptr smem, const f32x16 (&acc)[C::TM][C::TN], int chunk) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
  if (wn != chunk) return;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_l = j * 32 + (lane & 31);
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

// Staged chunk -> out[n][m] (row pitch ldo elements, pointer at the tile origin):
// rows n < n_rows, columns m < m_cols (m_cols a multiple of 8).
template <class C>
__device__ __forceinline__ void store_nm(lds_char_ptr smem, bf16_t* out, int64_t ldo, int64_t n_rows, int64_t m_cols,
                                         int chunk) {
  constexpr int CH = C::BM / 8;
  for (int idx = threadIdx.x; idx < C::NM_ROWS * CH; idx += C::NT) {
    const int n_l = idx / CH, ch = idx % CH;
    const int n = chunk * C::NM_ROWS + n_l;
    if (n < n_rows && ch * 8 < m_cols) {
      const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + n_l * C::PITCH_NM + ch * 16);
      *(u32x4*)(out + (int64_t)n * ldo + ch * 8) = v;
    }
  }
}

// Staged chunk [n][m] -> packed n-side matrix whose rows are the n index and whose k index is m:
// `strip` is block (n-tile, 0) of the destination, kb0 the first k-block (m0 / 64).  Whole rows are
// written (the packed buffers are padded to whole tiles; padding must be zeros).
template <class C>
__device__ __forceinline__ void store_nm_packed(lds_char_ptr smem, bf16_t* strip, int kb0, int chunk) {
  constexpr int CH = C::BM / 8;
  char* dst = (char*)strip + (int64_t)kb0 * C::STAGE_B;
  for (int idx = threadIdx.x; idx < C::NM_ROWS * CH; idx += C::NT) {
    const int n_l = idx / CH, ch = idx % CH;
    const int n = chunk * C::NM_ROWS + n_l;
    const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + n_l * C::PITCH_NM + ch * 16);
    *(u32x4*)(dst + (ch >> 3) * C::STAGE_B + n * kPackRowBytes + (ch & 7) * 16) = v;
  }
}

// LDS chunk [m][n] (m = the BM / MN_CHUNKS rows of wave rows chunk * WM / MN_CHUNKS ...): 2-byte
// writes, consecutive lanes write consecutive n.
template <class C>
__device__ __forceinline__ void stage_mn(lds_char_ptr smem, const f32x16 (&acc)[C::TM][C::TN], int chunk) {
  constexpr int WPC = C::WM / C::MN_CHUNKS;   // wave rows per chunk
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
  if (wm / WPC != chunk) return;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_l = wn * C::TN * 32 + j * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m_l = (wm % WPC) * C::TM * 32 + acc_row(i, r) + 4 * h;
        *(__attribute__((address_space(3))) bf16_t*)(smem + m_l * C::PITCH_MN + n_l * 2) = (bf16_t)acc[i][j][r];
      }
  }
}

// Staged chunk [m][n] -> packed n-side matrix whose rows are the m index (global row m0 + ...,
// blocks of BN rows) and whose k index is n: `base` is the destination matrix, n_kt its strip
// pitch in k-blocks, kb0 the first k-block (n0 / 64).
template <class C>
__device__ __forceinline__ void store_mn_packed(lds_char_ptr smem, bf16_t* base, int n_kt, int m0, int kb0, int chunk) {
  constexpr int CH = C::BN / 8;
  for (int idx = threadIdx.x; idx < C::MN_ROWS * CH; idx += C::NT) {
    const int m_l = idx / CH, ch = idx % CH;
    const int m = m0 + chunk * C::MN_ROWS + m_l;
    const int blk = m / C::BN, r = m - blk * C::BN;
    const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + m_l * C::PITCH_MN + ch * 16);
    char* dst = (char*)base + ((int64_t)blk * n_kt + kb0 + (ch >> 3)) * C::STAGE_B;
    *(u32x4*)(dst + r * kPackRowBytes + (ch & 7) * 16) = v;
  }
}

// Both packed copies of a finished tile: rows = n (tokens) with k = m, and rows = m with k = n.
template <class C>
__device__ __forceinline__ void store_tile_both_ways(lds_char_ptr smem, const f32x16 (&acc)[C::TM][C::TN],
                                                     bf16_t* Gp_strip, int m0, bf16_t* GTp, int gt_n_kt, int64_t n0) {
#pragma unroll 1
  for (int c = 0; c < C::NM_CHUNKS; ++c) {
    stage_nm<C>(smem, acc, c);
    __syncthreads();
    store_nm_packed<C>(smem, Gp_strip, m0 / kPackK, c);
    __syncthreads();
  }
#pragma unroll 1
  for (int c = 0; c < C::MN_CHUNKS; ++c) {
    stage_mn<C>(smem, acc, c);
    __syncthreads();
    store_mn_packed<C>(smem, GTp, gt_n_kt, m0, (int)(n0 / kPackK), c);
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// The same two packed copies from a tile already rounded to bf16 pairs:
// pk[i][j][p] holds rows acc_row(i, 2p) and acc_row(i, 2p) + 1 (low / high half) of column j.
// Half the registers of the fp32 tile, so nothing spills around the stores.
// ---------------------------------------------------------------------------

// 4 x 4 transpose of 16-byte pieces across the four lanes of a quad: lane q hands its piece c to
// lane c and ends up holding, as piece r, what lane r held as piece q.  Two butterfly steps
// (partner lane ^ 1, then lane ^ 2), each a select, a quad-permute DPP move and two selects per
// exchanged piece.  All four lanes of the quad must be active.
template <int CTRL, class V4>
__device__ __forceinline__ V4 quad_xchg(const V4 v) {
  V4 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const auto x = v[e];   // a copy: a vector element is not an object whose bytes can be reinterpreted in place
    r[e] = __builtin_bit_cast(decltype(x), __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
  }
  return r;
}
template <class V4>
__device__ __forceinline__ void quad_transpose(V4 (&p)[4]) {
  const bool b0 = (threadIdx.x & 1) != 0, b1 = (threadIdx.x & 2) != 0;
#pragma unroll
  for (int c = 0; c < 4; c += 2) {       // lane bit 0 <-> piece bit 0
    const V4 r = quad_xchg<0xB1 /* quad_perm 1,0,3,2 */>(b0 ? p[c] : p[c + 1]);
    p[c] = b0 ? r : p[c];
    p[c + 1] = b0 ? p[c + 1] : r;
  }
#pragma unroll
  for (int c = 0; c < 2; ++c) {          // lane bit 1 <-> piece bit 1
    const V4 r = quad_xchg<0x4E /* quad_perm 2,3,0,1 */>(b1 ? p[c] : p[c + 2]);
    p[c] = b1 ? r : p[c];
    p[c + 2] = b1 ? p[c + 2] : r;
  }
}

// Copy with rows = n, k = m, straight from registers.  A lane owns 4 consecutive m (8 bytes) of its
// row n per (i, q) and the other lane half owns the 8 bytes next to them.  The halves first trade
// registers (v_permlane32_swap: the lower half hands over its pieces q = 2, 3 and receives the
// upper half's q = 0, 1), after which each lane holds two 16-byte pieces per MFMA block row i, four
// in all: with its other half, the whole 128-byte line of row n in this k-block.  Stored as they are,
// every store instruction would scatter 16-byte pieces over 32 lines (measured: 43 bytes per write
// request over the kernel, where a request can carry 64).  So the four lanes of a quad, which hold four
// neighbouring rows, transpose their pieces first: lane q then holds piece q of each of the four
// rows, and every store instruction writes whole lines, 8 lanes per line (+2.7 % on the sweep).
// Destroys pk.  `strip` is block (n-tile, 0) of the destination, kb0 the first k-block (m0 / 64).
template <class C>
__device__ __forceinline__ void store_nm_packed_direct(uint32_t (&pk)[C::TM][C::TN][8], bf16_t* strip, int kb0) {
  static_assert(C::TM == 2 && C::TM * 32 == kPackK, "a wave row spans exactly one packed k-block: 4 pieces of 16 bytes per lane");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5, q = lane & 3;
  // piece q of a row sits at byte (q >> 1) * 64 + 32 h + 16 (q & 1) of its 128-byte line
  char* base = (char*)strip + (int64_t)(kb0 + wm) * C::STAGE_B + (q >> 1) * 64 + 32 * h + 16 * (q & 1);
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    u32x4 piece[4];
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      uint32_t a[4], b[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const auto r = __builtin_amdgcn_permlane32_swap(pk[i][j][e], pk[i][j][e + 4], false, false);
        a[e] = r[0];
        b[e] = r[1];
      }
      piece[2 * i] = u32x4{a[0], a[1], b[0], b[1]};
      piece[2 * i + 1] = u32x4{a[2], a[3], b[2], b[3]};
    }
    // the four lanes of a quad hold four neighbouring rows: after the transpose lane q holds piece q of
    // each of them, and every store instruction writes whole 128-byte lines (8 lanes per line)
    quad_transpose(piece);
    const int n_q = wn * C::TN * 32 + j * 32 + (lane & 28);
#pragma unroll
    for (int r = 0; r < 4; ++r) *(u32x4*)(base + (n_q + r) * kPackRowBytes) = piece[r];
  }
}

// LDS chunk [m][n] from the packed pairs: chunk i holds MFMA block row i of every wave row (32 rows
// each, WM * 32 rows in all), so all waves stage at once.  Neighbouring lanes (columns n, n + 1) swap
// halves so that each lane writes 4 bytes: the even lane row m (its own low half, the neighbour's
// low half), the odd lane row m + 1 (the neighbour's high half, its own high half).
template <class C>
__device__ __forceinline__ void stage_mn_pk(lds_char_ptr smem, const uint32_t (&pk)[C::TM][C::TN][8], const int i) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5, odd = lane & 1;
  // v_perm_b32 picks bytes from {neighbour (4..7), own (0..3)}
  const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_l = wn * C::TN * 32 + j * 32 + (lane & 31) - odd;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const uint32_t own = pk[i][j][p];
      const uint32_t nbr = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true);
      const uint32_t w = __builtin_amdgcn_perm(nbr, own, sel);
      const int m_l = wm * 32 + acc_row(0, 2 * p) + 4 * h + odd;
      *(__attribute__((address_space(3))) uint32_t*)(smem + m_l * C::PITCH_MN + n_l * 2) = w;
    }
  }
}

// Chunk i staged by stage_mn_pk -> packed n-side matrix whose rows are the m index (global row
// m0 + ..., blocks of BN rows) and whose k index is n; n_kt is the destination's strip pitch in
// k-blocks, kb0 the first k-block (n0 / 64).
template <class C>
__device__ __forceinline__ void store_mn_pk_packed(lds_char_ptr smem, bf16_t* base, int n_kt, int m0, int kb0, int i) {
  constexpr int CH = C::BN / 8;
  for (int idx = threadIdx.x; idx < C::WM * 32 * CH; idx += C::NT) {
    const int m_l = idx / CH, ch = idx % CH;
    const int m = m0 + (m_l >> 5) * (C::TM * 32) + i * 32 + (m_l & 31);
    const int blk = m / C::BN, r = m - blk * C::BN;
    const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(smem + m_l * C::PITCH_MN + ch * 16);
    char* dst = (char*)base + ((int64_t)blk * n_kt + kb0 + (ch >> 3)) * C::STAGE_B;
    *(u32x4*)(dst + r * kPackRowBytes + (ch & 7) * 16) = v;
  }
}

// Tile coordinates for a logical workgroup id: tiles are walked in strips of
// SN tiles along n, m fastest within a strip row, so that the ~32 workgroups
// resident on one XCD form a (32 / SN) x SN patch and share operand panels.
// The kernels use SN = 4: an 8 x 4 patch of 256 x 384 tiles needs 8 x 32 KB +
// 4 x 48 KB of operands per k-step, the least for 32 tiles (measured +1.5 %
// over 4 x 8, and 8 % over 2 x 16).
__device__ __forceinline__ void strip_tile(const int SN, int L, int MT, int NTl, int& mt, int& nt) {
  const int per_strip = SN * MT;
  const int strip = L / per_strip;
  const int rem = L - strip * per_strip;
  const int width = (NTl - strip * SN) < SN ? (NTl - strip * SN) : SN;
  mt = rem / width;
  nt = strip * SN + rem % width;
}
template <int SN>
__device__ __forceinline__ void strip_tile(int L, int MT, int NTl, int& mt, int& nt) {
  strip_tile(SN, L, MT, NTl, mt, nt);
}

// ---------------------------------------------------------------------------
// Forward: logits^T tiles with a streaming (online) log-sum-exp over the
// vocabulary.  The T x V logits never leave registers.
//   A = packed W [V, d]  (M = vocabulary),  B = packed H [T, d]  (N = tokens),  K = d.
// One workgroup owns one token tile and walks a contiguous range ("split") of
// vocabulary tiles, carrying per token the running pair
//     m2 = max_v z * log2(e),   s = sum_v 2^(z * log2(e) - m2)
// and merging a new tile by the usual rescaling rule.  The first k-block of
// the next vocabulary tile is requested before the current tile's epilogue.
// It writes one (m2, s) pair per token and split; a later kernel merges the
// splits.  With ENT it also carries u = sum_v 2^(z * log2(e) - m2) * z, from which
// the policy entropy follows as  lse - u / s  (one more FMA per logit).
// ---------------------------------------------------------------------------
template <class C, bool ENT>
__global__ void __launch_bounds__(C::NT)
k_fwd_lse(const bf16_t* __restrict__ Wp, const bf16_t* __restrict__ Hp, int V, int64_t T, int n_kt,
          int n_splits, int patch_tiles, float2* __restrict__ partials, float* __restrict__ upart, Gate gate) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;
  if (gate_closed(gate)) return;

  const int n_tiles = (int)((T + C::BN - 1) / C::BN);
  const int total = n_tiles * n_splits;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  // Consecutive logical ids walk `patch_tiles` token tiles first, then the vocabulary splits: the ~32
  // workgroups resident on one XCD are then patch_tiles token tiles x 32 / patch_tiles splits, which
  // walk their splits in step and share each W block patch_tiles ways (each H block is shared by the
  // splits of its token tile).  patch_tiles = 1 keeps one token tile's H strip to an XCD: every XCD
  // then streams all of W once per token tile, which is the better trade only while several H strips
  // would not fit its L2 (chosen on the host from the strip size).
  int split, nt;
  strip_tile(patch_tiles, L, n_splits, n_tiles, split, nt);
  const int MT = (V + C::BM - 1) / C::BM;
  const int mt_begin = (int)((int64_t)split * MT / n_splits);
  const int mt_end = (int)((int64_t)(split + 1) * MT / n_splits);
  const int64_t n0 = (int64_t)nt * C::BN;
  const int64_t strip_a = (int64_t)n_kt * (C::STAGE_A / 2), strip_b = (int64_t)n_kt * (C::STAGE_B / 2);

  Mainloop<C> ml;
  ml.setup();
  ml.set_b(Hp + nt * strip_b, n_kt);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;

  float m2[C::TN], s[C::TN], u[C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) { m2[j] = kNegHuge; s[j] = 0.f; u[j] = 0.f; }

  f32x16 acc[C::TM][C::TN];
  if (mt_begin < mt_end) {
    ml.set_a(Wp + mt_begin * strip_a, n_kt);
    ml.start(smem);
    if (n_kt > 1) ml.issue(1, smem, 1);
  }
  for (int mt = mt_begin; mt < mt_end; ++mt) {
    const int m0 = mt * C::BM;
    zero_acc<C>(acc);
    ml.template finish<true>(smem, n_kt, acc);
    if (mt + 1 < mt_end) {  // the epilogue below works in registers only: overlap it with the next tile's first loads
      ml.set_a(Wp + (mt + 1) * strip_a, n_kt);
      ml.start(smem);
      if (n_kt > 1) ml.issue(1, smem, 1);
    }

    if (m0 + C::BM > V) {  // ragged last vocabulary tile: rows >= V do not exist (their logits are 0, not -inf)
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
      float sum = 0.f, usum = 0.f;
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r], kLog2e, -mnew));
          sum += e;
          // masked rows hold -inf with e = 0: keep their product out (0 * inf)
          if (ENT) usum = __builtin_fmaf(e, e > 0.f ? acc[i][j][r] : 0.f, usum);
        }
      const float scale = __builtin_amdgcn_exp2f(m2[j] - mnew);
      s[j] = s[j] * scale + sum;
      if (ENT) u[j] = u[j] * scale + usum;
      m2[j] = mnew;
    }
  }

  // merge the two lane halves (same token, different vocabulary rows) ...
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const float mo = __shfl_xor(m2[j], 32, 64), so = __shfl_xor(s[j], 32, 64);
    const float M = fmaxf(m2[j], mo);
    const float fa = __builtin_amdgcn_exp2f(m2[j] - M), fb = __builtin_amdgcn_exp2f(mo - M);
    s[j] = s[j] * fa + so * fb;
    if (ENT) u[j] = u[j] * fa + __shfl_xor(u[j], 32, 64) * fb;
    m2[j] = M;
  }
  // ... then the WM waves stacked along the vocabulary, through LDS.
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  __attribute__((address_space(3))) f32x2* red = (__attribute__((address_space(3))) f32x2*)smem;
  __attribute__((address_space(3))) float* red_u = (__attribute__((address_space(3))) float*)(smem + C::RED_BYTES);
  if (h == 0) {
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      red[wm * C::BN + wn * C::TN * 32 + j * 32 + lane] = f32x2{m2[j], s[j]};
      if (ENT) red_u[wm * C::BN + wn * C::TN * 32 + j * 32 + lane] = u[j];
    }
  }
  __syncthreads();
  for (int n_l = threadIdx.x; n_l < C::BN; n_l += C::NT) {
    if (n0 + n_l < T) {
      f32x2 a = red[n_l];
      float ua = ENT ? red_u[n_l] : 0.f;
#pragma unroll
      for (int w = 1; w < C::WM; ++w) {
        const f32x2 b = red[w * C::BN + n_l];
        const float M = fmaxf(a.x, b.x);
        const float fa = __builtin_amdgcn_exp2f(a.x - M), fb = __builtin_amdgcn_exp2f(b.x - M);
        a.y = a.y * fa + b.y * fb;
        if (ENT) ua = ua * fa + red_u[w * C::BN + n_l] * fb;
        a.x = M;
      }
      partials[(int64_t)split * T + n0 + n_l] = make_float2(a.x, a.y);
      if (ENT) upart[(int64_t)split * T + n0 + n_l] = ua;
    }
  }
#endif
}

// ---------------------------------------------------------------------------
// Sampling (the data-generation step of Alg. 1, as a kernel on the same fused
// head): y_t = argmax_v (z_tv / temperature + g_tv), g a standard Gumbel variate
// drawn from Philox-4x32-10 with key = seed and counter (v / 4, t, 0), which is a
// draw from softmax(z_t / temperature).  Same streaming structure as the forward
// kernel: a workgroup owns a token tile and a split of the vocabulary tiles and
// carries per token the best (score, index) so far; the 4 consecutive vocabulary
// rows a lane owns in each accumulator quad are exactly one Philox block.
// Ties go to the smaller index.  Output: one (score, index) pair per token and
// split (index bit-cast into the pair's second float).
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_fwd_sample(const bf16_t* __restrict__ Wp, const bf16_t* __restrict__ Hp, int V, int64_t T, int n_kt, int n_splits,
             float inv_temperature, uint32_t seed_lo, uint32_t seed_hi, float2* __restrict__ partials) {
#if defined(__HIP_DEVICE_COMPILE__)
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
  const int64_t strip_a = (int64_t)n_kt * (C::STAGE_A / 2), strip_b = (int64_t)n_kt * (C::STAGE_B / 2);

  Mainloop<C> ml;
  ml.setup();
  ml.set_b(Hp + nt * strip_b, n_kt);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;

  float best[C::TN];
  int arg[C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) { best[j] = -__builtin_inff(); arg[j] = 0x7FFFFFFF; }

  f32x16 acc[C::TM][C::TN];
  if (mt_begin < mt_end) {
    ml.set_a(Wp + mt_begin * strip_a, n_kt);
    ml.start(smem);
    if (n_kt > 1) ml.issue(1, smem, 1);
  }
  for (int mt = mt_begin; mt < mt_end; ++mt) {
    const int m0 = mt * C::BM;
    zero_acc<C>(acc);
    ml.template finish<true>(smem, n_kt, acc);
    if (mt + 1 < mt_end) {
      ml.set_a(Wp + (mt + 1) * strip_a, n_kt);
      ml.start(smem);
      if (n_kt > 1) ml.issue(1, smem, 1);
    }
    const int row0 = m0 + wm * C::TM * 32 + 4 * h;
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      const int64_t t = n0 + wn * C::TN * 32 + j * 32 + (lane & 31);
      const uint32_t t_lo = (uint32_t)t, t_hi = (uint32_t)(t >> 32);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int v0 = row0 + i * 32 + 8 * q;          // multiple of 4: one Philox block
          uint32_t x[4];
          philox4x32_10((uint32_t)(v0 >> 2), t_lo, t_hi, 0u, seed_lo, seed_hi, x);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float sc = __builtin_fmaf(acc[i][j][4 * q + e], inv_temperature, gumbel_from_bits(x[e]));
            if (v0 + e < V && sc > best[j]) { best[j] = sc; arg[j] = v0 + e; }   // indices rise: strict > keeps the smallest
          }
        }
    }
  }

  // merge the two lane halves, then the WM waves stacked along the vocabulary (through LDS)
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const float so = __shfl_xor(best[j], 32, 64);
    const int io = __shfl_xor(arg[j], 32, 64);
    if (better(so, io, best[j], arg[j])) { best[j] = so; arg[j] = io; }
  }
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  __attribute__((address_space(3))) f32x2* red = (__attribute__((address_space(3))) f32x2*)smem;
  if (h == 0) {
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
      red[wm * C::BN + wn * C::TN * 32 + j * 32 + lane] = f32x2{best[j], __int_as_float(arg[j])};
  }
  __syncthreads();
  for (int n_l = threadIdx.x; n_l < C::BN; n_l += C::NT) {
    if (n0 + n_l < T) {
      f32x2 a = red[n_l];
#pragma unroll
      for (int w = 1; w < C::WM; ++w) {
        const f32x2 b = red[w * C::BN + n_l];
        if (better(b.x, __float_as_int(b.y), a.x, __float_as_int(a.y))) a = b;
      }
      partials[(int64_t)split * T + n0 + n_l] = make_float2(a.x, a.y);
    }
  }
#endif
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
// G is written twice, packed, for one panel of token rows:
//     Gp   rows = tokens,      k = vocabulary   -> B operand of the dH contraction
//     GTp  rows = vocabulary,  k = tokens       -> B operand of the dW contraction
// Entries outside the valid ranges are written as zeros (whole tiles are stored).
//   A = packed W (M = vocabulary), B = packed H, panel's first token tile (N = tokens).
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dz(const bf16_t* __restrict__ Wp, const bf16_t* __restrict__ Hp_panel, int V, int64_t n_valid, int n_kt,
         const int32_t* __restrict__ tokens, const float* __restrict__ lse2, const float* __restrict__ inv_omp,
         bf16_t* __restrict__ Gp, int g_n_kt, bf16_t* __restrict__ GTp, int gt_n_kt, Gate gate) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;
  if (gate_closed(gate)) return;

  const int MT = (V + C::BM - 1) / C::BM;
  const int NTl = (int)((n_valid + C::BN - 1) / C::BN);
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<4>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int64_t n0 = (int64_t)nt * C::BN;
  const int64_t strip_a = (int64_t)n_kt * (C::STAGE_A / 2), strip_b = (int64_t)n_kt * (C::STAGE_B / 2);

  Mainloop<C> ml;
  ml.setup();
  ml.set_a(Wp + mt * strip_a, n_kt);
  ml.set_b(Hp_panel + nt * strip_b, n_kt);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.start(smem);
  ml.finish(smem, n_kt, acc);

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

  // Gp: rows = tokens (n), k = vocabulary (m);  GTp: rows = vocabulary (m), k = tokens (n)
  store_tile_both_ways<C>(smem, acc, Gp + (int64_t)nt * g_n_kt * (C::STAGE_B / 2), m0, GTp, gt_n_kt, n0);
#endif
}

// ---------------------------------------------------------------------------
// Single-sweep variant of steps a1, a2 and a8: ONE pass over the logits serves
// both the log-sum-exp and the gradient.  The soft-max is written unnormalised
// against a per-token reference exponent ref2[t] that is known before the pass
// (an upper-bound-free guess: the largest of a sample of the row's logits, see
// k_sweep_ref), in the exp2 domain:
//     Pt[t][v] = 2^(z[t][v] * log2(e) - ref2[t])          (bf16, packed twice like G above)
//     spart[mt][t] = sum over the vocabulary tile mt of Pt[t][v]   (fp32, from the unrounded values)
// so that, with S_t = sum_mt spart[mt][t]:  lse_t = (ref2[t] + log2 S_t) ln 2  and
//     dL/dz[t][v] = c_t (1[v == y_t] - Pt[t][v] / S_t) = a_t * Gt[t][v],   a_t = -c_t / S_t,
//     Gt[t][v] = Pt[t][v]  (v != y_t),    Gt[t][y_t] = Pt[t][y_t] - S_t   (patched in by k_sweep_finish).
// The row factor a_t only exists once S_t and the rollout's residual are known, i.e. after the
// pass; it is applied by the same consumers as f_t above (dH epilogue, transposed H).  bf16 has
// fp32's exponent range, so the unnormalised values are as accurate as normalised ones as long
// as the row's largest logit stays within ~2^100 of the reference; k_sweep_finish checks that
// and otherwise sends the whole call down the two-pass path.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_sweep(const bf16_t* __restrict__ Wp, const bf16_t* __restrict__ Hp_panel, int V, int64_t n_valid, int n_kt,
        const float* __restrict__ ref2 /* panel-local */, bf16_t* __restrict__ Gp, int g_n_kt,
        bf16_t* __restrict__ GTp, int gt_n_kt, float* __restrict__ spart /* [MT][ld_s], panel-local */,
        int64_t ld_s, Gate gate) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;
  if (gate_closed(gate)) return;

  const int MT = (V + C::BM - 1) / C::BM;
  const int NTl = (int)((n_valid + C::BN - 1) / C::BN);
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<4>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int64_t n0 = (int64_t)nt * C::BN;
  const int64_t strip_a = (int64_t)n_kt * (C::STAGE_A / 2), strip_b = (int64_t)n_kt * (C::STAGE_B / 2);

  Mainloop<C> ml;
  ml.setup();
  ml.set_a(Wp + mt * strip_a, n_kt);
  ml.set_b(Hp_panel + nt * strip_b, n_kt);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5;
  const int row0 = m0 + wm * C::TM * 32 + 4 * h;   // first vocabulary row of this lane

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.start(smem);
  // the epilogue's per-token references are requested two k-blocks before the end, so that their
  // latency hides behind the last multiplications instead of stalling the epilogue
  const int k_early = n_kt > 2 ? (n_kt - 2) & ~1 : 0;
  ml.steps(smem, 0, k_early, n_kt, acc);
  float r2v[C::TN];
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int64_t n = n0 + wn * C::TN * 32 + j * 32 + (lane & 31);
    // token columns past the panel: reference +inf, every entry 2^(-inf) = 0
    r2v[j] = n < n_valid ? ref2[n] : __builtin_inff();
  }
  ml.steps(smem, k_early, n_kt, n_kt, acc);
  __syncthreads();

  if (m0 + C::BM > V) {  // ragged last vocabulary tile: rows >= V do not exist (2^(-inf) = 0 below)
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (row0 + acc_row(i, r) >= V) {
#pragma unroll
          for (int j = 0; j < C::TN; ++j) acc[i][j][r] = -__builtin_inff();
        }
  }
  float csum[C::TN];
  uint32_t pk[C::TM][C::TN][8];   // the tile as bf16 pairs: rows acc_row(i, 2p), +1
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const float r2 = r2v[j];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][2 * p], kLog2e, -r2));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][2 * p + 1], kLog2e, -r2));
        sum += e0;
        sum += e1;
        const bf16x2 v = {(bf16_t)e0, (bf16_t)e1};
        pk[i][j][p] = __builtin_bit_cast(uint32_t, v);
      }
    csum[j] = sum + __shfl_xor(sum, 32, 64);     // the two lane halves hold the same token
  }
  // row sums: the WM waves stacked along the vocabulary, through LDS, in a fixed order
  __attribute__((address_space(3))) float* red = (__attribute__((address_space(3))) float*)smem;
  if (h == 0) {
#pragma unroll
    for (int j = 0; j < C::TN; ++j) red[wm * C::BN + wn * C::TN * 32 + j * 32 + lane] = csum[j];
  }
  lds_barrier();
  for (int n_l = threadIdx.x; n_l < C::BN; n_l += C::NT) {
    if (n0 + n_l < n_valid) {
      float a = red[n_l];
#pragma unroll
      for (int w = 1; w < C::WM; ++w) a += red[w * C::BN + n_l];
      spart[(int64_t)mt * ld_s + n0 + n_l] = a;
    }
  }
  lds_barrier();
  // GTp: rows = vocabulary (m), k = tokens (n), through LDS, one MFMA block row of every wave at a time
  static_assert(C::WM * 32 * C::PITCH_MN <= C::LDS_BYTES, "staging chunk must fit");
#pragma unroll
  for (int i = 0; i < C::TM; ++i) {
    if (i > 0) lds_barrier();
    stage_mn_pk<C>(smem, pk, i);
    lds_barrier();
    store_mn_pk_packed<C>(smem, GTp, gt_n_kt, m0, (int)(n0 / kPackK), i);
  }
  // Gp: rows = tokens (n), k = vocabulary (m), straight from the registers (last: it consumes pk,
  // and its stores drain after the workgroup has gone)
  store_nm_packed_direct<C>(pk, Gp + (int64_t)nt * g_n_kt * (C::STAGE_B / 2), m0 / kPackK);
#endif
}

// ---------------------------------------------------------------------------
// Backward, step 2: dH[t][j] = f_t * sum_v G[t][v] * W[v][j]
//   A = packed W^T (rows = hidden index j, k = vocabulary), B = Gp (rows = tokens), K = V.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dh(const bf16_t* __restrict__ WTp, int wt_n_kt, const bf16_t* __restrict__ Gp, int g_n_kt, int d,
         int64_t n_valid, int nk /* k-blocks to contract: ceil(V / 64) */,
         const float* __restrict__ row_factor /* f_t, panel-local */, bf16_t* __restrict__ dH /* panel's first row */,
         Gate gate) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;
  if (gate_closed(gate)) return;

  const int MT = (d + C::BM - 1) / C::BM;
  const int NTl = (int)((n_valid + C::BN - 1) / C::BN);
  const int total = MT * NTl;
  const int L = xcd_logical_id(blockIdx.x, total);
  if (L >= total) return;
  int mt, nt;
  strip_tile<4>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int64_t n0 = (int64_t)nt * C::BN;

  Mainloop<C> ml;
  ml.setup();
  ml.set_a(WTp + (int64_t)mt * wt_n_kt * (C::STAGE_A / 2), wt_n_kt);
  ml.set_b(Gp + (int64_t)nt * g_n_kt * (C::STAGE_B / 2), g_n_kt);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.start(smem);
  ml.finish(smem, nk, acc);

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
#pragma unroll 1
  for (int c = 0; c < C::NM_CHUNKS; ++c) {
    stage_nm<C>(smem, acc, c);
    __syncthreads();
    store_nm<C>(smem, dH + n0 * d + m0, d, n_valid - n0, (int64_t)d - m0, c);
    __syncthreads();
  }
#endif
}

// fp32 tile -> dW[n][m] (row pitch d), overwritten or added to, straight from the accumulators.
// A lane owns 4 pieces of 4 consecutive m (16 bytes) of its row n per MFMA block; the four lanes of a
// quad (four neighbouring rows) trade pieces so that lane q holds piece q of each of the four rows:
// every load and store then covers whole 128-byte lines (8 lanes per line).  The four old values of
// an MFMA block are requested together, from clamped (always valid) addresses, before the transpose,
// so the read-add-write waits for memory once per block, not once per piece (eight at once spill).
template <class C, bool ACCUMULATE>
__device__ __forceinline__ void store_dw_tile(const f32x16 (&acc)[C::TM][C::TN], float* __restrict__ dW, int d, int V,
                                              int m0, int n0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int h = lane >> 5, q = lane & 3;
#pragma unroll
  for (int j = 0; j < C::TN; ++j) {
    const int n_q = n0 + wn * C::TN * 32 + j * 32 + (lane & 28);
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      f32x4 piece[4], old[4];
      const int m = m0 + wm * C::TM * 32 + i * 32 + 8 * q + 4 * h;
      if (ACCUMULATE) {
        const int mc = m < d ? m : d - 4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int nc = n_q + r < V ? n_q + r : V - 1;
          old[r] = *(const f32x4*)(dW + (int64_t)nc * d + mc);
        }
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
        piece[c] = f32x4{acc[i][j][4 * c + 0], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2], acc[i][j][4 * c + 3]};
      quad_transpose(piece);
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (m < d && n_q + r < V)
          *(f32x4*)(dW + (int64_t)(n_q + r) * d + m) = ACCUMULATE ? piece[r] + old[r] : piece[r];
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, step 3: dW[v][j] (+)= sum_t G[t][v] * (f_t H[t][j])
//   A = packed (diag(f) H)^T (rows = hidden index j, k = panel tokens), B = GTp (rows = vocabulary).
// fp32 output written straight from the accumulators: 4 consecutive j per lane.
// ---------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT)
k_bwd_dw(const bf16_t* __restrict__ HTp, const bf16_t* __restrict__ GTp, int t_n_kt /* strip pitch of both */, int d,
         int V, int nk /* k-blocks to contract: panel tokens / 64, rounded up to the tile */,
         float* __restrict__ dW, int accumulate, Gate gate) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char_ptr smem = (lds_char_ptr)smem_raw;
  if (gate_closed(gate)) return;

  const int MT = (d + C::BM - 1) / C::BM;
  const int NTl = (V + C::BN - 1) / C::BN;
  const int total = MT * NTl;
  const int L = xcd_round_major_id(blockIdx.x);   // launched in whole rounds of 256 workgroups
  if (L >= total) return;
  int mt, nt;
  strip_tile<4>(L, MT, NTl, mt, nt);
  const int m0 = mt * C::BM;
  const int n0 = nt * C::BN;

  Mainloop<C> ml;
  ml.setup();
  ml.set_a(HTp + (int64_t)mt * t_n_kt * (C::STAGE_A / 2), t_n_kt);
  ml.set_b(GTp + (int64_t)nt * t_n_kt * (C::STAGE_B / 2), t_n_kt);

  f32x16 acc[C::TM][C::TN];
  zero_acc<C>(acc);
  ml.start(smem);
  ml.finish(smem, nk, acc);

  if (accumulate) store_dw_tile<C, true>(acc, dW, d, V, m0, n0);
  else store_dw_tile<C, false>(acc, dW, d, V, m0, n0);
#endif
}

// ---------------------------------------------------------------------------
// Packing of row-major matrices into the block layout the main loop reads.
// ---------------------------------------------------------------------------

// dst = packed(src), src [R, K] row-major with leading dimension ld (K and ld multiples of 8),
// in blocks of `rb` rows (256 for an m-side operand, 384 for an n-side operand).  One workgroup
// per block; blocks in [0, n_rt) x [0, n_kt); everything outside [0, R) x [0, K) is written as zero.
__global__ void __launch_bounds__(256)
k_pack_rows(const bf16_t* __restrict__ src, int64_t R, int K, int64_t ld, bf16_t* __restrict__ dst, int n_kt, int rb) {
  const int kt = blockIdx.x;
  const int64_t rt = blockIdx.y;
  char* out = (char*)dst + (rt * n_kt + kt) * (int64_t)rb * kPackRowBytes;
  for (int idx = threadIdx.x; idx < rb * 8; idx += 256) {   // chunks of 16 B
    const int row = idx >> 3, c = idx & 7;
    const int64_t r = rt * rb + row;
    const int k = kt * kPackK + c * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < R && k < K) v = *(const u32x4*)(src + r * ld + k);
    *(u32x4*)(out + row * 128 + c * 16) = v;
  }
}

// dst = packed(S^T), an m-side operand (256-row blocks), where S [R, Ccols] is row-major (ld; Ccols and ld
// multiples of 8, rows 16-byte aligned) and optionally row-scaled:
// dst row j (a column of S), k index r (a row of S): dst(j, r) = bf16(S[r][j] * scale[r]).
// One workgroup per destination block (jt, kt): it reads S[kt*64 .. +64][jt*256 .. +256] in 16-byte
// pieces (8 columns of one row), four consecutive rows per thread, turns each 4 x 8 patch into eight
// 8-byte column pieces (4 rows of one column) and parks them in LDS as [row quad][column]; a
// destination chunk (8 consecutive r of one j, 16 bytes) is then two 8-byte LDS reads.
// Blocks in [0, n_jt) x [0, n_kt); zero outside [0, Ccols) x [0, R).
__global__ void __launch_bounds__(256)
k_pack_transposed(const bf16_t* __restrict__ src, int64_t R, int Ccols, int64_t ld, const float* __restrict__ scale,
                  bf16_t* __restrict__ dst, int n_kt, Gate gate) {
  // bytes per row quad: 256 columns x 8 bytes; +16 keeps the reads below off each other's banks
  constexpr int kPitch = kPackRowsA * 8 + 16;
  __shared__ __attribute__((aligned(16))) char tile[(kPackK / 4) * kPitch];
  if (gate_closed(gate)) return;
  const int kt = blockIdx.x, jt = blockIdx.y;
  const int64_t r0 = (int64_t)kt * kPackK;
  const int j0 = jt * kPackRowsA;
  const int cc = threadIdx.x & 31;                // 8-column piece of the 256 columns
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int rq = (threadIdx.x >> 5) + 8 * pass;   // row quad 0 .. 15
    const int j = j0 + cc * 8;
    u32x4 row[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t r = r0 + 4 * rq + k;
      row[k] = u32x4{0u, 0u, 0u, 0u};
      if (r < R && j < Ccols) {
        row[k] = *(const u32x4*)(src + r * ld + j);
        if (scale != nullptr) {
          const float sc = scale[r];
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            // a copy: a vector element is not an object whose bytes can be reinterpreted in place
            const uint32_t x = row[k][m];
            const bf16x2 v = __builtin_bit_cast(bf16x2, x);
            const bf16x2 w = {(bf16_t)((float)v[0] * sc), (bf16_t)((float)v[1] * sc)};
            row[k][m] = __builtin_bit_cast(uint32_t, w);
          }
        }
      }
    }
    // dword m of a row holds columns 2m (low half) and 2m + 1 (high half)
    char* out = tile + rq * kPitch + cc * 64;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t a0 = row[0][m], a1 = row[1][m], a2 = row[2][m], a3 = row[3][m];
      const u32x4 piece = {(a0 & 0xFFFFu) | (a1 << 16), (a2 & 0xFFFFu) | (a3 << 16),        // column 2m: rows 0..3
                           (a0 >> 16) | (a1 & 0xFFFF0000u), (a2 >> 16) | (a3 & 0xFFFF0000u)};  // column 2m + 1
      *(u32x4*)(out + m * 16) = piece;
    }
  }
  __syncthreads();
  char* outb = (char*)dst + ((int64_t)jt * n_kt + kt) * (int64_t)kPackBlockBytesA;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int idx = it * 256 + threadIdx.x;
    const int rowj = idx >> 3, c = idx & 7;                 // destination row (j), 8 consecutive k = row quads 2c, 2c + 1
    const u32x2 lo = *(const u32x2*)(tile + (2 * c) * kPitch + rowj * 8);
    const u32x2 hi = *(const u32x2*)(tile + (2 * c + 1) * kPitch + rowj * 8);
    *(u32x4*)(outb + rowj * 128 + c * 16) = u32x4{lo[0], lo[1], hi[0], hi[1]};
  }
}

}  // namespace oapl
