// Shared device-side definitions for the OAPL loss-head kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oapl {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLn2 = 0.6931471805599453094;
// "minus infinity" that survives (m - m) without producing NaN.
constexpr float kNegHuge = -3.0e38f;

// Packed bf16 operand layout of the MFMA kernels: a matrix is cut into blocks of R rows x 64 k
// (R * 128 bytes, row-major inside the block), R = 256 for operands that feed the tile's m side
// ("A": W, W^T, (f o H)^T) and R = 384 for operands that feed its n side ("B": H, G, G^T).
constexpr int kPackK = 64;                              // k-extent of a packed block
constexpr int kPackRowBytes = kPackK * 2;               // 128
constexpr int kPackRowsA = 256;                         // = tile extent along m
constexpr int kPackRowsB = 384;                         // = tile extent along n
constexpr int kPackBlockBytesA = kPackRowsA * kPackRowBytes;   // 32 KiB
constexpr int kPackBlockBytesB = kPackRowsB * kPackRowBytes;   // 48 KiB

// Status words recorded by kernels; the values are those of oapl_status.
constexpr int kErrOffsets = 4;
constexpr int kErrGroup = 5;
constexpr int kErrTokenRange = 9;

// First device-side error wins; later ones are dropped.
__device__ __forceinline__ void record_error(int* flag, int code) {
  atomicCAS(flag, 0, code);
}
// Errors in the batch structure (offsets, group ids) make the loss NaN whatever was recorded
// first, so they are also kept in the status word behind the first.
__device__ __forceinline__ void record_batch_error(int* flag, int code) {
  atomicCAS(flag + 1, 0, code);
  atomicCAS(flag, 0, code);
}
__device__ __forceinline__ bool batch_error(const int* flag) {
  return __hip_atomic_load(flag + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
}

// A kernel launched with a gate runs only if the flag word's truth value equals
// `want` (flag == nullptr: always runs).  The loss entry points use it to choose,
// on the device and in stream order, between the single-sweep path and the
// two-pass path without a host round trip.
struct Gate {
  const int* flag;
  int want;
};
__device__ __forceinline__ bool gate_closed(const Gate g) {
  return g.flag != nullptr && ((*g.flag != 0) != (g.want != 0));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// Workgroup ids are handed to the 8 XCDs round-robin, and each XCD has its own
// L2.  This turns the hardware id into a logical id such that every XCD works
// through one contiguous range of logical ids, so neighbouring tiles (which
// share operand panels) meet in the same L2.  `total` need not be a multiple
// of 8: launch round_up(total, 8) workgroups and drop ids >= total.
__device__ __forceinline__ int xcd_logical_id(int bid, int total) {
  const int per = (total + 7) >> 3;
  return (bid & 7) * per + (bid >> 3);
}

// The other way to keep neighbours in one L2: the 256 workgroups that run together (one per CU)
// take 256 consecutive logical ids, 32 per XCD, round after round, so that at any moment ALL XCDs
// work on neighbouring tiles and read the shared operand panels at about the same time (what one
// XCD fetched from HBM the others find in the memory-side cache).  Launch round_up(total, 256)
// workgroups and drop ids >= total.  Measured: +3.5 % on the dW contraction (whose m-side operand,
// the panel's transposed hidden states, is shared by every tile), nothing on dH, -1..-4 % on the sweep.
__device__ __forceinline__ int xcd_round_major_id(int bid) {
  const int j = bid >> 3;
  return (j >> 5) * 256 + (bid & 7) * 32 + (j & 31);
}

}  // namespace oapl
