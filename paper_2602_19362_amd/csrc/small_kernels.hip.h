// The O(T) and O(N) steps of the OAPL loss head: sampled-token logit gather,
// log-sum-exp finish, per-rollout segmented sums, group value estimate and
// loss (Sec. 3.1, Eq. 2 and Eq. 3) and token coefficients.  All bandwidth-trivial next to the
// three V x d contractions; written for exactness and a fixed summation order.
#pragma once

#include "common.hip.h"
#include "rng.hip.h"

namespace oapl {

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }

__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void k_fill_f32(float* p, int64_t n, float v, Gate gate = Gate{nullptr, 0}) {
  if (gate_closed(gate)) return;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void k_fill_f64(double* p, int64_t n, double v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// z_{t, y_t} = sum_k H[t][k] * W[y_t][k]: one wavefront per token, the gathered
// W row is read with the index exactly as given (checked against [0, V)).
// ACC is double for fp32 inputs and float for bf16 inputs (whose products are
// exact in fp32).
template <class T, class ACC>
__global__ void __launch_bounds__(256)
k_gather_logit(const T* __restrict__ H, const T* __restrict__ W, const int32_t* __restrict__ tokens,
               int64_t Ttok, int d, int V, float* __restrict__ zy, int* __restrict__ err) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Ttok) return;
  const int y = tokens[t];
  if (y < 0 || y >= V) {
    if (lane == 0) {
      record_error(err, kErrTokenRange);
      zy[t] = __builtin_nanf("");
    }
    return;
  }
  const T* h = H + t * d;
  const T* w = W + (int64_t)y * d;
  ACC acc = 0;
  for (int k = lane; k < d; k += 64) acc += (ACC)to_f32(h[k]) * (ACC)to_f32(w[k]);
  acc = wave_sum(acc);
  if (lane == 0) zy[t] = (float)acc;
}

// Merges the per-split soft-max partials of each token and finishes
//   lse_t = ln sum_v exp(z_tv),   logprob_t = min(z_{t,y_t} - lse_t, 0),
// and, when asked for, the entropy of the token's distribution from the extra
// partial u = sum b^(zeta - m) * z.
// A partial is (m, s) with s = sum b^(zeta - m): LOG2 = true means zeta =
// z * log2(e), b = 2 (the MFMA kernel's epilogue); false means zeta = z, b = e.
// Everything after the fp32 partials is done in double.
template <bool LOG2>
__global__ void __launch_bounds__(256)
k_lse_finish(const float2* __restrict__ partials, int n_parts, int64_t Ttok, const float* __restrict__ zy,
             const float* __restrict__ logq, float* __restrict__ logprob_out, float* __restrict__ lse_out,
             float* __restrict__ lse2_ws, double* __restrict__ diff_ws, float* __restrict__ omp_ws,
             float* __restrict__ inv_omp_ws, const float* __restrict__ upart, float* __restrict__ entropy_out,
             Gate gate) {
  if (gate_closed(gate)) return;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= Ttok) return;
  float M = kNegHuge;
  for (int p = 0; p < n_parts; ++p) M = fmaxf(M, partials[(int64_t)p * Ttok + t].x);
  double S = 0.0, U = 0.0;
  for (int p = 0; p < n_parts; ++p) {
    const float2 a = partials[(int64_t)p * Ttok + t];
    const double e = (double)a.x - (double)M;
    const double f = LOG2 ? exp2(e) : exp(e);
    S += (double)a.y * f;
    if (entropy_out) U += (double)upart[(int64_t)p * Ttok + t] * f;
  }
  const double lse = LOG2 ? ((double)M + log2(S)) * kLn2 : (double)M + log(S);
  double lp = (double)zy[t] - lse;   // NaN if the token was out of range
  if (lp > 0.0) lp = 0.0;            // the gathered logit is rounded separately from the sum
  if (logprob_out) logprob_out[t] = (float)lp;
  if (lse_out) lse_out[t] = (float)lse;
  // policy entropy  -sum_v p_v ln p_v = lse - sum_v p_v z_v  with  sum_v p_v z_v = U / S  (>= 0 up to rounding)
  if (entropy_out) entropy_out[t] = (float)fmax(lse - U / S, 0.0);
  // the backward kernels want lse in the domain their exponentials work in
  if (lse2_ws) lse2_ws[t] = (float)(LOG2 ? lse * (double)1.4426950408889634074 : lse);
  if (diff_ws) diff_ws[t] = lp - (double)logq[t];
  // 1 - p_{t,y_t}, accurate also when the sampled token has almost all the mass;
  // its reciprocal normalises the bf16 gradient rows (0 switches a row off when
  // the soft-max is one-hot at y_t to working precision, or the token is bad)
  if (omp_ws) {
    const double omp = -expm1(lp);
    const bool ok = omp > 1e-30;
    omp_ws[t] = ok ? (float)omp : 0.f;
    inv_omp_ws[t] = ok ? (float)(1.0 / omp) : 0.f;
  }
}

// Picks, per token, the best (score, index) pair over the vocabulary splits (ties to the smaller index).
__global__ void __launch_bounds__(256)
k_sample_finish(const float2* __restrict__ partials, int n_parts, int64_t Ttok, int32_t* __restrict__ tokens_out,
                float* __restrict__ score_out) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= Ttok) return;
  float best = -__builtin_inff();
  int arg = 0x7FFFFFFF;
  for (int p = 0; p < n_parts; ++p) {
    const float2 a = partials[(int64_t)p * Ttok + t];
    if (better(a.x, __float_as_int(a.y), best, arg)) { best = a.x; arg = __float_as_int(a.y); }
  }
  tokens_out[t] = arg;
  if (score_out) score_out[t] = best;
}

// out[s] = sum_{t in [off[s], off[s+1])} x[t] in double: one workgroup per
// rollout, each thread a strided partial in a fixed order, wavefront shuffle
// reduction, then the 4 wave totals in order.  Bit-reproducible.  Offsets are
// clamped to [0, limit] (limit < 0: only to a >= 0, b >= a) so malformed input
// cannot read below the buffer or, with a limit, past it.
template <class T>
__global__ void __launch_bounds__(256)
k_segmented_sum(const T* __restrict__ x, const int64_t* __restrict__ off, int n_seq, int64_t limit,
                double* __restrict__ out, Gate gate = Gate{nullptr, 0}) {
  __shared__ double wsum[4];
  if (gate_closed(gate)) return;
  const int s = blockIdx.x;
  if (s >= n_seq) return;
  int64_t a = off[s], b = off[s + 1];
  a = a < 0 ? 0 : a;
  b = b < a ? a : b;
  if (limit >= 0) {
    a = a > limit ? limit : a;
    b = b > limit ? limit : b;
  }
  double acc = 0.0;
  for (int64_t t = a + threadIdx.x; t < b; t += 256) acc += (double)x[t];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) out[s] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
}

// Butterfly reductions over a wavefront: every lane ends with the same value, combined in a
// fixed order (bit-reproducible).
__device__ __forceinline__ double wave_allsum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_allmax(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_allsum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Group value estimate, one wavefront per prompt (4 prompts per workgroup):
//   V*_g = beta_v ln( (1/G_g) sum_{s in g} exp(r_s / beta_v) )            Eq. 2
//        = m_g + beta_v ln( (1/G_g) sum exp((r_s - m_g) / beta_v) ),  m_g = max_{s in g} r_s
// (same value; the shift keeps exp() in range for small beta and makes all-equal rewards return
// exactly r).  Group ids come in any order, so the wavefront walks the rollouts lane-strided and
// keeps those of its prompt: lane-local partial max / count / sum in rollout order, then shuffle
// butterflies.  A prompt without rollouts gets NaN and records the group error.
__global__ void __launch_bounds__(256)
k_group_value(const float* __restrict__ rewards, const int32_t* __restrict__ gid, int n_seq, int n_groups,
              double beta_v, double* __restrict__ vstar_ws, float* __restrict__ vstar_out, int* __restrict__ err,
              Gate gate) {
  if (gate_closed(gate)) return;
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= n_groups) return;
  double m = -1.0e300;
  int cnt = 0;
  for (int s = lane; s < n_seq; s += 64)
    if (gid[s] == g) { m = fmax(m, (double)rewards[s]); ++cnt; }
  m = wave_allmax(m);
  cnt = wave_allsum(cnt);
  double v;
  if (cnt == 0) {
    if (lane == 0) record_batch_error(err, kErrGroup);
    v = __builtin_nan("");
  } else {
    double sum = 0.0;
    for (int s = lane; s < n_seq; s += 64)
      if (gid[s] == g) sum += exp(((double)rewards[s] - m) / beta_v);
    sum = wave_allsum(sum);
    v = m + beta_v * log(sum / (double)cnt);
  }
  if (lane == 0) {
    vstar_ws[g] = v;
    if (vstar_out) vstar_out[g] = (float)v;
  }
}

// Residuals and loss (one workgroup walks the rollouts; fixed summation order):
//   delta_s = beta_l Delta_s - (r_s - V*_{g(s)})
//   loss    = scale sum_s delta_s^2                                           Eq. 3
//   cseq_s  = scale 2 beta_l delta_s      (d loss / d ln pi(y_t) for every token of s)
// Also validates offsets and group ids; on a violation (or an empty prompt found by
// k_group_value, whose V* is NaN) the loss is NaN and the status word is set.
__global__ void __launch_bounds__(256)
k_residual_loss(const double* __restrict__ Delta, const float* __restrict__ rewards,
                const int32_t* __restrict__ gid, const int64_t* __restrict__ off, int n_seq, int n_groups,
                int64_t Ttok, double beta_l, double scale, const double* __restrict__ vstar_ws,
                float* __restrict__ cseq, float* __restrict__ loss_out, float* __restrict__ seq_logratio_out,
                int* __restrict__ err, Gate gate) {
  __shared__ double wsum[4];
  __shared__ int bad;
  if (gate_closed(gate)) return;
  const int tid = threadIdx.x;
  if (tid == 0) bad = (off[0] != 0 || off[n_seq] != Ttok) ? kErrOffsets : 0;
  __syncthreads();
  double acc = 0.0;
  for (int s = tid; s < n_seq; s += 256) {
    if (off[s + 1] < off[s]) atomicCAS(&bad, 0, kErrOffsets);
    const int g = gid[s];
    const bool g_ok = g >= 0 && g < n_groups;
    if (!g_ok) atomicCAS(&bad, 0, kErrGroup);
    const double v = g_ok ? vstar_ws[g] : __builtin_nan("");
    const double delta = beta_l * Delta[s] - ((double)rewards[s] - v);
    cseq[s] = (float)(scale * 2.0 * beta_l * delta);
    if (seq_logratio_out) seq_logratio_out[s] = (float)Delta[s];
    acc += delta * delta;
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) wsum[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double loss = scale * (((wsum[0] + wsum[1]) + wsum[2]) + wsum[3]);
    if (bad) record_batch_error(err, bad);
    if (batch_error(err)) loss = __builtin_nan("");
    loss_out[0] = (float)loss;
  }
}

// GRPO baseline (Sec. 2, the displayed GRPO objective), group step, one wavefront per prompt:
// mean and population standard deviation of the prompt's rewards and its size G_g (kept behind
// the per-rollout weights).  A prompt without rollouts gets NaN and records the group error.
__global__ void __launch_bounds__(256)
k_grpo_group_stats(const float* __restrict__ rewards, const int32_t* __restrict__ gid, int n_seq, int n_groups,
                   double* __restrict__ gmean, double* __restrict__ gstd, double* __restrict__ gsize,
                   int* __restrict__ err, Gate gate) {
  if (gate_closed(gate)) return;
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= n_groups) return;
  double sum = 0.0;
  int cnt = 0;
  for (int s = lane; s < n_seq; s += 64)
    if (gid[s] == g) { sum += (double)rewards[s]; ++cnt; }
  sum = wave_allsum(sum);
  cnt = wave_allsum(cnt);
  if (cnt == 0) {
    if (lane == 0) {
      record_batch_error(err, kErrGroup);
      gmean[g] = __builtin_nan("");
      gstd[g] = __builtin_nan("");
      gsize[g] = 0.0;
    }
    return;
  }
  const double mean = sum / cnt;
  double var = 0.0;
  for (int s = lane; s < n_seq; s += 64)
    if (gid[s] == g) { const double dlt = (double)rewards[s] - mean; var += dlt * dlt; }
  var = wave_allsum(var);
  if (lane == 0) {
    gmean[g] = mean;
    gstd[g] = sqrt(var / cnt);
    gsize[g] = (double)cnt;
  }
}

// GRPO, rollout step: the normalised advantage
//   A_s = (r_s - mean_g r) / (std_g r + adv_eps)
// and the weight w_s = scale / (G_g |y_s|) of rollout s (0 for an empty rollout).  Validates
// offsets and group ids like the OAPL kernel and records the status.
__global__ void __launch_bounds__(256)
k_grpo_advantage(const float* __restrict__ rewards, const int32_t* __restrict__ gid, const int64_t* __restrict__ off,
                 int n_seq, int n_groups, int64_t Ttok, double adv_eps, double scale,
                 const double* __restrict__ gmean, const double* __restrict__ gstd, const double* __restrict__ gsize,
                 float* __restrict__ adv, double* __restrict__ wseq, float* __restrict__ adv_out,
                 int* __restrict__ err, Gate gate) {
  if (gate_closed(gate)) return;
  if (blockIdx.x == 0 && threadIdx.x == 0 && (off[0] != 0 || off[n_seq] != Ttok)) record_batch_error(err, kErrOffsets);
  for (int s = blockIdx.x * 256 + threadIdx.x; s < n_seq; s += gridDim.x * 256) {
    if (off[s + 1] < off[s]) record_batch_error(err, kErrOffsets);
    const int g = gid[s];
    const bool ok = g >= 0 && g < n_groups;
    if (!ok) record_batch_error(err, kErrGroup);
    const double a = ok ? ((double)rewards[s] - gmean[g]) / (gstd[g] + adv_eps) : __builtin_nan("");
    const int64_t len = off[s + 1] - off[s];
    adv[s] = (float)a;
    if (adv_out) adv_out[s] = (float)a;
    wseq[s] = (ok && len > 0 && gsize[g] > 0.0) ? scale / (gsize[g] * (double)len) : 0.0;
  }
}

// GRPO, token step: one workgroup per rollout.  With r_t = pi / pi_old and IS_t = pi_old / pi_vllm,
//   term_t = IS_t min(r_t A, clip(r_t, 1 - eps, 1 + eps) A),   d term_t / d ln pi(y_t) = IS_t r_t A if unclipped else 0,
// it writes the loss gradient coefficient c_t = -w_s d term_t (times factor[t] if given) and the
// rollout's loss share -w_s sum_t term_t (double, fixed order).  lp comes as diff = lp - logq in double.
__global__ void __launch_bounds__(256)
k_grpo_tokens(const double* __restrict__ diff, const float* __restrict__ logq, const float* __restrict__ logp_old,
              const int64_t* __restrict__ off, int n_seq, int64_t Ttok, const float* __restrict__ adv,
              const double* __restrict__ wseq, double clip_eps, const float* __restrict__ factor,
              float* __restrict__ coef, double* __restrict__ seqterm, Gate gate) {
  __shared__ double wsum[4];
  if (gate_closed(gate)) return;
  const int s = blockIdx.x;
  if (s >= n_seq) return;
  int64_t a = off[s], b = off[s + 1];
  a = a < 0 ? 0 : (a > Ttok ? Ttok : a);
  b = b < a ? a : (b > Ttok ? Ttok : b);
  const double A = (double)adv[s], w = wseq[s];
  double acc = 0.0;
  for (int64_t t = a + threadIdx.x; t < b; t += 256) {
    const double q = (double)logq[t], lo = (double)logp_old[t];
    const double lp = diff[t] + q;
    const double r = exp(lp - lo), is = exp(lo - q);
    const double unclipped = r * A;
    const double rc = r < 1.0 - clip_eps ? 1.0 - clip_eps : (r > 1.0 + clip_eps ? 1.0 + clip_eps : r);
    const double clipped = rc * A;
    acc += is * (unclipped <= clipped ? unclipped : clipped);
    const double g = unclipped <= clipped ? -w * is * unclipped : 0.0;
    coef[t] = (float)(factor ? g * (double)factor[t] : g);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) seqterm[s] = -w * (((wsum[0] + wsum[1]) + wsum[2]) + wsum[3]);
}

// loss = sum_s seqterm[s] (one workgroup, fixed order), NaN if an offsets / group error was recorded.
__global__ void __launch_bounds__(256)
k_grpo_loss(const double* __restrict__ seqterm, int n_seq, const int* __restrict__ err,
            float* __restrict__ loss_out, Gate gate) {
  __shared__ double wsum[4];
  if (gate_closed(gate)) return;
  double acc = 0.0;
  for (int s = threadIdx.x; s < n_seq; s += 256) acc += seqterm[s];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double loss = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
    if (batch_error(err)) loss = __builtin_nan("");
    loss_out[0] = (float)loss;
  }
}

// coef[t] = cseq[s(t)] (times factor[t] if given): one workgroup per rollout
// writes its token range (clamped to [0, T], so malformed offsets cannot write
// out of bounds).
__global__ void __launch_bounds__(256)
k_token_coefficients(const float* __restrict__ cseq, const int64_t* __restrict__ off, int n_seq, int64_t Ttok,
                     const float* __restrict__ factor, float* __restrict__ coef, Gate gate) {
  if (gate_closed(gate)) return;
  const int s = blockIdx.x;
  if (s >= n_seq) return;
  int64_t a = off[s], b = off[s + 1];
  a = a < 0 ? 0 : (a > Ttok ? Ttok : a);
  b = b < a ? a : (b > Ttok ? Ttok : b);
  const float c = cseq[s];
  for (int64_t t = a + threadIdx.x; t < b; t += 256) coef[t] = factor ? c * factor[t] : c;
}

// ---------------------------------------------------------------------------
// Helpers of the single-sweep loss path (see k_sweep).
// ---------------------------------------------------------------------------

// The single-sweep path finishes a panel of token rows before it knows the later panels, so a
// rollout must end at most one panel after it starts: any rollout longer than `panel_rows`
// (or malformed offsets) raises the flag that sends the call down the two-pass path instead.
__global__ void __launch_bounds__(256)
k_sweep_plan(const int64_t* __restrict__ off, int n_seq, int64_t Ttok, int64_t panel_rows, int* __restrict__ flag) {
  bool bad = threadIdx.x == 0 && blockIdx.x == 0 && (off[0] != 0 || off[n_seq] != Ttok);
  for (int s = blockIdx.x * 256 + threadIdx.x; s < n_seq; s += gridDim.x * 256) {
    const int64_t len = off[s + 1] - off[s];
    bad |= len < 0 || len > panel_rows;
  }
  if (bad) atomicCAS(flag, 0, 1);
}

// Reference exponent of a token row for k_sweep: the largest logit among a sample of the row
// (the first vocabulary tile, whose running maximum `sample` carries in .x, and the sampled
// token's own logit) plus a margin, in the exp2 domain.  Some entry of the row then equals
// 2^-margin, so S_t >= 2^-margin, and entries down to 2^-(126 - margin) of the row's largest
// stay normal bf16 numbers.
constexpr float kSweepMargin = 40.f;
constexpr float kSweepLimit = 1.2676506e30f;   // 2^100: largest S_t the single sweep accepts
__global__ void __launch_bounds__(256)
k_sweep_ref(const float2* __restrict__ sample, const float* __restrict__ zy, int64_t Ttok, float* __restrict__ ref2) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= Ttok) return;
  ref2[t] = fmaxf(sample[t].x, zy[t] * kLog2e) + kSweepMargin;    // fmaxf drops a NaN zy (token out of range)
}

// Finishes one panel of the single sweep.  Per token row (panel-local index n, global t0 + n):
//   S = sum of the vocabulary-tile partial sums (double, fixed order),  lse = (ref2 + log2 S) ln 2,
//   logprob = min(z_y - lse, 0),  diff = logprob - logq,  nis = -1 / S  (row factor of the gradient, times the
//   correction below),
// and patches the sampled token's entry of the unnormalised soft-max panel, in both packed
// copies, to  Pt[y] - S = -S (1 - p_y)  (computed from expm1 so it is accurate when p_y -> 1).
// Rows whose sum left the accepted range raise the fallback flag.
constexpr int kFinishSlices = 8;
constexpr int kFinishRows = 32;      // token rows per workgroup of kFinishSlices * kFinishRows threads
__global__ void __launch_bounds__(kFinishSlices * kFinishRows)
k_sweep_finish(const float* __restrict__ spart, int n_vt, int64_t ld_s, int64_t n_valid,
               const float* __restrict__ ref2, const float* __restrict__ zy, const float* __restrict__ logq,
               const int32_t* __restrict__ tokens, int V, float* __restrict__ logprob_out,
               double* __restrict__ diff, float* __restrict__ nis, bf16_t* __restrict__ Gp, int g_n_kt,
               bf16_t* __restrict__ GTp, int gt_n_kt, int* __restrict__ flag, Gate gate) {
  if (gate_closed(gate)) return;
  // kFinishRows token rows per workgroup; the tile sums of a row are added in kFinishSlices interleaved slices
  // (slice s takes tiles s, s + kFinishSlices, ...), then the slices in order: a fixed order, and
  // enough workgroups to fill the chip with a panel's 12288 rows.
  __shared__ double part[kFinishSlices][kFinishRows];
  const int col = threadIdx.x % kFinishRows, slice = threadIdx.x / kFinishRows;
  const int64_t n = (int64_t)blockIdx.x * kFinishRows + col;
  double acc = 0.0;
  if (n < n_valid)
    for (int mt = slice; mt < n_vt; mt += kFinishSlices) acc += (double)spart[(int64_t)mt * ld_s + n];
  part[slice][col] = acc;
  __syncthreads();
  if (slice != 0 || n >= n_valid) return;
  double S = part[0][col];
#pragma unroll
  for (int s = 1; s < kFinishSlices; ++s) S += part[s][col];
  if (!(S <= (double)kSweepLimit)) atomicCAS(flag, 0, 1);     // also catches inf and NaN
  const double lse = ((double)ref2[n] + log2(S)) * kLn2;
  double lp = (double)zy[n] - lse;     // NaN if the token was out of range
  if (lp > 0.0) lp = 0.0;
  if (logprob_out) logprob_out[n] = (float)lp;
  diff[n] = lp - (double)logq[n];
  double row_factor = -1.0 / S;
  const int y = tokens[n];
  if (y >= 0 && y < V) {
    const double entry = S * expm1(lp);                        // -S (1 - p_y)
    const bf16_t patch = (bf16_t)(float)entry;
    // The sampled token's entry carries nearly all of the row's gradient, and bf16 keeps 8 bits of it.
    // The row factor absorbs that rounding: factor * patch is then the exact entry, and the relative
    // error (<= 2^-8) moves to the row's other entries, whose joint weight in the gradient is small.
    const double kept = (double)(float)patch;
    if (kept != 0.0 && isfinite(entry)) row_factor *= entry / kept;
    // both copies are n-side operands: blocks of kPackRowsB rows x 64 k
    const int64_t blk = (int64_t)kPackRowsB * kPackK;             // elements of a packed block
    const int64_t nb = n / kPackRowsB, nr = n - nb * kPackRowsB;  // token row block / row inside it
    const int yb = y / kPackRowsB, yr = y - yb * kPackRowsB;      // vocabulary row block / row inside it
    Gp[(nb * g_n_kt + (y >> 6)) * blk + nr * kPackK + (y & 63)] = patch;
    GTp[((int64_t)yb * gt_n_kt + (n >> 6)) * blk + (int64_t)yr * kPackK + (n & 63)] = patch;
  }
  nis[n] = (float)row_factor;
}

}  // namespace oapl
