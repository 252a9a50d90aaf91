// C ABI of the OAPL loss head: argument checks, workspace plan, launch order.
// Every step of the path runs in the kernels of this directory; nothing here
// computes on the host and nothing falls back to a CPU path.
#include "oapl.h"

#include <math.h>
#include <mutex>
#include <utility>
#include <vector>

#include "gemm_bf16.hip.h"
#include "gemm_f32.hip.h"
#include "small_kernels.hip.h"

namespace oapl {

// 256 x 384 x 64 tiles, 8 wavefronts in a 4 x 2 grid, each a 64 x 192 patch
// (2 x 6 MFMA blocks, 192 accumulator registers per lane), two wavefronts per
// SIMD; operands in a ring of 2 LDS stages (160 KB, the whole LDS of a CU).
typedef TileCfg<4, 2, 2, 6, 2> Cfg;
static_assert(Cfg::BN == kPackRowsB, "n-side operands of the loss path are packed in blocks of one tile");
// The sampling kernel carries a running (score, index) pair per column through the main loop and
// draws Philox blocks in its epilogue: it keeps the 256 x 256 tile (128 accumulators per lane),
// with H packed in 256-row blocks for it.
typedef TileCfg<4, 2, 2, 4, 2> CfgSample;

// Most token rows per backward panel (bf16 path): 32 token tiles, the fastest size measured (the dH
// contraction then has d / 256 x 32 tiles, whole rounds of 256 workgroups for d a multiple of 2048;
// larger panels run 2 .. 3 % slower, smaller ones pay more for the read-add-write of dW).  A smaller
// workspace makes panels smaller; a larger one buys more panel buffers (longer rollouts on the single
// sweep), never larger panels.
constexpr int64_t kPanelBf16 = 12288;
constexpr int64_t kPanelF32 = 4096;    // ... (fp32 path)
constexpr int64_t kGroupScanLimit = (int64_t)1 << 32;   // n_seq * n_groups: every prompt's wavefront walks all rollouts
constexpr int kStatusWords = 64;       // 256-byte header
constexpr int kNumCU = 256;            // MI355X compute units (one workgroup of the dense kernels each: it fills the LDS)

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Plan {
  int64_t T = 0;
  int d = 0, V = 0, n_seq = 0, n_groups = 0, dtype = 0;
  bool bwd = false;
  int n_parts = 0;     // soft-max partials per token
  int n_parts_s = 0;   // (score, index) partials per token of the sampling kernel
  int64_t Tp = 0;      // rows of one backward panel
  int n_buf = 1;       // panel buffers of the single sweep (a ring; one if the batch is one panel)
  size_t size_G = 0, size_GT = 0;   // bytes of one panel buffer of each packed copy
  // packed-operand geometry (bf16 path): row tiles and k-blocks (strip pitches)
  int n_rt_v = 0, n_rt_d = 0, n_kt_d = 0, n_kt_v = 0, n_kt_g = 0, n_kt_t = 0;
  int n_rb_v = 0;      // 384-row blocks of a matrix whose rows are the vocabulary (G^T)
  int64_t n_rt_T = 0;  // 384-row token tiles of the whole batch
  size_t off_status = 0, off_partials = 0, off_upart = 0, off_zy = 0, off_lse2 = 0, off_diff = 0, off_coef = 0, off_delta = 0,
         off_cseq = 0, off_vstar = 0, off_gw = 0, off_omp = 0, off_inv = 0, off_Wp = 0, off_Hp = 0, off_WTp = 0, off_HTp = 0,
         off_G = 0, off_GT = 0, off_ref2 = 0, off_spart = 0, total = 0;
  bool sweep = false;  // single-sweep loss path available (bf16 with backward)
};

constexpr int kFlagWord = 8;   // status word that selects the two-pass path on the device
// A call this small gains nothing from the sweep's saved pass; it takes the two-pass path, whose one-hot
// gradient entry is exact rather than exact up to the row-factor correction.
constexpr int64_t kSweepMinTokens = 64;

// Largest panel the plan may use: `max_panel_rows` <= 0 or above the library's size means that
// size; other values are rounded down to whole token tiles (bf16), with one tile as the least.
static int64_t panel_cap(int dtype, int64_t max_panel_rows) {
  const int64_t deflt = dtype == OAPL_BF16 ? kPanelBf16 : kPanelF32;
  if (max_panel_rows <= 0 || max_panel_rows > deflt) return deflt;
  if (dtype != OAPL_BF16) return max_panel_rows;
  return max_panel_rows < Cfg::BN ? Cfg::BN : max_panel_rows / Cfg::BN * Cfg::BN;
}

// `panel_buffers`: how many panels the single sweep keeps before their gradient contractions run
// (<= 0: two, the least for a batch of several panels; never more than the batch has panels).
static bool make_plan(Plan& p, int64_t T, int d, int V, int n_seq, int n_groups, int dtype, bool bwd,
                      int64_t max_panel_rows = 0, int64_t panel_buffers = 0, int64_t exact_panel_rows = 0) {
  if (T < 0 || d < 1 || V < 1 || n_seq < 0 || n_groups < 1) return false;
  if (dtype != OAPL_F32 && dtype != OAPL_BF16) return false;
  if (dtype == OAPL_BF16 && (d % 8) != 0) return false;
  // a packed row-tile strip (K / 64 blocks of 32 or 48 KiB) must stay below 2 GiB for 32-bit buffer offsets,
  // and the packing kernels index token tiles with gridDim.y
  if ((int64_t)d > (1 << 21) || (int64_t)V > (1 << 21)) return false;
  if (dtype == OAPL_BF16 && T > (int64_t)65535 * 256) return false;
  // the fp32 kernels index 64-row token tiles with gridDim.y
  if (dtype == OAPL_F32 && T > (int64_t)65535 * 64) return false;
  if ((int64_t)n_seq * n_groups > kGroupScanLimit) return false;
  const int64_t cap = panel_cap(dtype, max_panel_rows);
  p.T = T; p.d = d; p.V = V; p.n_seq = n_seq; p.n_groups = n_groups; p.dtype = dtype; p.bwd = bwd;
  if (dtype == OAPL_BF16) {
    const int64_t n_tiles = (T + Cfg::BN - 1) / Cfg::BN;
    const int MT = (V + Cfg::BM - 1) / Cfg::BM;
    // Vocabulary splits of the streaming kernels: one workgroup per (token tile, split), one
    // workgroup per CU at a time.  Pick the split count that wastes the least of the last round
    // of workgroups and of the uneven division of vocabulary tiles, with at least ~8 tiles each.
    auto pick_splits = [&](int64_t tiles) {
      const int64_t max_splits = MT / 8 > 1 ? (MT / 8 < 64 ? MT / 8 : 64) : 1;
      int64_t splits = 1;
      double best = -1.0;
      for (int64_t c = 1; c <= max_splits && tiles > 0; ++c) {
        const int64_t wgs = tiles * c;
        const double rounds = (double)wgs / kNumCU;
        const double fill = rounds / (double)((wgs + kNumCU - 1) / kNumCU);      // occupancy of the last round
        const double even = ((double)MT / c) / (double)((MT + c - 1) / c);       // equal work per workgroup
        const double score = fill * even;
        if (score > best + 1e-9) { best = score; splits = c; }
      }
      return (int)splits;
    };
    p.n_parts = pick_splits(n_tiles);
    p.n_parts_s = pick_splits((T + CfgSample::BN - 1) / CfgSample::BN);
    // Panel size: a multiple of the token tile, at most `cap` rows.  One panel if T fits; otherwise
    // the size (between half the cap and the cap) that costs the fewest rounds of kNumCU workgroups in
    // the dH contraction -- its tiles (d / 256 x panel rows / 384, each K = V long) are few and long, so
    // a partly filled last round is expensive -- plus a charge per panel for the fp32 read-add-write
    // pass over dW.  Ties go to the larger panel (longer rollouts fit the single sweep).
    if (T <= cap) {
      p.Tp = round_up(T > 0 ? T : 1, Cfg::BN);
    } else if (exact_panel_rows > 0) {   // a size an earlier plan for the same shapes chose
      p.Tp = exact_panel_rows;
    } else {
      const int64_t mtd = (d + Cfg::BM - 1) / Cfg::BM;
      const int64_t k_max = cap / Cfg::BN;
      double best = 1e300;
      for (int64_t k = k_max; k >= (k_max + 1) / 2; --k) {
        const int64_t rows = k * Cfg::BN;
        const int64_t full = T / rows, rest = T - full * rows;
        const int64_t rounds_full = (mtd * k + kNumCU - 1) / kNumCU;
        const int64_t rounds_rest = (mtd * ((rest + Cfg::BN - 1) / Cfg::BN) + kNumCU - 1) / kNumCU;
        const double cost = (double)(full * rounds_full + rounds_rest) + 0.35 * (double)(full + (rest > 0 ? 1 : 0));
        if (cost < best - 1e-9) { best = cost; p.Tp = rows; }
      }
    }
    p.n_rt_v = MT;
    p.n_rb_v = (int)(round_up((int64_t)MT * Cfg::BM, Cfg::BN) / Cfg::BN);
    p.n_rt_d = (d + Cfg::BM - 1) / Cfg::BM;
    p.n_rt_T = n_tiles > 0 ? n_tiles : 1;
    p.n_kt_d = (d + kPackK - 1) / kPackK;
    p.n_kt_v = (V + kPackK - 1) / kPackK;            // W^T strips: exactly the k-blocks the dH contraction walks
    p.n_kt_g = MT * (Cfg::BM / kPackK);              // G strips: whole vocabulary tiles
    p.n_kt_t = (int)(p.Tp / kPackK);                 // strips whose k index is the panel token
  } else {
    p.n_parts = p.n_parts_s = (V + 63) / 64;
    p.Tp = T < cap ? (T > 0 ? T : 1) : cap;
  }
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) / 256 * 256; return at; };
  const size_t Tn = (size_t)(T > 0 ? T : 1);
  p.off_status = take(kStatusWords * 4);
  p.off_partials = take(Tn * (size_t)(p.n_parts > p.n_parts_s ? p.n_parts : p.n_parts_s) * 8);
  p.off_upart = take(Tn * (size_t)p.n_parts * 4);
  p.off_zy = take(Tn * 4);
  p.off_lse2 = take(Tn * 4);
  p.off_diff = take(Tn * 8);
  p.off_coef = take(Tn * 4);
  p.off_omp = take(Tn * 4);
  p.off_inv = take(Tn * 4);
  p.off_delta = take((size_t)(n_seq > 0 ? n_seq : 1) * 8);
  p.off_cseq = take((size_t)(n_seq > 0 ? n_seq : 1) * 4);
  p.off_vstar = take((size_t)n_groups * 16);
  p.off_gw = take((size_t)((n_seq > 0 ? n_seq : 1) + n_groups) * 8);
  if (dtype == OAPL_BF16) {
    p.off_Wp = take((size_t)p.n_rt_v * p.n_kt_d * kPackBlockBytesA);
    {  // packed H: 384-row blocks, or 256-row blocks for the sampling kernel (whichever is larger)
      const size_t a = (size_t)p.n_rt_T * p.n_kt_d * kPackBlockBytesB;
      const size_t b = (size_t)((T + CfgSample::BN - 1) / CfgSample::BN > 0 ? (T + CfgSample::BN - 1) / CfgSample::BN : 1) *
                       p.n_kt_d * CfgSample::STAGE_B;
      p.off_Hp = take(a > b ? a : b);
    }
  }
  if (bwd) {
    if (dtype == OAPL_BF16) {
      p.off_WTp = take((size_t)p.n_rt_d * p.n_kt_v * kPackBlockBytesA);
      p.off_HTp = take((size_t)p.n_rt_d * p.n_kt_t * kPackBlockBytesA);
      // Panel buffers, both packed copies.  The single sweep keeps a ring of them: a panel's gradient
      // contractions run once every rollout that touches it is scored, i.e. n_buf - 1 panels later, so
      // rollouts of up to (n_buf - 1) panels are served (the two-pass schedule uses the first buffer only).
      const int64_t n_panels = (T + p.Tp - 1) / p.Tp;
      p.n_buf = (int)(n_panels <= 1 ? 1 : (panel_buffers < 2 ? 2 : (panel_buffers > n_panels ? n_panels : panel_buffers)));
      p.size_G = ((size_t)(p.Tp / Cfg::BN) * p.n_kt_g * kPackBlockBytesB + 255) / 256 * 256;
      p.size_GT = ((size_t)p.n_rb_v * p.n_kt_t * kPackBlockBytesB + 255) / 256 * 256;
      p.off_G = take(p.size_G * p.n_buf);
      p.off_GT = take(p.size_GT * p.n_buf);
      // single-sweep path: reference exponents and per-vocabulary-tile row sums of one panel
      p.sweep = true;
      p.off_ref2 = take(Tn * 4);
      p.off_spart = take((size_t)p.n_rt_v * (size_t)p.Tp * 4);
    } else {
      p.off_G = take((size_t)p.Tp * V * 4);
    }
  }
  p.total = o;
  return true;
}

static inline unsigned grid1d(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// Optional per-kernel timing of the four dense kernels: when switched on, every
// launch is bracketed by a pair of events recorded on the launch stream itself.
enum DenseKernel { kFwdLse = 0, kBwdDz = 1, kBwdDh = 2, kBwdDw = 3, kFwdSample = 4, kSweep = 5, kNumDense = 6 };
struct TimingState {
  std::mutex mu;
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[kNumDense];
};
static TimingState& timing() {
  static TimingState t;
  return t;
}
struct ScopedKernelTimer {
  hipStream_t st;
  hipEvent_t stop = nullptr;
  ScopedKernelTimer(int which, hipStream_t s, bool enabled = true) : st(s) {
    if (!enabled) return;
    TimingState& t = timing();
    std::lock_guard<std::mutex> g(t.mu);
    if (!t.on) return;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    (void)hipEventRecord(a, st);
    stop = b;
    t.ev[which].emplace_back(a, b);
  }
  ~ScopedKernelTimer() {
    if (stop) (void)hipEventRecord(stop, st);
  }
};

#define OAPL_LAUNCH_CHECK()                                   \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return OAPL_ERR_HIP; \
  } while (0)

template <class K>
static bool allow_big_lds(K kernel, int bytes) {
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
}

static bool prepare_kernels() {
  static std::once_flag once;
  static bool ok = false;
  std::call_once(once, [] {
    ok = allow_big_lds(k_fwd_lse<Cfg, false>, Cfg::LDS_BYTES) && allow_big_lds(k_fwd_lse<Cfg, true>, Cfg::LDS_BYTES) &&
         allow_big_lds(k_fwd_sample<CfgSample>, CfgSample::LDS_BYTES) && allow_big_lds(k_bwd_dz<Cfg>, Cfg::LDS_BYTES) &&
         allow_big_lds(k_bwd_dh<Cfg>, Cfg::LDS_BYTES) && allow_big_lds(k_bwd_dw<Cfg>, Cfg::LDS_BYTES) &&
         allow_big_lds(k_sweep<Cfg>, Cfg::LDS_BYTES);
  });
  return ok;
}

// Steps a1-a3 of the path: partial soft-max statistics, sampled-token logit,
// finish.  Writes logprob / lse if wanted, and (for the loss) lse in the
// kernels' exponent domain plus logprob - logq in double.
constexpr Gate kNoGate{nullptr, 0};

// Clears the status header, gathers the sampled tokens' logits and (bf16) packs W and H.
static int prepare_operands(const Plan& p, const void* H, const void* W, const int32_t* tokens, char* ws,
                            hipStream_t st) {
  int* status = (int*)(ws + p.off_status);
  float* zy = (float*)(ws + p.off_zy);
  const int64_t T = p.T;
  k_fill_i32<<<1, 64, 0, st>>>(status, kStatusWords, 0);
  OAPL_LAUNCH_CHECK();
  if (T == 0) return OAPL_OK;
  if (p.dtype == OAPL_BF16) {
    if (!prepare_kernels()) return OAPL_ERR_HIP;
    k_gather_logit<bf16_t, float><<<grid1d(T, 4), 256, 0, st>>>((const bf16_t*)H, (const bf16_t*)W, tokens, T, p.d,
                                                                p.V, zy, status);
    OAPL_LAUNCH_CHECK();
    bf16_t* Wp = (bf16_t*)(ws + p.off_Wp);
    bf16_t* Hp = (bf16_t*)(ws + p.off_Hp);
    k_pack_rows<<<dim3(p.n_kt_d, p.n_rt_v), 256, 0, st>>>((const bf16_t*)W, p.V, p.d, p.d, Wp, p.n_kt_d, Cfg::BM);
    OAPL_LAUNCH_CHECK();
    k_pack_rows<<<dim3(p.n_kt_d, (unsigned)p.n_rt_T), 256, 0, st>>>((const bf16_t*)H, T, p.d, p.d, Hp, p.n_kt_d,
                                                                    Cfg::BN);
    OAPL_LAUNCH_CHECK();
  } else {
    k_gather_logit<float, double><<<grid1d(T, 4), 256, 0, st>>>((const float*)H, (const float*)W, tokens, T, p.d, p.V,
                                                                zy, status);
    OAPL_LAUNCH_CHECK();
  }
  return OAPL_OK;
}

// (after prepare_operands)
static int forward_scores(const Plan& p, const void* H, const void* W, const int32_t* tokens, const float* logq,
                          float* logprob_out, float* lse_out, float* entropy_out, char* ws, bool keep_for_loss,
                          hipStream_t st, Gate gate = kNoGate) {
  float2* partials = (float2*)(ws + p.off_partials);
  float* upart = entropy_out ? (float*)(ws + p.off_upart) : nullptr;
  float* zy = (float*)(ws + p.off_zy);
  float* lse2 = keep_for_loss ? (float*)(ws + p.off_lse2) : nullptr;
  double* diff = keep_for_loss ? (double*)(ws + p.off_diff) : nullptr;
  float* omp = keep_for_loss ? (float*)(ws + p.off_omp) : nullptr;
  float* inv = keep_for_loss ? (float*)(ws + p.off_inv) : nullptr;
  const int64_t T = p.T;
  if (T == 0) return OAPL_OK;
  const bool timed = gate.flag == nullptr;

  if (p.dtype == OAPL_BF16) {
    const bf16_t* Wp = (const bf16_t*)(ws + p.off_Wp);
    const bf16_t* Hp = (const bf16_t*)(ws + p.off_Hp);
    const int64_t n_tiles = (T + Cfg::BN - 1) / Cfg::BN;
    const int64_t total = n_tiles * p.n_parts;
    // token tiles per XCD patch: four while a token tile's packed H strip is at most 2 MiB (d <= 2730:
    // +4 % measured at d = 2048), one beyond that (four strips of 3 MiB thrash the 4 MiB L2: -5 % at d = 4096)
    const int patch_tiles = (size_t)p.n_kt_d * kPackBlockBytesB <= ((size_t)2 << 20) ? 4 : 1;
    {
      ScopedKernelTimer tm(kFwdLse, st, timed);
      if (entropy_out)
        k_fwd_lse<Cfg, true><<<(unsigned)round_up(total, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
            Wp, Hp, p.V, T, p.n_kt_d, p.n_parts, patch_tiles, partials, upart, gate);
      else
        k_fwd_lse<Cfg, false><<<(unsigned)round_up(total, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
            Wp, Hp, p.V, T, p.n_kt_d, p.n_parts, patch_tiles, partials, nullptr, gate);
    }
    OAPL_LAUNCH_CHECK();
    k_lse_finish<true><<<grid1d(T, 256), 256, 0, st>>>(partials, p.n_parts, T, zy, logq, logprob_out, lse_out, lse2,
                                                       diff, omp, inv, upart, entropy_out, gate);
    OAPL_LAUNCH_CHECK();
  } else {
    F32Operand A{(const float*)H, p.d, 1}, B{(const float*)W, p.d, 1};
    dim3 grid(grid1d(p.V, 64), grid1d(T, 64));
    k_gemm_f32<<<grid, 256, 0, st>>>(A, B, T, (int64_t)p.V, (int64_t)p.d, EpiLseF32{partials, T, upart});
    OAPL_LAUNCH_CHECK();
    k_lse_finish<false><<<grid1d(T, 256), 256, 0, st>>>(partials, p.n_parts, T, zy, logq, logprob_out, lse_out, lse2,
                                                        diff, omp, inv, upart, entropy_out, kNoGate);
    OAPL_LAUNCH_CHECK();
  }
  return OAPL_OK;
}

// Steps a8-a10, two-pass form: panel by panel, recompute the soft-max tiles into dZ and run
// the two gradient contractions.  `wt_packed`: W^T has been packed already by this call.
static int backward_grads(const Plan& p, const void* H, const void* W, const int32_t* tokens, void* dH, float* dW,
                          char* ws, hipStream_t st, Gate gate = kNoGate, bool wt_packed = false) {
  const int64_t T = p.T;
  const int d = p.d, V = p.V;
  const float* lse2 = (const float*)(ws + p.off_lse2);
  const float* coef = (const float*)(ws + p.off_coef);  // bf16: f_t = c_t (1 - p_y); fp32: c_t
  const float* inv = (const float*)(ws + p.off_inv);
  const bool timed = gate.flag == nullptr;
  if (T == 0) {
    k_fill_f32<<<1024, 256, 0, st>>>(dW, (int64_t)V * d, 0.f, gate);
    OAPL_LAUNCH_CHECK();
    return OAPL_OK;
  }
  if (p.dtype == OAPL_BF16) {
    const bf16_t* Wp = (const bf16_t*)(ws + p.off_Wp);   // packed by prepare_operands
    const bf16_t* Hp = (const bf16_t*)(ws + p.off_Hp);
    bf16_t* WTp = (bf16_t*)(ws + p.off_WTp);
    bf16_t* HTp = (bf16_t*)(ws + p.off_HTp);
    bf16_t* G = (bf16_t*)(ws + p.off_G);
    bf16_t* GT = (bf16_t*)(ws + p.off_GT);
    if (!wt_packed) {
      k_pack_transposed<<<dim3(p.n_kt_v, p.n_rt_d), 256, 0, st>>>((const bf16_t*)W, V, d, d, nullptr, WTp, p.n_kt_v,
                                                                  gate);
      OAPL_LAUNCH_CHECK();
    }
    const int MTv = p.n_rt_v, MTd = p.n_rt_d;
    const int NTv = (V + Cfg::BN - 1) / Cfg::BN;   // vocabulary tiles on the n side (dW contraction)
    const int64_t strip_d = (int64_t)p.n_kt_d * (kPackBlockBytesB / 2);   // one token tile of packed H
    for (int64_t t0 = 0; t0 < T; t0 += p.Tp) {
      const int64_t nv = (T - t0) < p.Tp ? (T - t0) : p.Tp;
      const int64_t Kt = round_up(nv, Cfg::BN);
      const int64_t NTl = Kt / Cfg::BN;
      // (diag(f) H)^T of this panel, packed; token columns in [nv, Kt) come out as zeros
      k_pack_transposed<<<dim3((unsigned)(Kt / kPackK), p.n_rt_d), 256, 0, st>>>(
          (const bf16_t*)H + t0 * d, nv, d, d, coef + t0, HTp, p.n_kt_t, gate);
      OAPL_LAUNCH_CHECK();
      {
        ScopedKernelTimer tm(kBwdDz, st, timed);
        k_bwd_dz<Cfg><<<(unsigned)round_up(MTv * NTl, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
            Wp, Hp + (t0 / Cfg::BN) * strip_d, V, nv, p.n_kt_d, tokens + t0, lse2 + t0, inv + t0, G, p.n_kt_g, GT,
            p.n_kt_t, gate);
      }
      OAPL_LAUNCH_CHECK();
      {
        ScopedKernelTimer tm(kBwdDh, st, timed);
        k_bwd_dh<Cfg><<<(unsigned)round_up(MTd * NTl, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
            WTp, p.n_kt_v, G, p.n_kt_g, d, nv, p.n_kt_v, coef + t0, (bf16_t*)dH + t0 * d, gate);
      }
      OAPL_LAUNCH_CHECK();
      {
        ScopedKernelTimer tm(kBwdDw, st, timed);
        k_bwd_dw<Cfg><<<(unsigned)round_up((int64_t)MTd * NTv, kNumCU), Cfg::NT, Cfg::LDS_BYTES, st>>>(
            HTp, GT, p.n_kt_t, d, V, (int)(Kt / kPackK), dW, t0 > 0 ? 1 : 0, gate);
      }
      OAPL_LAUNCH_CHECK();
    }
  } else {
    float* dZ = (float*)(ws + p.off_G);
    for (int64_t t0 = 0; t0 < T; t0 += p.Tp) {
      const int64_t nv = (T - t0) < p.Tp ? (T - t0) : p.Tp;
      const float* Hp = (const float*)H + t0 * d;
      {
        F32Operand A{Hp, d, 1}, B{(const float*)W, d, 1};
        dim3 grid(grid1d(V, 64), grid1d(nv, 64));
        k_gemm_f32<<<grid, 256, 0, st>>>(A, B, nv, (int64_t)V, (int64_t)d,
                                         EpiDzF32{tokens + t0, lse2 + t0, coef + t0, dZ, (int64_t)V});
        OAPL_LAUNCH_CHECK();
      }
      {  // dH[t][j] = sum_v dZ[t][v] W[v][j]
        F32Operand A{dZ, V, 1}, B{(const float*)W, 1, d};
        dim3 grid(grid1d(d, 64), grid1d(nv, 64));
        k_gemm_f32<<<grid, 256, 0, st>>>(A, B, nv, (int64_t)d, (int64_t)V, EpiStoreF32{(float*)dH + t0 * d, d, 0});
        OAPL_LAUNCH_CHECK();
      }
      {  // dW[v][j] (+)= sum_t dZ[t][v] H[t][j]
        F32Operand A{dZ, 1, V}, B{Hp, 1, d};
        dim3 grid(grid1d(d, 64), grid1d(V, 64));
        k_gemm_f32<<<grid, 256, 0, st>>>(A, B, (int64_t)V, (int64_t)d, nv, EpiStoreF32{dW, d, t0 > 0 ? 1 : 0});
        OAPL_LAUNCH_CHECK();
      }
    }
  }
  return OAPL_OK;
}

// Steps a1-a3 and a8-a10 in ONE pass over the logits (bf16, T > 0).  Per panel of token rows:
// k_sweep writes the unnormalised soft-max panel and its row sums, k_sweep_finish turns the sums
// into log-probs; the objective's O(T) kernels (`objective`, which must fill coef[t] = c_t * nis[t]
// for every token whose rollout is complete and may run any number of times) then give the row
// factors, and the two gradient contractions consume the panel.  A rollout may straddle a panel
// boundary, so a panel's contractions run after the NEXT panel's sweep (two panel buffers); by
// then every rollout that touches it is complete, because no rollout is longer than a panel
// (k_sweep_plan raises the fallback flag otherwise).  All kernels here run only while the flag is 0.
template <class Objective>
static int sweep_path(const Plan& p, const void* H, const void* W, const int32_t* tokens, const float* logq,
                      const int64_t* seq_offsets, float* logprob_out, void* dH, float* dW, char* ws, hipStream_t st,
                      Objective&& objective) {
  const int64_t T = p.T;
  const int d = p.d, V = p.V;
  int* flag = (int*)(ws + p.off_status) + kFlagWord;
  const Gate fast{flag, 0};
  const bf16_t* Wp = (const bf16_t*)(ws + p.off_Wp);
  const bf16_t* Hp = (const bf16_t*)(ws + p.off_Hp);
  bf16_t* WTp = (bf16_t*)(ws + p.off_WTp);
  bf16_t* HTp = (bf16_t*)(ws + p.off_HTp);
  auto Gbuf = [&](int64_t k) { return (bf16_t*)(ws + p.off_G + (size_t)(k % p.n_buf) * p.size_G); };
  auto GTbuf = [&](int64_t k) { return (bf16_t*)(ws + p.off_GT + (size_t)(k % p.n_buf) * p.size_GT); };
  float2* sample = (float2*)(ws + p.off_partials);
  const float* zy = (const float*)(ws + p.off_zy);
  float* ref2 = (float*)(ws + p.off_ref2);
  float* spart = (float*)(ws + p.off_spart);
  double* diff = (double*)(ws + p.off_diff);
  float* nis = (float*)(ws + p.off_inv);
  const float* coef = (const float*)(ws + p.off_coef);
  const int MTv = p.n_rt_v, MTd = p.n_rt_d;
  const int NTv = (V + Cfg::BN - 1) / Cfg::BN;     // vocabulary tiles on the n side (dW contraction)
  const int64_t strip_d = (int64_t)p.n_kt_d * (kPackBlockBytesB / 2);   // one token tile of packed H
  const int64_t n_tiles = (T + Cfg::BN - 1) / Cfg::BN;

  // a rollout may span at most n_buf - 1 panels' worth of rows (any length if the batch is one panel)
  k_sweep_plan<<<grid1d(p.n_seq > 0 ? p.n_seq : 1, 256), 256, 0, st>>>(
      seq_offsets, p.n_seq, T, p.n_buf > 1 ? (int64_t)(p.n_buf - 1) * p.Tp : p.Tp, flag);
  OAPL_LAUNCH_CHECK();
  k_pack_transposed<<<dim3(p.n_kt_v, p.n_rt_d), 256, 0, st>>>((const bf16_t*)W, V, d, d, nullptr, WTp, p.n_kt_v,
                                                              kNoGate);
  OAPL_LAUNCH_CHECK();
  // reference exponents: running maximum over the first vocabulary tile, one workgroup per token tile
  k_fwd_lse<Cfg, false><<<(unsigned)round_up(n_tiles, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
      Wp, Hp, V < Cfg::BM ? V : Cfg::BM, T, p.n_kt_d, 1, 1, sample, nullptr, fast);
  OAPL_LAUNCH_CHECK();
  k_sweep_ref<<<grid1d(T, 256), 256, 0, st>>>(sample, zy, T, ref2);
  OAPL_LAUNCH_CHECK();
  // rows not swept yet must read as "no contribution" in the objective's kernels
  k_fill_f64<<<grid1d(T, 256 * 8), 256, 0, st>>>(diff, T, 0.0);
  OAPL_LAUNCH_CHECK();
  k_fill_f32<<<grid1d(T, 256 * 8), 256, 0, st>>>(nis, T, 0.f);
  OAPL_LAUNCH_CHECK();

  const int64_t n_panels = (T + p.Tp - 1) / p.Tp;
  auto gradients = [&](int64_t k) -> int {
    const int64_t t0 = k * p.Tp;
    const int64_t nv = (T - t0) < p.Tp ? (T - t0) : p.Tp;
    const int64_t Kt = round_up(nv, Cfg::BN);
    const int64_t NTl = Kt / Cfg::BN;
    if (int rc = objective(fast, nis)) return rc;
    k_pack_transposed<<<dim3((unsigned)(Kt / kPackK), p.n_rt_d), 256, 0, st>>>(
        (const bf16_t*)H + t0 * d, nv, d, d, coef + t0, HTp, p.n_kt_t, fast);
    OAPL_LAUNCH_CHECK();
    {
      ScopedKernelTimer tm(kBwdDh, st);
      k_bwd_dh<Cfg><<<(unsigned)round_up(MTd * NTl, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
          WTp, p.n_kt_v, Gbuf(k), p.n_kt_g, d, nv, p.n_kt_v, coef + t0, (bf16_t*)dH + t0 * d, fast);
    }
    OAPL_LAUNCH_CHECK();
    {
      ScopedKernelTimer tm(kBwdDw, st);
      k_bwd_dw<Cfg><<<(unsigned)round_up((int64_t)MTd * NTv, kNumCU), Cfg::NT, Cfg::LDS_BYTES, st>>>(
          HTp, GTbuf(k), p.n_kt_t, d, V, (int)(Kt / kPackK), dW, k > 0 ? 1 : 0, fast);
    }
    OAPL_LAUNCH_CHECK();
    return OAPL_OK;
  };
  for (int64_t k = 0; k < n_panels; ++k) {
    const int64_t t0 = k * p.Tp;
    const int64_t nv = (T - t0) < p.Tp ? (T - t0) : p.Tp;
    const int64_t NTl = round_up(nv, Cfg::BN) / Cfg::BN;
    {
      ScopedKernelTimer tm(kSweep, st);
      k_sweep<Cfg><<<(unsigned)round_up(MTv * NTl, 8), Cfg::NT, Cfg::LDS_BYTES, st>>>(
          Wp, Hp + (t0 / Cfg::BN) * strip_d, V, nv, p.n_kt_d, ref2 + t0, Gbuf(k), p.n_kt_g, GTbuf(k),
          p.n_kt_t, spart, p.Tp, fast);
    }
    OAPL_LAUNCH_CHECK();
    k_sweep_finish<<<grid1d(nv, kFinishRows), kFinishSlices * kFinishRows, 0, st>>>(
        spart, MTv, p.Tp, nv, ref2 + t0, zy + t0, logq + t0, tokens + t0, V,
        logprob_out ? logprob_out + t0 : nullptr, diff + t0, nis + t0, Gbuf(k), p.n_kt_g, GTbuf(k), p.n_kt_t, flag,
        fast);
    OAPL_LAUNCH_CHECK();
    if (k >= p.n_buf - 1 && p.n_buf > 1)
      if (int rc = gradients(k - (p.n_buf - 1))) return rc;
  }
  for (int64_t k = n_panels - (p.n_buf > 1 ? p.n_buf - 1 : 1); k < n_panels; ++k)
    if (int rc = gradients(k)) return rc;
  return OAPL_OK;
}

static int check_workspace(const void* ws, size_t have, size_t need) {
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || have < need) return OAPL_ERR_WORKSPACE;
  return OAPL_OK;
}

// The plan of a loss call: the workspace the caller hands over is the budget.  Panel size first:
// the default panel (the fastest) if two buffers of it fit, else the largest that does.  Then as
// many panel buffers as fit (and the batch has panels): they decide how long a rollout the single
// sweep serves, not how fast it runs.
static int fit_plan(Plan& p, int64_t T, int d, int V, int n_seq, int n_groups, int dtype, bool bwd, const void* ws,
                    size_t have) {
  if (!make_plan(p, T, d, V, n_seq, n_groups, dtype, bwd)) return OAPL_ERR_SHAPE;
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0) return OAPL_ERR_WORKSPACE;
  if (!bwd) return p.total <= have ? OAPL_OK : OAPL_ERR_WORKSPACE;
  if (p.total > have) {
    const int64_t step = dtype == OAPL_BF16 ? Cfg::BN : 64;
    bool found = false;
    for (int64_t rows = (p.Tp - 1) / step * step; rows >= step && !found; rows -= step) {
      Plan q;
      if (make_plan(q, T, d, V, n_seq, n_groups, dtype, bwd, rows) && q.total <= have) {
        p = q;
        found = true;
      }
    }
    if (!found) return OAPL_ERR_WORKSPACE;
  }
  if (p.sweep && p.n_buf >= 2) {
    const size_t per_buffer = p.size_G + p.size_GT;
    const int64_t extra = (int64_t)((have - p.total) / per_buffer);
    if (extra > 0) {
      Plan q;
      if (make_plan(q, T, d, V, n_seq, n_groups, dtype, bwd, p.Tp, p.n_buf + extra, p.Tp) && q.total <= have) p = q;
    }
  }
  return OAPL_OK;
}

static int loss_impl(const void* H, const void* W, const int32_t* tokens, const float* logq,
                     const int64_t* seq_offsets, const float* rewards, const int32_t* group_ids, int64_t T, int32_t d,
                     int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype, float beta_value, float beta_loss,
                     float loss_scale, uint32_t flags, float* loss_out, float* logprob_out, float* seq_logratio_out,
                     float* vstar_out, void* dH, float* dW, void* workspace, size_t workspace_bytes, void* stream,
                     bool checks_only = false) {
  if (dtype != OAPL_F32 && dtype != OAPL_BF16) return OAPL_ERR_DTYPE;
  if (flags & ~(uint32_t)OAPL_FLAG_TWO_PASS) return OAPL_ERR_SHAPE;
  const bool bwd = (dH != nullptr) || (dW != nullptr);
  Plan p;
  if (!make_plan(p, T, d, V, n_seq, n_groups, dtype, bwd)) return OAPL_ERR_SHAPE;
  // gradients come as a pair; an empty batch has no dH rows, so its pointer may be NULL
  if (!W || !seq_offsets || !loss_out || (bwd && (!dW || (T > 0 && !dH)))) return OAPL_ERR_NULL;
  if (T > 0 && (!H || !tokens || !logq)) return OAPL_ERR_NULL;
  if (n_seq > 0 && (!rewards || !group_ids)) return OAPL_ERR_NULL;
  if (!(beta_value > 0.f) || !(beta_loss > 0.f) || !isfinite(beta_value) || !isfinite(beta_loss) ||
      !isfinite(loss_scale))
    return OAPL_ERR_BETA;
  if (int rc = fit_plan(p, T, d, V, n_seq, n_groups, dtype, bwd, workspace, workspace_bytes)) return rc;
  if (checks_only) return OAPL_OK;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  int* status = (int*)(ws + p.off_status);
  double* Delta = (double*)(ws + p.off_delta);
  float* cseq = (float*)(ws + p.off_cseq);
  float* coef = (float*)(ws + p.off_coef);

  // Steps a4-a7 from logprob - logq [T]: per-rollout sums, Eq. 2, Eq. 3, token coefficients
  // coef[t] = c_t * factor[t] (factor = NULL: c_t itself).
  auto objective = [&](Gate gate, const float* factor) -> int {
    if (n_seq > 0) {
      k_segmented_sum<double><<<n_seq, 256, 0, st>>>((const double*)(ws + p.off_diff), seq_offsets, n_seq, T, Delta,
                                                     gate);
      OAPL_LAUNCH_CHECK();
    }
    k_residual_loss<<<1, 256, 0, st>>>(Delta, rewards, group_ids, seq_offsets, n_seq, n_groups, T,
                                       (double)beta_loss, (double)loss_scale, (const double*)(ws + p.off_vstar), cseq,
                                       loss_out, seq_logratio_out, status, gate);
    OAPL_LAUNCH_CHECK();
    if (bwd && T > 0) {
      k_fill_f32<<<grid1d(T, 256 * 8), 256, 0, st>>>(coef, T, 0.f, gate);
      OAPL_LAUNCH_CHECK();
      if (n_seq > 0) {
        k_token_coefficients<<<n_seq, 256, 0, st>>>(cseq, seq_offsets, n_seq, T, factor, coef, gate);
        OAPL_LAUNCH_CHECK();
      }
    }
    return OAPL_OK;
  };

  if (int rc = prepare_operands(p, H, W, tokens, ws, st)) return rc;
  // Eq. 2 needs the rewards only: one wavefront per prompt, before anything is scored
  k_group_value<<<grid1d(n_groups, 4), 256, 0, st>>>(rewards, group_ids, n_seq, n_groups, (double)beta_value,
                                                     (double*)(ws + p.off_vstar), vstar_out, status, kNoGate);
  OAPL_LAUNCH_CHECK();
  // bf16 with gradients: one sweep over the logits; the two-pass path behind it runs only if the
  // sweep's preconditions fail on this call's data (decided on the device, in stream order)
  const bool sweep = bwd && T >= kSweepMinTokens && p.sweep && !(flags & OAPL_FLAG_TWO_PASS);
  Gate slow = kNoGate;
  if (sweep) {
    if (int rc = sweep_path(p, H, W, tokens, logq, seq_offsets, logprob_out, dH, dW, ws, st, objective)) return rc;
    slow = Gate{status + kFlagWord, 1};
  }
  if (int rc = forward_scores(p, H, W, tokens, logq, logprob_out, nullptr, nullptr, ws, true, st, slow)) return rc;
  const float* factor = (bwd && p.dtype == OAPL_BF16) ? (const float*)(ws + p.off_omp) : nullptr;
  if (int rc = objective(slow, factor)) return rc;
  if (!bwd) return OAPL_OK;
  return backward_grads(p, H, W, tokens, dH, dW, ws, st, slow, sweep);
}

// The paper's baseline objective on the same fused head (Sec. 2): scores, group advantages,
// clipped importance-weighted token terms, then the same backward with other coefficients.
static int grpo_impl(const void* H, const void* W, const int32_t* tokens, const float* logq, const float* logp_old,
                     const int64_t* seq_offsets, const float* rewards, const int32_t* group_ids, int64_t T, int32_t d,
                     int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype, float clip_eps, float adv_eps,
                     float loss_scale, uint32_t flags, float* loss_out, float* logprob_out, float* adv_out, void* dH,
                     float* dW, void* workspace, size_t workspace_bytes, void* stream) {
  if (dtype != OAPL_F32 && dtype != OAPL_BF16) return OAPL_ERR_DTYPE;
  if (flags & ~(uint32_t)OAPL_FLAG_TWO_PASS) return OAPL_ERR_SHAPE;
  const bool bwd = (dH != nullptr) || (dW != nullptr);
  Plan p;
  if (!make_plan(p, T, d, V, n_seq, n_groups, dtype, bwd)) return OAPL_ERR_SHAPE;
  if (!W || !seq_offsets || !loss_out || (bwd && (!dW || (T > 0 && !dH)))) return OAPL_ERR_NULL;
  if (T > 0 && (!H || !tokens || !logq || !logp_old)) return OAPL_ERR_NULL;
  if (n_seq > 0 && (!rewards || !group_ids)) return OAPL_ERR_NULL;
  if (!(clip_eps >= 0.f) || !(clip_eps < 1.f) || !(adv_eps >= 0.f) || !isfinite(adv_eps) || !isfinite(loss_scale))
    return OAPL_ERR_BETA;
  if (int rc = fit_plan(p, T, d, V, n_seq, n_groups, dtype, bwd, workspace, workspace_bytes)) return rc;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  int* status = (int*)(ws + p.off_status);
  float* adv = (float*)(ws + p.off_cseq);
  double* gstat = (double*)(ws + p.off_vstar);          // [2 n_groups]: mean, std
  double* wseq = (double*)(ws + p.off_gw);              // [n_seq + n_groups]
  double* seqterm = (double*)(ws + p.off_delta);
  float* coef = (float*)(ws + p.off_coef);

  auto objective = [&](Gate gate, const float* factor) -> int {
    if (T > 0) {
      k_fill_f32<<<grid1d(T, 256 * 8), 256, 0, st>>>(coef, T, 0.f, gate);
      OAPL_LAUNCH_CHECK();
    }
    if (n_seq > 0) {
      k_grpo_tokens<<<n_seq, 256, 0, st>>>((const double*)(ws + p.off_diff), logq, logp_old, seq_offsets, n_seq, T,
                                           adv, wseq, (double)clip_eps, factor, coef, seqterm, gate);
      OAPL_LAUNCH_CHECK();
    }
    k_grpo_loss<<<1, 256, 0, st>>>(seqterm, n_seq, status, loss_out, gate);
    OAPL_LAUNCH_CHECK();
    return OAPL_OK;
  };

  if (int rc = prepare_operands(p, H, W, tokens, ws, st)) return rc;
  k_grpo_group_stats<<<grid1d(n_groups, 4), 256, 0, st>>>(rewards, group_ids, n_seq, n_groups, gstat,
                                                          gstat + n_groups, wseq + (n_seq > 0 ? n_seq : 1), status,
                                                          kNoGate);
  OAPL_LAUNCH_CHECK();
  k_grpo_advantage<<<grid1d(n_seq > 0 ? n_seq : 1, 256), 256, 0, st>>>(
      rewards, group_ids, seq_offsets, n_seq, n_groups, T, (double)adv_eps, (double)loss_scale, gstat,
      gstat + n_groups, wseq + (n_seq > 0 ? n_seq : 1), adv, wseq, adv_out, status, kNoGate);
  OAPL_LAUNCH_CHECK();
  const bool sweep = bwd && T >= kSweepMinTokens && p.sweep && !(flags & OAPL_FLAG_TWO_PASS);
  Gate slow = kNoGate;
  if (sweep) {
    if (int rc = sweep_path(p, H, W, tokens, logq, seq_offsets, logprob_out, dH, dW, ws, st, objective)) return rc;
    slow = Gate{status + kFlagWord, 1};
  }
  if (int rc = forward_scores(p, H, W, tokens, logq, logprob_out, nullptr, nullptr, ws, true, st, slow)) return rc;
  const float* factor = (bwd && p.dtype == OAPL_BF16) ? (const float*)(ws + p.off_omp) : nullptr;
  if (int rc = objective(slow, factor)) return rc;
  if (!bwd) return OAPL_OK;
  return backward_grads(p, H, W, tokens, dH, dW, ws, st, slow, sweep);
}

// Scratch of the entry point that allocates nothing: every GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (the array's name is only a host-side stand-in
// for it): resolved once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return OAPL_ERR_HIP;
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return OAPL_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return OAPL_OK;
}

}  // namespace oapl

using namespace oapl;

extern "C" {

const char* oapl_status_string(int32_t status) {
  switch (status) {
    case OAPL_OK: return "ok";
    case OAPL_ERR_NULL: return "a required pointer is NULL";
    case OAPL_ERR_SHAPE: return "a size is non-positive or unsupported";
    case OAPL_ERR_DTYPE: return "unknown dtype";
    case OAPL_ERR_OFFSETS: return "seq_offsets malformed";
    case OAPL_ERR_GROUP: return "group id out of range or empty group";
    case OAPL_ERR_BETA: return "beta must be positive and finite (loss_scale finite)";
    case OAPL_ERR_WORKSPACE: return "workspace NULL, misaligned or too small";
    case OAPL_ERR_HIP: return "HIP launch or runtime call failed";
    case OAPL_ERR_TOKEN_RANGE: return "sampled token outside [0, V)";
    case OAPL_ERR_SCRATCH_LIMIT: return "sizes need more than the library's 64 MiB static scratch";
    default: return "unknown status";
  }
}

size_t oapl_workspace_bytes(int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype,
                            int32_t with_backward) {
  Plan p;
  if (!make_plan(p, T, d, V, n_seq, n_groups, dtype, with_backward != 0)) return 0;
  return p.total;
}

size_t oapl_workspace_bytes_for(int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype,
                                int32_t with_backward, int64_t max_panel_rows, int64_t max_rollout_len,
                                int64_t* panel_rows_out, int32_t* panel_buffers_out) {
  Plan p, full;
  if (!make_plan(p, T, d, V, n_seq, n_groups, dtype, with_backward != 0, max_panel_rows)) return 0;
  if (!make_plan(full, T, d, V, n_seq, n_groups, dtype, with_backward != 0)) return 0;
  // Buffers for the longest rollout, 1 + ceil(len / panel): only at the library's own panel size.  A
  // loss call derives its plan from the byte count alone, and k buffers of a smaller panel could not
  // be told from two buffers of a panel k / 2 times as large (which it prefers: larger panels are faster).
  if (max_rollout_len > p.Tp && p.n_buf >= 2 && p.Tp == full.Tp) {
    const int64_t want = 1 + (max_rollout_len + p.Tp - 1) / p.Tp;
    Plan q;
    if (!make_plan(q, T, d, V, n_seq, n_groups, dtype, with_backward != 0, p.Tp, want, p.Tp)) return 0;
    p = q;
  }
  if (panel_rows_out) *panel_rows_out = p.Tp;
  if (panel_buffers_out) *panel_buffers_out = p.n_buf;
  return p.total;
}

int32_t oapl_logprob_fwd(const void* H, const void* W, const int32_t* tokens, int64_t T, int32_t d, int32_t V,
                         int32_t dtype, float* logprob_out, float* lse_out, float* entropy_out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (dtype != OAPL_F32 && dtype != OAPL_BF16) return OAPL_ERR_DTYPE;
  Plan p;
  if (!make_plan(p, T, d, V, 0, 1, dtype, false)) return OAPL_ERR_SHAPE;
  if (!W) return OAPL_ERR_NULL;
  if (T > 0 && (!H || !tokens || !logprob_out)) return OAPL_ERR_NULL;
  if (int rc = check_workspace(workspace, workspace_bytes, p.total)) return rc;
  if (int rc = prepare_operands(p, H, W, tokens, (char*)workspace, (hipStream_t)stream)) return rc;
  return forward_scores(p, H, W, tokens, nullptr, logprob_out, lse_out, entropy_out, (char*)workspace, false,
                        (hipStream_t)stream);
}

int32_t oapl_sample_tokens(const void* H, const void* W, int64_t T, int32_t d, int32_t V, int32_t dtype,
                           float temperature, uint64_t seed, int32_t* tokens_out, float* score_out, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (dtype != OAPL_F32 && dtype != OAPL_BF16) return OAPL_ERR_DTYPE;
  Plan p;
  if (!make_plan(p, T, d, V, 0, 1, dtype, false)) return OAPL_ERR_SHAPE;
  if (!W) return OAPL_ERR_NULL;
  if (T > 0 && (!H || !tokens_out)) return OAPL_ERR_NULL;
  if (!(temperature > 0.f) || !isfinite(temperature)) return OAPL_ERR_BETA;
  if (int rc = check_workspace(workspace, workspace_bytes, p.total)) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  k_fill_i32<<<1, 64, 0, st>>>((int*)(ws + p.off_status), kStatusWords, 0);
  OAPL_LAUNCH_CHECK();
  if (T == 0) return OAPL_OK;
  float2* partials = (float2*)(ws + p.off_partials);
  const float inv_t = 1.0f / temperature;
  const uint32_t s_lo = (uint32_t)seed, s_hi = (uint32_t)(seed >> 32);
  if (dtype == OAPL_BF16) {
    if (!prepare_kernels()) return OAPL_ERR_HIP;
    bf16_t* Wp = (bf16_t*)(ws + p.off_Wp);
    bf16_t* Hp = (bf16_t*)(ws + p.off_Hp);
    k_pack_rows<<<dim3(p.n_kt_d, p.n_rt_v), 256, 0, st>>>((const bf16_t*)W, V, d, d, Wp, p.n_kt_d, Cfg::BM);
    OAPL_LAUNCH_CHECK();
    const int64_t n_tiles = (T + CfgSample::BN - 1) / CfgSample::BN;
    k_pack_rows<<<dim3(p.n_kt_d, (unsigned)n_tiles), 256, 0, st>>>((const bf16_t*)H, T, d, d, Hp, p.n_kt_d,
                                                                   CfgSample::BN);
    OAPL_LAUNCH_CHECK();
    const int64_t total = n_tiles * p.n_parts_s;
    {
      ScopedKernelTimer tm(kFwdSample, st);
      k_fwd_sample<CfgSample><<<(unsigned)round_up(total, 8), CfgSample::NT, CfgSample::LDS_BYTES, st>>>(
          Wp, Hp, V, T, p.n_kt_d, p.n_parts_s, inv_t, s_lo, s_hi, partials);
    }
    OAPL_LAUNCH_CHECK();
  } else {
    F32Operand A{(const float*)H, d, 1}, B{(const float*)W, d, 1};
    dim3 grid(grid1d(V, 64), grid1d(T, 64));
    k_gemm_f32<<<grid, 256, 0, st>>>(A, B, T, (int64_t)V, (int64_t)d, EpiSampleF32{partials, T, inv_t, s_lo, s_hi});
    OAPL_LAUNCH_CHECK();
  }
  k_sample_finish<<<grid1d(T, 256), 256, 0, st>>>(partials, p.n_parts_s, T, tokens_out, score_out);
  OAPL_LAUNCH_CHECK();
  return OAPL_OK;
}

int32_t oapl_loss_fwd_bwd(const void* H, const void* W, const int32_t* tokens, const float* logq,
                          const int64_t* seq_offsets, const float* rewards, const int32_t* group_ids, int64_t T,
                          int32_t d, int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype, float beta,
                          float loss_scale, float* loss_out, float* logprob_out, float* seq_logratio_out,
                          float* vstar_out, void* dH, float* dW, void* workspace, size_t workspace_bytes,
                          void* stream) {
  return loss_impl(H, W, tokens, logq, seq_offsets, rewards, group_ids, T, d, V, n_seq, n_groups, dtype, beta, beta,
                   loss_scale, 0u, loss_out, logprob_out, seq_logratio_out, vstar_out, dH, dW, workspace,
                   workspace_bytes, stream);
}

int32_t oapl_loss_fwd_bwd_two_beta(const void* H, const void* W, const int32_t* tokens, const float* logq,
                                   const int64_t* seq_offsets, const float* rewards, const int32_t* group_ids,
                                   int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype,
                                   float beta_value, float beta_loss, float loss_scale, uint32_t flags,
                                   float* loss_out, float* logprob_out, float* seq_logratio_out, float* vstar_out,
                                   void* dH, float* dW, void* workspace, size_t workspace_bytes, void* stream) {
  return loss_impl(H, W, tokens, logq, seq_offsets, rewards, group_ids, T, d, V, n_seq, n_groups, dtype, beta_value,
                   beta_loss, loss_scale, flags, loss_out, logprob_out, seq_logratio_out, vstar_out, dH, dW, workspace,
                   workspace_bytes, stream);
}

int32_t oapl_loss_fwd_bwd_noalloc(const void* H, const void* W, const int32_t* tokens, const float* logq,
                                  const int64_t* seq_offsets, const float* rewards, const int32_t* group_ids,
                                  int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups, int32_t dtype,
                                  float beta, float loss_scale, float* loss_out, float* logprob_out,
                                  float* seq_logratio_out, float* vstar_out, void* dH, float* dW, void* stream) {
  // every host-side check first, against an aligned stand-in of the scratch's size; nothing is launched
  int rc = loss_impl(H, W, tokens, logq, seq_offsets, rewards, group_ids, T, d, V, n_seq, n_groups, dtype, beta, beta,
                     loss_scale, 0u, loss_out, logprob_out, seq_logratio_out, vstar_out, dH, dW, (void*)(uintptr_t)256,
                     kStaticScratchBytes, stream, true);
  if (rc == OAPL_ERR_WORKSPACE) return OAPL_ERR_SCRATCH_LIMIT;
  if (rc != OAPL_OK) return rc;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws)) != OAPL_OK) return rc;
  return loss_impl(H, W, tokens, logq, seq_offsets, rewards, group_ids, T, d, V, n_seq, n_groups, dtype, beta, beta,
                   loss_scale, 0u, loss_out, logprob_out, seq_logratio_out, vstar_out, dH, dW, ws, kStaticScratchBytes,
                   stream);
}

int32_t oapl_grpo_loss_fwd_bwd(const void* H, const void* W, const int32_t* tokens, const float* logq,
                               const float* logp_old, const int64_t* seq_offsets, const float* rewards,
                               const int32_t* group_ids, int64_t T, int32_t d, int32_t V, int32_t n_seq,
                               int32_t n_groups, int32_t dtype, float clip_eps, float adv_eps, float loss_scale,
                               uint32_t flags, float* loss_out, float* logprob_out, float* adv_out, void* dH,
                               float* dW, void* workspace, size_t workspace_bytes, void* stream) {
  return grpo_impl(H, W, tokens, logq, logp_old, seq_offsets, rewards, group_ids, T, d, V, n_seq, n_groups, dtype,
                   clip_eps, adv_eps, loss_scale, flags, loss_out, logprob_out, adv_out, dH, dW, workspace, workspace_bytes,
                   stream);
}

int32_t oapl_segmented_sum_f32(const float* x, const int64_t* seq_offsets, int32_t n_seq, double* out, void* stream) {
  if (n_seq < 0) return OAPL_ERR_SHAPE;
  if (n_seq == 0) return OAPL_OK;
  if (!x || !seq_offsets || !out) return OAPL_ERR_NULL;
  k_segmented_sum<float><<<n_seq, 256, 0, (hipStream_t)stream>>>(x, seq_offsets, n_seq, -1, out);
  OAPL_LAUNCH_CHECK();
  return OAPL_OK;
}

int32_t oapl_timing_enable(int32_t enable) {
  TimingState& t = timing();
  std::lock_guard<std::mutex> g(t.mu);
  for (auto& v : t.ev) {
    for (auto& e : v) {
      (void)hipEventDestroy(e.first);
      (void)hipEventDestroy(e.second);
    }
    v.clear();
  }
  t.on = enable != 0;
  return OAPL_OK;
}

int32_t oapl_timing_read(int32_t kernel, double* total_ms, int64_t* launches) {
  if (kernel < 0 || kernel >= kNumDense) return OAPL_ERR_SHAPE;
  if (!total_ms || !launches) return OAPL_ERR_NULL;
  TimingState& t = timing();
  std::lock_guard<std::mutex> g(t.mu);
  double sum = 0.0;
  for (auto& e : t.ev[kernel]) {
    if (hipEventSynchronize(e.second) != hipSuccess) return OAPL_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e.first, e.second) != hipSuccess) return OAPL_ERR_HIP;
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int64_t)t.ev[kernel].size();
  return OAPL_OK;
}

int32_t oapl_read_path_taken(const void* workspace, void* stream, int32_t* two_pass_out) {
  if (!workspace || !two_pass_out) return OAPL_ERR_NULL;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return OAPL_ERR_HIP;
  int32_t v = 0;
  if (hipMemcpy(&v, (const int32_t*)workspace + kFlagWord, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess)
    return OAPL_ERR_HIP;
  *two_pass_out = v != 0;
  return OAPL_OK;
}

int32_t oapl_read_device_status(const void* workspace, void* stream, int32_t* status_out) {
  if (!workspace || !status_out) return OAPL_ERR_NULL;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return OAPL_ERR_HIP;
  int32_t v = 0;
  if (hipMemcpy(&v, workspace, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return OAPL_ERR_HIP;
  *status_out = v;
  return OAPL_OK;
}

}  // extern "C"
