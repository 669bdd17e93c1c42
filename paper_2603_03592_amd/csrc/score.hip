// Check statistics between submissions and a reference point, the flag rule, and the EMA
// reference update.  All three kernels are streaming (HBM-bound) passes.
//
//   score_tokens_kernel : one pass over claim and reference.  Per token it forms the sums the
//                         whole distance family needs (Omega_L1, Omega_L2, Omega_SFR of the
//                         paragraph "Choice of Distance Measure", and the per-token relative
//                         L2), then folds 16 tokens into one partial record.
//   score_finalize_kernel: deterministic reduction of the records of one submission, the
//                         scores, and the flag Gamma > tau (Eq. test_statistic; a submission
//                         is flagged when any enabled metric exceeds its threshold).
//   ema_update_kernel   : Eq. momentum_def over the un-flagged submissions.
#include <mutex>

#include "common.h"

namespace sv {

namespace {

constexpr int kTPW = kScoreTokensPerWG / 4;  // tokens per wave

// NEED_L1 / NEED_Z / NEED_SFR prune the sums a launch does not need (the statistic family is
// requested by mask): with only the relative L2 enabled a token costs two FMAs per element and the
// pass is bound by HBM; with all eight sums it is bound by the vector ALUs (about 18 ops/element).
template <typename EC, typename ER, bool NEED_L1, bool NEED_Z, bool NEED_SFR>
__global__ __launch_bounds__(256) void score_tokens_kernel(const EC* __restrict__ claims, int64_t claim_stride,
                                                           const ER* __restrict__ ref, int64_t ref_stride, int64_t T, int D,
                                                           int n_claims, int tiles_per_claim, float* __restrict__ token_scores,
                                                           ScorePartial* __restrict__ partials) {
  // Workgroup ids go round-robin over the 8 XCDs (each with its own L2): ids congruent mod 8 get a contiguous run of
  // token tiles, and within a run the claim index varies fastest, so the submissions that share a tile of the
  // reference run together on one XCD and fetch it from memory once instead of once per XCD.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int claim = slot % n_claims;
  const int tile = xcd * ((tiles_per_claim + 7) >> 3) + slot / n_claims;
  if (tile >= tiles_per_claim) return;               // the last XCD's run may be short (whole workgroup leaves)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const EC* cbase = claims + (int64_t)claim * claim_stride;
  const ER* rbase = ref + (int64_t)claim * ref_stride;

  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  float best = -1.0f;
  int best_t = 0, bad = 0;

  for (int i = 0; i < kTPW; ++i) {
    const int64_t t = (int64_t)tile * kScoreTokensPerWG + i * 4 + wave;
    if (t >= T) break;  // uniform per wave
    const EC* c = cbase + t * D;
    const ER* r = rbase + t * D;
    float sc = 0, sr = 0, scc = 0, srr = 0, sad = 0, sdd = 0;
    int nsi = 0;
    auto accumulate = [&](const float (&cv)[8], const float (&rv)[8]) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float a = cv[j], b = rv[j], d = a - b;
        srr = fmaf(b, b, srr); sdd = fmaf(d, d, sdd);
        if (NEED_Z) { sc += a; sr += b; scc = fmaf(a, a, scc); }
        if (NEED_L1) sad += fabsf(d);
        // sign(a) != sign(b) with sign(0) = 0: the two signs agree iff both "positive" and both "negative" tests agree
        if (NEED_SFR) nsi += (int)(((a > 0.0f) != (b > 0.0f)) | ((a < 0.0f) != (b < 0.0f)));
      }
    };
    int k = lane * 8;
    for (; k + 1536 < D; k += 2048) {                 // four 16-byte loads of each operand in flight per lane
      float c0[8], c1[8], c2[8], c3[8], r0[8], r1[8], r2[8], r3[8];
      load8(c + k, c0); load8(c + k + 512, c1); load8(c + k + 1024, c2); load8(c + k + 1536, c3);
      load8(r + k, r0); load8(r + k + 512, r1); load8(r + k + 1024, r2); load8(r + k + 1536, r3);
      accumulate(c0, r0); accumulate(c1, r1); accumulate(c2, r2); accumulate(c3, r3);
    }
    for (; k < D; k += 512) {
      float cv[8], rv[8];
      load8(c + k, cv);
      load8(r + k, rv);
      accumulate(cv, rv);
    }
    srr = wave_sum(srr); sdd = wave_sum(sdd);
    if (NEED_Z) { sc = wave_sum(sc); sr = wave_sum(sr); scc = wave_sum(scc); }
    if (NEED_L1) sad = wave_sum(sad);
    float ns = 0.0f;
    if (NEED_SFR) ns = wave_sum((float)nsi);      // at most D / 64 per lane: exact in fp32
    const float rel = sqrtf(sdd) / fmaxf(sqrtf(srr), 1e-30f);
    if (lane == 0 && token_scores) token_scores[(int64_t)claim * T + t] = rel;
    acc[0] += sc; acc[1] += sr; acc[2] += scc; acc[3] += srr;
    acc[4] += (double)sc - (double)sr;            // sum of differences, only used for the mean of d in the z-scored L2
    acc[5] += sad; acc[6] += sdd; acc[7] += ns;
    if (!(rel <= 3.0e38f)) bad = 1;           // NaN or inf
    else if (rel > best) { best = rel; best_t = (int)t; }
  }

  __shared__ double s_acc[4][8];
  __shared__ float s_best[4];
  __shared__ int s_bt[4], s_bad[4];
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) s_acc[wave][j] = acc[j];
    s_best[wave] = best; s_bt[wave] = best_t; s_bad[wave] = bad;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ScorePartial p;
#pragma unroll
    for (int j = 0; j < 8; ++j) p.s[j] = s_acc[0][j] + s_acc[1][j] + s_acc[2][j] + s_acc[3][j];
    float b = -1.0f; int bt = 0, bd = 0;
    for (int w = 0; w < 4; ++w) {
      bd |= s_bad[w];
      if (s_best[w] > b || (s_best[w] == b && s_best[w] >= 0.0f && s_bt[w] < bt)) { b = s_best[w]; bt = s_bt[w]; }
    }
    p.max_rel = b; p.argmax = bt; p.bad = bd; p.pad = 0;
    partials[(int64_t)claim * tiles_per_claim + tile] = p;
  }
}

// ---------------------------------------------------------------------------------------------
// The same statistics for several submissions against ONE shared reference, rows of any multiple of 2 KB.  A wave
// owns a token and takes its row in parts of NU KB (NU = 2 or 4): it loads the reference part into registers once,
// forms the reference's own sums and -- for the sign-flip ratio -- one class mask per element, and then streams the
// same part of every submission of its group past them, the next submission's loads in flight while the current one
// is reduced.  Compared with score_tokens_kernel the reference is read once per group instead of once per submission,
// and its share of the arithmetic is paid once: 7-8 vector instructions per element instead of 16, which moves the
// all-statistics pass from the vector ALUs' bound to the memory's.
//   sign test: sign(a) == sign(b), with sign(0) = sign(NaN) = 0, is one v_cmp_class of a against the set of classes
//   that b's sign allows; the matches are counted on the scalar unit from the lane mask.
// Lane c of a wave adds up submission c's sums over the parts of a token (a predicated add after each wave
// reduction) and closes the token -- per-token relative L2, running sums -- for all submissions at once; the four
// waves' sums are folded per submission at the end, into the same per-(submission, tile) records as above.
// With SUM the kernel also writes, per element, the sum over the group's submissions whose bit in `skip` is clear
// (added in index order, fp32): the mean the EMA update needs, without another pass over the submissions.  SUM needs
// the whole set in one group.
constexpr int kGroupMax = 32;                 // submissions per group (<= 64: one lane each)

__device__ __forceinline__ float dpp_add(float v, int ctrl_sel) {
  const int x = __float_as_int(v);
  int y;
  switch (ctrl_sel) {                                            // immediate operands
    case 0: y = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false); break;     // quad_perm [1,0,3,2]
    case 1: y = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false); break;     // quad_perm [2,3,0,1]
    case 2: y = __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false); break;    // row_half_mirror
    default: y = __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, false); break;   // row_mirror
  }
  return v + __int_as_float(y);
}
// Sum over the 64 lanes without the LDS crossbar: four exchange steps inside each row of 16 lanes, then the four row
// sums are read as scalars.  Every lane gets the same value (a fixed order: run-to-run identical).
__device__ __forceinline__ float wave_sum_rows(float v) {
  v = dpp_add(v, 0); v = dpp_add(v, 1); v = dpp_add(v, 2); v = dpp_add(v, 3);
  const int x = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(x, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(x, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(x, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(x, 48));
  return (r0 + r1) + (r2 + r3);
}

template <typename E, int N> struct RawUnit;                     // N consecutive elements as they come from memory
template <> struct RawUnit<bf16, 8> { bf16x8 v; __device__ __forceinline__ void load(const bf16* p) { v = *reinterpret_cast<const bf16x8*>(p); }
                                      __device__ __forceinline__ float get(int i) const { return static_cast<float>(v[i]); } };
template <> struct RawUnit<bf16, 4> { bf16x4 v; __device__ __forceinline__ void load(const bf16* p) { v = *reinterpret_cast<const bf16x4*>(p); }
                                      __device__ __forceinline__ float get(int i) const { return static_cast<float>(v[i]); } };
template <> struct RawUnit<float, 4> { f32x4 v; __device__ __forceinline__ void load(const float* p) { v = *reinterpret_cast<const f32x4*>(p); }
                                       __device__ __forceinline__ float get(int i) const { return v[i]; } };
template <> struct RawUnit<float, 8> { f32x4 a, b; __device__ __forceinline__ void load(const float* p) { a = *reinterpret_cast<const f32x4*>(p); b = *reinterpret_cast<const f32x4*>(p + 4); }
                                       __device__ __forceinline__ float get(int i) const { return i < 4 ? a[i] : b[i - 4]; } };

template <typename EC, typename ER, int NU, bool FULL, bool SUM>
__global__ __launch_bounds__(256) void score_parts_kernel(const EC* __restrict__ claims, int64_t claim_stride, const ER* __restrict__ ref,
                                                          int64_t T, int D, int n_claims, int G, int n_groups, int tiles_per_claim,
                                                          float* __restrict__ token_scores, ScorePartial* __restrict__ partials,
                                                          uint32_t skip, float* __restrict__ sum_out) {
  constexpr int EPU = 16 / (int)sizeof(EC);            // elements per 16-byte unit of a submission's row
  constexpr int PE = NU * 64 * EPU;                    // elements per part
  const int parts = D / PE;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int group = slot % n_groups;
  const int tile = xcd * ((tiles_per_claim + 7) >> 3) + slot / n_groups;
  if (tile >= tiles_per_claim) return;
  const int c0 = group * G, nc = min(G, n_claims - c0);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;

  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};            // lane c: submission c0 + c
  float best = -1.0f;
  int best_t = 0, bad = 0;

  for (int i = 0; i < kTPW; ++i) {
    const int64_t t = (int64_t)tile * kScoreTokensPerWG + i * 4 + wave;
    if (t >= T) break;                                 // uniform per wave
    const EC* cb = claims + (int64_t)c0 * claim_stride + t * D + lane * EPU;
    RawUnit<EC, EPU> bufA[NU], bufB[NU];
    auto fetch = [&](RawUnit<EC, EPU> (&buf)[NU], int q) {       // q = part * nc + submission
      const int part = q / nc, c = q - part * nc;
      const EC* p = cb + (int64_t)c * claim_stride + part * PE;
#pragma unroll
      for (int m = 0; m < NU; ++m) buf[m].load(p + m * 64 * EPU);
    };
    float sr = 0, srr = 0;                             // the reference's sums: per lane until the token is closed
    float tsdd = 0, tsc = 0, tscc = 0, tsad = 0;       // lane c: submission c's sums over the parts done so far
    int tmatch = 0;
    fetch(bufA, 0);
    const int nq = parts * nc;
    for (int part = 0; part < parts; ++part) {
      const ER* r = ref + t * D + part * PE + lane * EPU;
      float rv[NU][EPU], ssum[NU][EPU];
      int cls[NU][EPU];
#pragma unroll
      for (int m = 0; m < NU; ++m) {
        RawUnit<ER, EPU> u;
        u.load(r + m * 64 * EPU);
#pragma unroll
        for (int j = 0; j < EPU; ++j) {
          const float b = u.get(j);
          rv[m][j] = b;
          srr = fmaf(b, b, srr);
          if (SUM) ssum[m][j] = 0.0f;
          if (FULL) {
            sr += b;
            // classes a may have for sign(a) == sign(b): {+denormal, +normal, +inf}, {-inf, -normal, -denormal}, {NaNs, -0, +0}
            cls[m][j] = b > 0.0f ? 0x380 : (b < 0.0f ? 0x01C : 0x063);
          }
        }
      }
      auto reduce = [&](const RawUnit<EC, EPU> (&buf)[NU], int c) {
        float sc = 0, scc = 0, sad = 0, sdd = 0;
        int match = 0;                                  // wave-uniform
        const bool add = SUM && ((skip >> (c0 + c)) & 1u) == 0;
#pragma unroll
        for (int m = 0; m < NU; ++m)
#pragma unroll
          for (int j = 0; j < EPU; ++j) {
            const float a = buf[m].get(j), d = a - rv[m][j];
            sdd = fmaf(d, d, sdd);
            if (SUM && add) ssum[m][j] += a;
            if (FULL) {
              sc += a; scc = fmaf(a, a, scc); sad += fabsf(d);
              // the compare's lane mask goes straight to the scalar unit (through the generic ballot the compiler
              // turns the predicate into a register value and compares again)
              uint64_t lanes;
              asm("v_cmp_class_f32_e64 %0, %1, %2" : "=s"(lanes) : "v"(a), "v"(cls[m][j]));
              match += __builtin_popcountll(lanes);
              asm volatile("" : "+s"(match));        // count now: otherwise all the masks stay live until the predicated adds
            }
          }
        sdd = wave_sum_rows(sdd);
        if (FULL) { sc = wave_sum_rows(sc); scc = wave_sum_rows(scc); sad = wave_sum_rows(sad); }
        if (lane == c) { tsdd += sdd; tsc += sc; tscc += scc; tsad += sad; tmatch += match; }
      };
      // The next (part, submission) is fetched before the current one is reduced -- unconditionally (past the end:
      // the last one again, never used), because a fetch behind a branch makes the compiler's wait for the current
      // buffer cover the younger loads too, and nothing would be in flight during the reduction.
      const int q0 = part * nc;
      for (int c = 0; c < nc; c += 2) {
        fetch(bufB, min(q0 + c + 1, nq - 1));
        reduce(bufA, c);
        if (c + 1 < nc) {
          fetch(bufA, min(q0 + c + 2, nq - 1));
          reduce(bufB, c + 1);
        } else {                                       // odd group: the next part's first submission sits in B
#pragma unroll
          for (int m = 0; m < NU; ++m) bufA[m] = bufB[m];
        }
      }
      if (SUM) {
        float* so = sum_out + t * D + part * PE + lane * EPU;
#pragma unroll
        for (int m = 0; m < NU; ++m) {
          if (EPU == 8) {
            f32x4 lo, hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) { lo[j] = ssum[m][j]; hi[j] = ssum[m][(EPU == 8) ? 4 + j : j]; }
            *reinterpret_cast<f32x4*>(so + m * 64 * EPU) = lo;
            *reinterpret_cast<f32x4*>(so + m * 64 * EPU + 4) = hi;
          } else {
            f32x4 lo;
#pragma unroll
            for (int j = 0; j < 4; ++j) lo[j] = ssum[m][j];
            *reinterpret_cast<f32x4*>(so + m * 64 * EPU) = lo;
          }
        }
      }
    }
    // close the token: every lane for its own submission
    srr = wave_sum_rows(srr);
    if (FULL) sr = wave_sum_rows(sr);
    const float rel = sqrtf(tsdd) / fmaxf(sqrtf(srr), 1e-30f);
    if (lane < nc) {
      if (token_scores) token_scores[(int64_t)(c0 + lane) * T + t] = rel;
      acc[0] += tsc; acc[1] += sr; acc[2] += tscc; acc[3] += srr;
      acc[4] += (double)tsc - (double)sr;
      acc[5] += tsad; acc[6] += tsdd;
      if (FULL) acc[7] += (double)(D - tmatch);
      if (!(rel <= 3.0e38f)) bad = 1;
      else if (rel > best) { best = rel; best_t = (int)t; }
    }
  }

  __shared__ double s_acc[4][kGroupMax][8];
  __shared__ float s_best[4][kGroupMax];
  __shared__ int s_bt[4][kGroupMax], s_bad[4][kGroupMax];
  if (lane < nc) {
#pragma unroll
    for (int j = 0; j < 8; ++j) s_acc[wave][lane][j] = acc[j];
    s_best[wave][lane] = best; s_bt[wave][lane] = best_t; s_bad[wave][lane] = bad;
  }
  __syncthreads();
  if ((int)threadIdx.x < nc) {
    const int c = threadIdx.x;
    ScorePartial p;
#pragma unroll
    for (int j = 0; j < 8; ++j) p.s[j] = s_acc[0][c][j] + s_acc[1][c][j] + s_acc[2][c][j] + s_acc[3][c][j];
    float b = -1.0f; int bt = 0, bd = 0;
    for (int w = 0; w < 4; ++w) {
      bd |= s_bad[w][c];
      if (s_best[w][c] > b || (s_best[w][c] == b && s_best[w][c] >= 0.0f && s_bt[w][c] < bt)) { b = s_best[w][c]; bt = s_bt[w][c]; }
    }
    p.max_rel = b; p.argmax = bt; p.bad = bd; p.pad = 0;
    partials[(int64_t)(c0 + c) * tiles_per_claim + tile] = p;
  }
}

// m <- beta m + (1 - beta) / n * sum: the EMA update from the sum a score_parts_kernel launch has written
__global__ __launch_bounds__(256) void ema_from_sum_kernel(float* __restrict__ m, const float* __restrict__ sum, int64_t n_vec, float beta, float w) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n_vec) return;
  float mv[8], sv8[8];
  load8(m + v * 8, mv);
  load8(sum + v * 8, sv8);
#pragma unroll
  for (int j = 0; j < 8; ++j) mv[j] = beta * mv[j] + w * sv8[j];
  store8(m + v * 8, mv);
}

struct Tau4 { float v[4]; };

__global__ __launch_bounds__(256) void score_finalize_kernel(const ScorePartial* __restrict__ partials, int tiles_per_claim,
                                                             int64_t T, int D, uint32_t mask, Tau4 tau, int reduce,
                                                             sv_result* __restrict__ results) {
  const int claim = blockIdx.x, tid = threadIdx.x;
  const ScorePartial* p = partials + (int64_t)claim * tiles_per_claim;
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  float best = -1.0f; int bt = 0, bad = 0;
  for (int i = tid; i < tiles_per_claim; i += 256) {     // tiles visited in increasing order
    const ScorePartial q = p[i];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += q.s[j];
    bad |= q.bad;
    if (q.max_rel > best) { best = q.max_rel; bt = q.argmax; }
  }
  __shared__ double s_acc[256][8];
  __shared__ float s_best[256];
  __shared__ int s_bt[256], s_bad[256];
#pragma unroll
  for (int j = 0; j < 8; ++j) s_acc[tid][j] = acc[j];
  s_best[tid] = best; s_bt[tid] = bt; s_bad[tid] = bad;
  __syncthreads();
  for (int stride = 128; stride > 0; stride >>= 1) {     // fixed tree: run-to-run identical
    if (tid < stride) {
#pragma unroll
      for (int j = 0; j < 8; ++j) s_acc[tid][j] += s_acc[tid + stride][j];
      s_bad[tid] |= s_bad[tid + stride];
      const float o = s_best[tid + stride];
      if (o > s_best[tid] || (o == s_best[tid] && s_bt[tid + stride] < s_bt[tid])) { s_best[tid] = o; s_bt[tid] = s_bt[tid + stride]; }
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double n = (double)T * (double)D;
    const double Sc = s_acc[0][0], Sr = s_acc[0][1], Scc = s_acc[0][2], Srr = s_acc[0][3];
    const double Sd = s_acc[0][4], Sad = s_acc[0][5], Sdd = s_acc[0][6], Ns = s_acc[0][7];
    const double nan = __longlong_as_double(0x7ff8000000000000LL);
    double sc[4];
    const double grel = sqrt(Sdd) / fmax(sqrt(Srr), 1e-30);
    const double mrel = s_bad[0] ? nan : (double)fmaxf(s_best[0], 0.0f);
    sc[SV_IDX_RELL2] = (reduce == SV_REDUCE_MAX_TOKEN) ? mrel : grel;
    sc[SV_IDX_L1] = Sad / n;
    // z-scored L2 = 2 (1 - rho) = (var_d - (sd_c - sd_r)^2) / (sd_c sd_r): no cancellation for rho ~ 1
    const double mc = Sc / n, mr = Sr / n, md = Sd / n;
    const double vc = Scc / n - mc * mc, vr = Srr / n - mr * mr, vd = fmax(Sdd / n - md * md, 0.0);
    const bool const_c = !(vc > 1e-10 * (Scc / n)), const_r = !(vr > 1e-10 * (Srr / n));
    if (Scc != Scc || Srr != Srr) sc[SV_IDX_ZL2] = nan;
    else if (const_c && const_r) sc[SV_IDX_ZL2] = 0.0;
    else if (const_c || const_r) sc[SV_IDX_ZL2] = 2.0;
    else {
      const double a = sqrt(vc), b = sqrt(vr);
      sc[SV_IDX_ZL2] = fmax(vd - (a - b) * (a - b), 0.0) / (a * b);
    }
    sc[SV_IDX_SFR] = Ns / n;
    sv_result r;
    uint32_t flag = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool on = ((mask >> i) & 1u) || i == SV_IDX_RELL2;         // the relative L2 is always formed
      r.score[i] = on ? (float)sc[i] : 0.0f;
      if (((mask >> i) & 1u) && !(r.score[i] <= tau.v[i])) flag = 1;   // strict '>'; non-finite scores are flagged
    }
    r.flag = flag; r.metric_mask = mask;
    r.max_token_rell2 = (float)mrel; r.argmax_token = s_bt[0];
    results[claim] = r;
  }
}

template <typename E>
__global__ __launch_bounds__(256) void ema_update_kernel(float* __restrict__ m, const E* __restrict__ claims, int64_t claim_stride,
                                                         int n_claims, const uint8_t* __restrict__ flags, int64_t n_vec, float beta) {
  // the un-flagged submissions of this step, compacted once per workgroup
  __shared__ int clean[1024];
  __shared__ int s_n;
  if (threadIdx.x == 0) {
    int n = 0;
    for (int i = 0; i < n_claims && n < 1024; ++i)
      if (flags == nullptr || flags[i] == 0) clean[n++] = i;
    s_n = n;
  }
  __syncthreads();
  const int n_clean = s_n;
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n_vec || n_clean == 0) return;   // every submission flagged: the EMA is left as it is
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const E* base = claims + v * 8;
  int i = 0;
  for (; i + 3 < n_clean; i += 4) {
    float x0[8], x1[8], x2[8], x3[8];
    load8(base + (int64_t)clean[i] * claim_stride, x0);
    load8(base + (int64_t)clean[i + 1] * claim_stride, x1);
    load8(base + (int64_t)clean[i + 2] * claim_stride, x2);
    load8(base + (int64_t)clean[i + 3] * claim_stride, x3);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += (x0[j] + x1[j]) + (x2[j] + x3[j]);
  }
  for (; i < n_clean; ++i) {
    float x[8];
    load8(base + (int64_t)clean[i] * claim_stride, x);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += x[j];
  }
  float mv[8];
  load8(m + v * 8, mv);
  const float w = (1.0f - beta) / (float)n_clean;
#pragma unroll
  for (int j = 0; j < 8; ++j) mv[j] = beta * mv[j] + w * acc[j];
  store8(m + v * 8, mv);
}

}  // namespace

bool score_sum_supported(int n_claims, int64_t ref_stride, int claim_dtype, int D) {
  const int64_t row_bytes = (int64_t)D * (claim_dtype == SV_BF16 ? 2 : 4);
  return n_claims >= 1 && n_claims <= kGroupMax && ref_stride == 0 && row_bytes % 2048 == 0;
}

hipError_t launch_ema_from_sum(float* m, const float* sum, int n_summed, int64_t T, int D, float beta, hipStream_t st) {
  if (n_summed <= 0 || T <= 0) return hipSuccess;    // nobody entered the sum: the EMA is left as it is
  const int64_t n_vec = T * D / 8;
  hipLaunchKernelGGL(ema_from_sum_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, st, m, sum, n_vec, beta,
                     (1.0f - beta) / (float)n_summed);
  return hipGetLastError();
}

hipError_t launch_score(const void* claims, int64_t claim_stride, int n_claims, const void* ref, int64_t ref_stride,
                        int claim_dtype, int ref_dtype, int64_t T, int D, uint32_t mask, const float* tau4, int reduce,
                        float* token_scores, sv_result* results, ScorePartial* scratch, int64_t scratch_elems,
                        hipStream_t st, uint32_t skip, float* sum_out) {
  if (n_claims <= 0 || T <= 0) return hipSuccess;
  if (sum_out && !score_sum_supported(n_claims, ref_stride, claim_dtype, D)) return hipErrorInvalidValue;
  const int64_t tiles = (T + kScoreTokensPerWG - 1) / kScoreTokensPerWG;
  int64_t per_launch = scratch_elems / tiles;
  if (per_launch < 1) return hipErrorInvalidValue;
  if (per_launch * (tiles + 7) > 0x7fffffffLL) per_launch = 0x7fffffffLL / (tiles + 7);
  Tau4 tau;
  for (int i = 0; i < 4; ++i) tau.v[i] = tau4 ? tau4[i] : 0.0f;
  const int64_t csz = claim_dtype == SV_BF16 ? 2 : 4, rsz = ref_dtype == SV_BF16 ? 2 : 4;
  for (int64_t c0 = 0; c0 < n_claims; c0 += per_launch) {
    const int nc = (int)((n_claims - c0 < per_launch) ? (n_claims - c0) : per_launch);
    const char* cp = (const char*)claims + c0 * claim_stride * csz;
    const char* rp = (const char*)ref + c0 * ref_stride * rsz;
    float* ts = token_scores ? token_scores + c0 * T : nullptr;
    const dim3 grid((unsigned)(8 * ((tiles + 7) / 8) * nc)), block(256);
    const int64_t row_bytes = (int64_t)D * csz;
    const bool full = (mask & (SV_M_L1 | SV_M_ZL2 | SV_M_SFR)) != 0;
    // shared reference and several submissions (or their sum wanted), rows of a multiple of 2 KB: the kernel that
    // keeps the reference in registers
    if (ref_stride == 0 && row_bytes % 2048 == 0 && (sum_out || nc >= 2)) {
      if (sum_out && (nc != n_claims || nc * tiles > scratch_elems)) return hipErrorInvalidValue;   // one launch, one group
      int G = sum_out ? nc : 16;
      while (!sum_out && G > 4 && tiles * ((nc + G - 1) / G) < 1024) G >>= 1;
      const int n_groups = (nc + G - 1) / G;
      const dim3 ggrid((unsigned)(8 * ((tiles + 7) / 8) * n_groups));
#define SV_LAUNCH_PARTS5(EC, ER, NU, FULL, SUM)                                                                       \
  hipLaunchKernelGGL((score_parts_kernel<EC, ER, NU, FULL, SUM>), ggrid, block, 0, st, (const EC*)cp, claim_stride, (const ER*)rp, T, D, nc, \
                     G, n_groups, (int)tiles, ts, scratch, skip, sum_out)
#define SV_LAUNCH_PARTS3(EC, ER, NU)                                                                                  \
  do {                                                                                                                \
    if (sum_out) { if (full) SV_LAUNCH_PARTS5(EC, ER, NU, true, true); else SV_LAUNCH_PARTS5(EC, ER, NU, false, true); } \
    else { if (full) SV_LAUNCH_PARTS5(EC, ER, NU, true, false); else SV_LAUNCH_PARTS5(EC, ER, NU, false, false); }     \
  } while (0)
#define SV_LAUNCH_PARTS(EC, ER)                                                                                       \
  do { if (row_bytes % 4096 == 0) SV_LAUNCH_PARTS3(EC, ER, 4); else SV_LAUNCH_PARTS3(EC, ER, 2); } while (0)
      if (claim_dtype == SV_BF16 && ref_dtype == SV_BF16) SV_LAUNCH_PARTS(bf16, bf16);
      else if (claim_dtype == SV_BF16) SV_LAUNCH_PARTS(bf16, float);
      else if (ref_dtype == SV_BF16) SV_LAUNCH_PARTS(float, bf16);
      else SV_LAUNCH_PARTS(float, float);
#undef SV_LAUNCH_PARTS
#undef SV_LAUNCH_PARTS3
#undef SV_LAUNCH_PARTS5
      hipLaunchKernelGGL(score_finalize_kernel, dim3(nc), dim3(256), 0, st, scratch, (int)tiles, T, D, mask, tau, reduce,
                         results + c0);
      continue;
    }
#define SV_LAUNCH_SCORE3(EC, ER, L1, Z, SFR)                                                                           \
  hipLaunchKernelGGL((score_tokens_kernel<EC, ER, L1, Z, SFR>), grid, block, 0, st, (const EC*)cp, claim_stride,          \
                     (const ER*)rp, ref_stride, T, D, nc, (int)tiles, ts, scratch)
#define SV_LAUNCH_SCORE(EC, ER)                                                                                          \
  do {                                                                                                                   \
    const bool l1 = mask & SV_M_L1, z = mask & SV_M_ZL2, sfr = mask & SV_M_SFR;                                          \
    if (!l1 && !z && !sfr) SV_LAUNCH_SCORE3(EC, ER, false, false, false);                                                \
    else if (l1 && !z && !sfr) SV_LAUNCH_SCORE3(EC, ER, true, false, false);                                             \
    else if (!l1 && !z && sfr) SV_LAUNCH_SCORE3(EC, ER, false, false, true);                                             \
    else if (!l1 && z && !sfr) SV_LAUNCH_SCORE3(EC, ER, false, true, false);                                             \
    else SV_LAUNCH_SCORE3(EC, ER, true, true, true);                                                                     \
  } while (0)
    if (claim_dtype == SV_BF16 && ref_dtype == SV_BF16) SV_LAUNCH_SCORE(bf16, bf16);
    else if (claim_dtype == SV_BF16) SV_LAUNCH_SCORE(bf16, float);
    else if (ref_dtype == SV_BF16) SV_LAUNCH_SCORE(float, bf16);
    else SV_LAUNCH_SCORE(float, float);
#undef SV_LAUNCH_SCORE
#undef SV_LAUNCH_SCORE3
    hipLaunchKernelGGL(score_finalize_kernel, dim3(nc), dim3(256), 0, st, scratch, (int)tiles, T, D, mask, tau, reduce,
                       results + c0);
  }
  return hipGetLastError();
}

// Alg. gradient_replacement: every signal whose mask byte is set is overwritten with the reference point m
// (rounded to the signal's dtype); the others are left alone.  The workgroups of a signal stride over its 8-element vectors.
template <typename E>
__global__ __launch_bounds__(256) void replace_kernel(E* __restrict__ signals, int64_t stride, const uint8_t* __restrict__ mask,
                                                      const float* __restrict__ m, int64_t n_vec) {
  if (mask[blockIdx.y] == 0) return;
  for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n_vec; v += (int64_t)gridDim.x * 256) {
    float x[8];
    load8(m + v * 8, x);
    store8(signals + (int64_t)blockIdx.y * stride + v * 8, x);
  }
}

hipError_t launch_replace(void* signals, int64_t stride, int n, int dtype, const uint8_t* mask, const float* m, int64_t T, int D,
                          hipStream_t st) {
  if (n <= 0 || T <= 0) return hipSuccess;
  const int64_t n_vec = T * D / 8;
  // few workgroups per signal: most signals are left alone, and a workgroup that only reads its mask byte should be cheap
  const dim3 grid((unsigned)min((n_vec + 255) / 256, (int64_t)1024), (unsigned)n), block(256);
  if (dtype == SV_BF16) hipLaunchKernelGGL(replace_kernel<bf16>, grid, block, 0, st, (bf16*)signals, stride, mask, m, n_vec);
  else hipLaunchKernelGGL(replace_kernel<float>, grid, block, 0, st, (float*)signals, stride, mask, m, n_vec);
  return hipGetLastError();
}

hipError_t launch_ema(float* m, const void* claims, int64_t claim_stride, int n_claims, int claim_dtype,
                      const uint8_t* flags, int64_t T, int D, float beta, hipStream_t st) {
  if (n_claims <= 0 || T <= 0) return hipSuccess;
  const int64_t n_vec = T * D / 8;
  const dim3 grid((unsigned)((n_vec + 255) / 256)), block(256);
  if (claim_dtype == SV_BF16)
    hipLaunchKernelGGL(ema_update_kernel<bf16>, grid, block, 0, st, m, (const bf16*)claims, claim_stride, n_claims, flags, n_vec, beta);
  else
    hipLaunchKernelGGL(ema_update_kernel<float>, grid, block, 0, st, m, (const float*)claims, claim_stride, n_claims, flags, n_vec, beta);
  return hipGetLastError();
}

}  // namespace sv

// ---------------------------------------------------------------------------------------------------------------
// The statistic for callers that cannot allocate.  sv_score_and_flag keeps its per-(submission, token tile) partial
// records in the context's workspace, which sv_create allocates; here the same records live in a file-scope device
// array that exists once per GPU from the moment the library's code object is loaded on it until the process ends.
namespace {

constexpr int64_t kStaticScoreRecords = 1 << 16;          // 5 MiB: e.g. 128 submissions of 8192 tokens
static __device__ __align__(256) unsigned char scratch[kStaticScoreRecords * sizeof(sv::ScorePartial)];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
sv::ScorePartial* g_static_ptr[kMaxDevices] = {};          // device address of `scratch` on each GPU, asked for once

// The array's name is a host-side handle, not a device address: the address on the CURRENT device comes from the
// runtime, once per device, and only that pointer is ever handed to a kernel.
hipError_t static_score_scratch(sv::ScorePartial** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = (sv::ScorePartial*)p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" sv_status sv_score_and_flag_noalloc(const void* claims, int64_t claim_stride, int32_t n_claims, const void* ref,
                                               int64_t ref_stride, int32_t claim_dtype, int32_t ref_dtype, int64_t T, int32_t D,
                                               uint32_t metric_mask, const float* tau, int32_t reduce, float* token_scores_out,
                                               sv_result* results_dev, void* stream) {
  using sv::set_global_error;
  if (n_claims < 0 || T < 0 || D < 1) { set_global_error("negative size"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!claims || !ref || !results_dev || !tau) { set_global_error("claims, ref, tau and results_dev must be non-NULL"); return SV_EINVAL; }
  if ((claim_dtype != SV_F32 && claim_dtype != SV_BF16) || (ref_dtype != SV_F32 && ref_dtype != SV_BF16)) {
    set_global_error("unknown dtype");
    return SV_EINVAL;
  }
  if (reduce != SV_REDUCE_GLOBAL && reduce != SV_REDUCE_MAX_TOKEN) { set_global_error("unknown reduce"); return SV_EINVAL; }
  if (D % 8) { set_global_error("D must be a multiple of 8"); return SV_EUNSUPPORTED; }
  if (T > 0x7fffffffLL || claim_stride < 0 || ref_stride < 0) { set_global_error("T or a stride is out of range"); return SV_EINVAL; }
  const int64_t tiles = (T + sv::kScoreTokensPerWG - 1) / sv::kScoreTokensPerWG;
  if (tiles * (int64_t)n_claims > kStaticScoreRecords) {
    set_global_error("n_claims * ceil(T / %d) = %lld exceeds the %lld partial records of the static scratch: split the call or use "
                     "sv_score_and_flag with a context", sv::kScoreTokensPerWG, (long long)(tiles * n_claims), (long long)kStaticScoreRecords);
    return SV_EUNSUPPORTED;
  }
  sv::ScorePartial* records = nullptr;
  hipError_t e = static_score_scratch(&records);
  if (e != hipSuccess) { set_global_error("hipGetSymbolAddress of the static scratch failed: %s", hipGetErrorString(e)); return SV_EHIP; }
  // every record the finalize step reads is written by the pass before it in this same call, so nothing has to be
  // cleared between calls; the records of an earlier, larger call beyond this call's range are simply not read
  e = sv::launch_score(claims, claim_stride, n_claims, ref, ref_stride, claim_dtype, ref_dtype, T, D, metric_mask, tau, reduce,
                       token_scores_out, results_dev, records, kStaticScoreRecords, (hipStream_t)stream);
  if (e != hipSuccess) { set_global_error("launching the score pass failed: %s", hipGetErrorString(e)); return SV_EHIP; }
  return SV_OK;
}
