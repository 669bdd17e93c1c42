// Sliced Wasserstein statistic Omega_SW (paragraph "Choice of Distance Measure"): the mean over L
// directions u of the 1-Wasserstein distance between the two signals projected on u.  The samples
// of a signal are its T token vectors; with equal sample counts W1 on the line is the mean absolute
// difference of the sorted projections.
//
// Three steps, all on the caller's stream:
//   project : P[l][t] = <x_t, u_l>          MFMA, HBM-bound (one read of the signal)
//   sort    : every row P[l][.] ascending   bitonic network in LDS (+ global steps for long rows)
//   W1      : sum_t |P_claim[l][t] - P_ref[l][t]| fused into the claim's last sort stage, fixed
//             summation order; a finalize kernel averages over l and applies the threshold.
#include "common.h"

namespace sv {
namespace {

constexpr int kSortChunkMax = (int)kSwSortChunkMax;   // floats sorted in LDS by one workgroup (64 KB)

// ---------------------------------------------------------------------------------------------
// Projection.  A workgroup of 4 waves owns 256 tokens (64 per wave, two blocks of 32) and all
// L = 32 * LB directions; the contraction runs over the feature axis in steps of 16 on
// v_mfma_f32_32x32x16_bf16 with the directions in the A slot, so a lane ends up with one token
// (lane & 31) and the directions 8q + 4 (lane >> 5) + r of each block of 32.
// The signal is streamed in chunks of 128 bytes per row (64 bf16 or 32 fp32 features): the
// [256 rows x 128 B] tile goes global -> LDS with global_load_lds (8 lanes fetch one row's 128
// contiguous bytes; the 16-byte pieces are XOR-swizzled by choosing which piece a lane fetches),
// three tiles deep, so that two chunks are always in flight and the wait at the end of a chunk
// leaves the youngest one outstanding.  The matching [L x chunk] piece of the directions takes the same
// road.  Fragments are 16-byte LDS reads, conflict-free with the swizzle.
// fp32 signals are split into three bf16 terms (x = hi + mid + lo exactly), three MFMAs per step:
// every product is exact in fp32, so the result has fp32-accumulation accuracy.
__device__ __forceinline__ int sw_swz(int row) { return (row ^ (row >> 3)) & 7; }

template <int LB>
__device__ __forceinline__ void mac_bf16(const bf16x8 (&u)[LB], const bf16x8& x, f32x16 (&acc)[LB]) {
#pragma unroll
  for (int b = 0; b < LB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u[b], x, acc[b], 0, 0, 0);
}

template <int LB>
__device__ __forceinline__ void mac_f32(const bf16x8 (&u)[LB], const f32x4& x0, const f32x4& x1, f32x16 (&acc)[LB]) {
  bf16x8 hi, mid, lo;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float x = i < 4 ? x0[i] : x1[i - 4];
    const bf16 a = (bf16)x;
    const float r1 = x - (float)a;
    const bf16 b = (bf16)r1;
    const float r2 = r1 - (float)b;
    hi[i] = a; mid[i] = b; lo[i] = (bf16)r2;
  }
  mac_bf16<LB>(u, lo, acc);
  mac_bf16<LB>(u, mid, acc);
  mac_bf16<LB>(u, hi, acc);
}

constexpr int kSwTile = 256 * 128;     // bytes of one signal tile in LDS
constexpr int kSwDepth = 3;            // signal tiles (and direction chunks) in LDS: two chunks in flight

template <int N> __device__ __forceinline__ void wait_vm_lds_barrier() {      // wait until at most N vector-memory loads are in flight
  static_assert(N >= 9 && N <= 12, "8 signal loads + 1..4 direction loads per chunk");
  if (N == 9) asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else if (N == 10) asm volatile("s_waitcnt vmcnt(10) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else if (N == 11) asm volatile("s_waitcnt vmcnt(11) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <typename E, int LB>
__device__ __forceinline__ void sw_project_body(const char* __restrict__ xbase, const bf16* __restrict__ U, int D, int64_t T, int64_t Tpad,
                                                float* __restrict__ out, char* smem, unsigned sig) {
  constexpr bool kBf16 = sizeof(E) == 2;
  constexpr int KC = 128 / (int)sizeof(E);            // features per chunk
  constexpr int NSTEP = KC / 16;                      // MFMA k steps per chunk
  constexpr int UPITCH = KC * 2;                      // bytes of a direction row per chunk: 128 (bf16 signal) or 64 (fp32 signal)
  constexpr int UTILE = LB * 32 * UPITCH;
  constexpr int UINSTR = UTILE / 1024;                // direct-to-LDS instructions per directions' chunk
  constexpr int UW = (UINSTR + 3) / 4;                // ... per wave (every wave issues the same number: the waits count them)
  constexpr int RPI = 1024 / UPITCH;                  // direction rows per instruction: 8 or 16
  char* xs = smem;                                    // kSwDepth signal tiles
  char* us = smem + kSwDepth * kSwTile;               // kSwDepth direction chunks
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l31 = lane & 31, lhi = lane >> 5;
  const int64_t tile0 = (int64_t)blockIdx.x * 256;
  // direct-to-LDS plan: instruction i of this wave covers the tile rows (wave + 4 i) * 8 .. + 7
  int64_t xoff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (wave + 4 * i) * 8 + (lane >> 3), c = (lane & 7) ^ sw_swz(r);
    xoff[i] = min(tile0 + r, T - 1) * (int64_t)D * (int64_t)sizeof(E) + c * 16;     // rows past the end re-read the last one
  }
  // The directions' chunk [L rows x UPITCH bytes] goes the same way (no registers, so the only vector-memory
  // operations in flight are direct-to-LDS loads and the waits can count them exactly; staged through registers, the
  // compiler's wait before the LDS write also waited for the youngest signal chunk).  Instruction j of this wave covers
  // the rows RPI * i .. + RPI - 1, i = min(wave + 4 j, UINSTR - 1) (a repeated instruction rewrites the same bytes).
  // 16-byte pieces are XOR-swizzled by the row so that the 32 rows a fragment read touches spread over the banks.
  auto u_swz = [](int r) { return kBf16 ? sw_swz(r) : ((r >> 2) & 3); };
  int64_t uoff[UW];
  int ulds[UW];
#pragma unroll
  for (int j = 0; j < UW; ++j) {
    const int i = min(wave + 4 * j, UINSTR - 1);
    const int r = i * RPI + lane / (UPITCH / 16), c = (lane % (UPITCH / 16)) ^ u_swz(r);
    uoff[j] = (int64_t)r * D * 2 + c * 16;
    ulds[j] = i * 1024;
  }
  // Workgroups that run together start at different chunks: with a row pitch that is a multiple of the memory
  // channels' interleave, everybody reading column chunk kc of its rows at the same time would camp on few channels.
  const int nchunk = D / KC;
  const int rot = (int)((blockIdx.x * 5u + sig * 3u) % (unsigned)nchunk);      // sig: index of the signal in its tensor
  auto chunk_of = [&](int kc) { const int c = kc + rot; return c >= nchunk ? c - nchunk : c; };
  auto dma = [&](int kc, int stage) {
    const int ck = chunk_of(kc);
#pragma unroll
    for (int j = 0; j < UW; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)((const char*)U + uoff[j] + (int64_t)ck * UPITCH),
                                       (__attribute__((address_space(3))) void*)(us + stage * UTILE + ulds[j]), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xbase + xoff[i] + (int64_t)ck * 128),
                                       (__attribute__((address_space(3))) void*)(xs + stage * kSwTile + (wave + 4 * i) * 1024), 16, 0, 0);
  };
  f32x16 acc[2][LB];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int b = 0; b < LB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tb][b][i] = 0.0f;

  dma(0, 0);
  dma(nchunk > 1 ? 1 : 0, 1);                          // a second chunk is always issued: the waits below count on it
  wait_vm_lds_barrier<8 + UW>();
  int st = 0;                                          // LDS tile of chunk kc
  for (int kc = 0; kc < nchunk; ++kc) {
    const int st2 = st == 0 ? kSwDepth - 1 : st - 1;   // tile of chunk kc + 2: the one chunk kc - 1 was read from
    dma(kc + 2 < nchunk ? kc + 2 : nchunk - 1, st2);   // past the end: re-read the last chunk (never used)
    const char* xt = xs + st * kSwTile;
    const char* ub = us + st * UTILE;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
      bf16x8 u[LB];
#pragma unroll
      for (int b = 0; b < LB; ++b) {
        const int r = b * 32 + l31;
        u[b] = *reinterpret_cast<const bf16x8*>(ub + r * UPITCH + (((2 * s + lhi) ^ u_swz(r)) << 4));
      }
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        const int r = wave * 64 + tb * 32 + l31;
        if (kBf16) {
          const bf16x8 x = *reinterpret_cast<const bf16x8*>(xt + r * 128 + (((2 * s + lhi) ^ sw_swz(r)) << 4));
          mac_bf16<LB>(u, x, acc[tb]);
        } else {
          const int c = 2 * (2 * s + lhi);
          const f32x4 x0 = *reinterpret_cast<const f32x4*>(xt + r * 128 + ((c ^ sw_swz(r)) << 4));
          const f32x4 x1 = *reinterpret_cast<const f32x4*>(xt + r * 128 + (((c + 1) ^ sw_swz(r)) << 4));
          mac_f32<LB>(u, x0, x1, acc[tb]);
        }
      }
    }
    // chunk kc + 1 has landed (only the loads of chunk kc + 2 may still be in flight) and this wave is done with
    // tile st; after the barrier that holds for the whole workgroup
    wait_vm_lds_barrier<8 + UW>();
    st = st + 1 >= kSwDepth ? 0 : st + 1;
  }
  __builtin_amdgcn_s_waitcnt(0);                       // every direct-to-LDS load has landed before the LDS is given back
  const float inf = __builtin_huge_valf();             // padding sorts behind every real sample
  const int64_t t0 = tile0 + wave * 64;
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t t = t0 + tb * 32 + l31;
    if (t >= Tpad) continue;
#pragma unroll
    for (int b = 0; b < LB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        out[(int64_t)(b * 32 + (i >> 2) * 8 + lhi * 4 + (i & 3)) * Tpad + t] = t < T ? acc[tb][b][i] : inf;
  }
}

// The launch covers n2 (0 or 1) signals of type E2 at X2 -- projected into P2 -- in the grid rows 0 .. n2 - 1, and behind
// them the signals X + i * x_stride of type E, projected into the slots P + i * L * Tpad.  A single reference tensor has
// too few token tiles to fill the chip; in one launch with the submissions it runs beside them.
template <typename E, typename E2, int LB>
__global__ __launch_bounds__(256) void sw_project_kernel(const E* __restrict__ X, int64_t x_stride, const E2* __restrict__ X2, int n2,
                                                         const bf16* __restrict__ U, int D, int64_t T, int64_t Tpad,
                                                         float* __restrict__ P, float* __restrict__ P2) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int y = blockIdx.y;                           // uniform
  if constexpr (sizeof(E) == sizeof(E2)) {
    const char* xb = y < n2 ? (const char*)X2 : (const char*)(X + (int64_t)(y - n2) * x_stride);
    float* out = y < n2 ? P2 : P + (int64_t)(y - n2) * (LB * 32) * Tpad;
    sw_project_body<E, LB>(xb, U, D, T, Tpad, out, smem, y < n2 ? y : y - n2);
  } else {
    if (y < n2) sw_project_body<E2, LB>((const char*)X2, U, D, T, Tpad, P2, smem, y);
    else sw_project_body<E, LB>((const char*)(X + (int64_t)(y - n2) * x_stride), U, D, T, Tpad, P + (int64_t)(y - n2) * (LB * 32) * Tpad, smem, y - n2);
  }
}

// ---------------------------------------------------------------------------------------------
// Bitonic sorting network on rows of length Tpad (a power of two).  Element i of a row is compared
// with i ^ j in the stage (k, j), ascending where (i & k) == 0.
//
// sw_sort_chunk_kernel keeps a chunk of `ch` consecutive elements in LDS and runs the stages
// (k, j) for k = k_first, 2 k_first, ..., k_last and j = min(k / 2, ch / 2) ... 1 on it.  With
// k_first = 2 and k_last = ch it sorts the chunk from scratch; with k_first = k_last = k > ch it
// finishes stage k after sw_sort_global_kernel has done the strides j >= ch.
// If `ref` is non-null (only for ch == Tpad) the sorted row is not written back; instead the
// workgroup adds up |row[i] - ref_row[i]| over the T real samples in a fixed order and stores the
// sum in w1[first_seg + segment]; the reference row is row (segment % L) of `ref` when ref_shared,
// else row `segment`.
//
// The network is LDS-bound when every stage is a round trip, so a thread takes eight float4 vectors
// v0 + m s (m = 0..7) into registers and runs up to three stages (vector strides 4s, 2s, s) on them
// per round trip; the last pass of a level (s = 1: 32 consecutive elements) also runs the strides
// 2 and 1 inside the vectors, and the first pass of a sort from scratch runs all of the levels
// k = 2 .. 32 (15 stages).  13 levels of an 8192-element row take 24 round trips instead of 91.
// The comparator and the order of the stages are those of the plain network, so the result is the same for
// every input.  Vectors are XOR-swizzled in LDS (bits 4, 5, 6 of the vector index folded into bits
// 1, 2 and 0 + 3) so that 16 neighbouring lanes hit 16 different 16-byte slots at every stride.
template <int A, int B>
__device__ __forceinline__ void cx_in(f32x4& v, bool asc) {          // components A and B of one vector
  const float a = v[A], b = v[B];
  const bool swap = (a > b) == asc;
  v[A] = swap ? b : a; v[B] = swap ? a : b;
}
__device__ __forceinline__ void cxv(f32x4& a, f32x4& b, bool asc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool swap = (a[i] > b[i]) == asc;
    const float na = swap ? b[i] : a[i], nb = swap ? a[i] : b[i];
    a[i] = na; b[i] = nb;
  }
}
// vectors m and m + SM of the eight, direction of vector m
template <int SM>
__device__ __forceinline__ void vec_stage(f32x4 (&e)[8], const bool (&asc)[8]) {
#pragma unroll
  for (int m = 0; m < 8; ++m)
    if ((m & SM) == 0) cxv(e[m], e[m + SM], asc[m]);
}
// strides 2 and 1 inside every vector
__device__ __forceinline__ void in_stages(f32x4 (&e)[8], const bool (&asc)[8], bool with_stride2) {
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    if (with_stride2) { cx_in<0, 2>(e[m], asc[m]); cx_in<1, 3>(e[m], asc[m]); }
    cx_in<0, 1>(e[m], asc[m]); cx_in<2, 3>(e[m], asc[m]);
  }
}

__global__ __launch_bounds__(512) void sw_sort_chunk_kernel(float* __restrict__ P, int64_t Tpad, int ch, int64_t k_first, int64_t k_last,
                                                            const float* __restrict__ ref, int ref_shared, int L, int64_t T,
                                                            float* __restrict__ w1, int first_seg) {
  extern __shared__ __attribute__((aligned(16))) float s[];
  f32x4* s4 = reinterpret_cast<f32x4*>(s);
  const int tid = threadIdx.x, nt = blockDim.x;
  const int64_t gbase = (int64_t)blockIdx.x * ch;
  float* row = P + (int64_t)blockIdx.y * Tpad + gbase;
  const int nvec = ch >> 2, ngroups = ch >> 5;
  const bool swz = nvec >= 128;                       // the swizzle permutes inside blocks of 128 vectors
  auto phys = [&](int v) { return swz ? v ^ ((((v >> 4) & 3) << 1) | (((v >> 6) & 1) * 9)) : v; };
  for (int v = tid; v < nvec; v += nt) s4[phys(v)] = *reinterpret_cast<const f32x4*>(row + 4 * v);
  __syncthreads();

  // one round trip: the stages `mask` (4: stride 4s, 2: stride 2s, 1: stride s, in vectors) of level k, and with
  // in_vec (s = 1 only) the strides 2 and 1 inside the vectors
  auto pass = [&](int64_t k, int s_log, int mask, bool in_vec) {
    for (int g = tid; g < ngroups; g += nt) {
      const int v0 = ((g >> s_log) << (3 + s_log)) + (g & ((1 << s_log) - 1));
      f32x4 e[8];
      bool asc[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const int v = v0 + (m << s_log);
        e[m] = s4[phys(v)];
        asc[m] = ((gbase + 4 * (int64_t)v) & k) == 0;
      }
      if (mask & 4) vec_stage<4>(e, asc);
      if (mask & 2) vec_stage<2>(e, asc);
      if (mask & 1) vec_stage<1>(e, asc);
      if (in_vec) in_stages(e, asc, true);
#pragma unroll
      for (int m = 0; m < 8; ++m) s4[phys(v0 + (m << s_log))] = e[m];
    }
    __syncthreads();
  };

  int64_t k = k_first;
  if (k_first <= 2) {                                  // levels 2 .. 32 on 32 consecutive elements, one round trip
    for (int g = tid; g < ngroups; g += nt) {
      f32x4 e[8];
      bool asc[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) e[m] = s4[phys(8 * g + m)];
#pragma unroll
      for (int m = 0; m < 8; ++m) { cx_in<0, 1>(e[m], true); cx_in<2, 3>(e[m], false); }                // level 2
#pragma unroll
      for (int m = 0; m < 8; ++m) asc[m] = (m & 1) == 0;                                                  // level 4
      in_stages(e, asc, true);
#pragma unroll
      for (int m = 0; m < 8; ++m) asc[m] = (m & 2) == 0;                                                  // level 8
      vec_stage<1>(e, asc); in_stages(e, asc, true);
#pragma unroll
      for (int m = 0; m < 8; ++m) asc[m] = (m & 4) == 0;                                                  // level 16
      vec_stage<2>(e, asc); vec_stage<1>(e, asc); in_stages(e, asc, true);
      const bool a32 = ((gbase + 32 * (int64_t)g) & 32) == 0;                                             // level 32
#pragma unroll
      for (int m = 0; m < 8; ++m) asc[m] = a32;
      vec_stage<4>(e, asc); vec_stage<2>(e, asc); vec_stage<1>(e, asc); in_stages(e, asc, true);
#pragma unroll
      for (int m = 0; m < 8; ++m) s4[phys(8 * g + m)] = e[m];
    }
    __syncthreads();
    k = 64;
  }
  for (; k <= k_last; k <<= 1) {
    // vector-stride stages of this level inside the chunk: strides min(k, ch) / 8 ... 1
    int cur = 0;
    for (int64_t j = (k < ch ? k : (int64_t)ch) >> 3; j >= 1; j >>= 1) ++cur;
    while (cur > 3) {                                  // leading stages: first the remainder, then threes
      const int g = (cur - 3) % 3 == 0 ? 3 : (cur - 3) % 3;
      // the eight vectors always span twice the top stride (s = top / 4); a remainder runs the upper stages only
      pass(k, cur - 3, g == 3 ? 7 : (g == 2 ? 6 : 4), false);
      cur -= g;
    }
    pass(k, 0, cur == 3 ? 7 : (cur == 2 ? 3 : 1), true);
  }
  if (ref == nullptr) {
    for (int v = tid; v < nvec; v += nt) *reinterpret_cast<f32x4*>(row + 4 * v) = s4[phys(v)];
    return;
  }
  const int seg = blockIdx.y;
  const float* rrow = ref + (int64_t)(ref_shared ? seg % L : seg) * Tpad;
  float sum = 0.0f;
  for (int v = tid; 4 * (int64_t)v < T; v += nt) {   // the padding (+inf on both sides) is left out
    const f32x4 a = s4[phys(v)], b = *reinterpret_cast<const f32x4*>(rrow + 4 * v);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4 * (int64_t)v + i < T) sum += fabsf(a[i] - b[i]);
  }
  sum = wave_sum(sum);
  __syncthreads();                                  // the row is no longer needed: reuse its first words
  if ((tid & 63) == 0) s[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.0f;
    for (int w = 0; w < nt / 64; ++w) tot += s[w];
    w1[first_seg + seg] = tot;
  }
}

// One stage (k, j) with j >= chunk size, straight on global memory.
__global__ __launch_bounds__(256) void sw_sort_global_kernel(float* __restrict__ P, int64_t Tpad, int64_t k, int64_t j) {
  const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= (Tpad >> 1)) return;
  float* row = P + (int64_t)blockIdx.y * Tpad;
  const int64_t i = 2 * p - (p & (j - 1));
  const bool asc = (i & k) == 0;
  const float a = row[i], b = row[i + j];
  if ((a > b) == asc) { row[i] = b; row[i + j] = a; }
}

// Unfused W1 for rows longer than one chunk: one workgroup per segment, fixed order.
__global__ __launch_bounds__(256) void sw_w1_kernel(const float* __restrict__ P, const float* __restrict__ ref, int ref_shared, int L,
                                                    int64_t T, int64_t Tpad, float* __restrict__ w1, int first_seg) {
  __shared__ float red[4];
  const int seg = blockIdx.x;
  const float* a = P + (int64_t)seg * Tpad;
  const float* b = ref + (int64_t)(ref_shared ? seg % L : seg) * Tpad;
  float sum = 0.0f;
  for (int64_t i = threadIdx.x; i < T; i += 256) sum += fabsf(a[i] - b[i]);
  sum = block_sum_256(sum, red);
  if (threadIdx.x == 0) w1[first_seg + seg] = sum;
}

// Omega_SW = (1 / L) sum_l (1 / T) sum_t |...|; flagged iff not (Omega_SW <= tau).
__global__ void sw_finalize_kernel(const float* __restrict__ w1, int n_claims, int L, int64_t T, float tau, float* __restrict__ sw_out,
                                   sv_result* __restrict__ results) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_claims) return;
  double tot = 0.0;
  for (int l = 0; l < L; ++l) tot += (double)w1[(int64_t)c * L + l];
  const float v = T > 0 ? (float)(tot / ((double)L * (double)T)) : 0.0f;
  if (sw_out) sw_out[c] = v;
  if (results) {
    results[c].metric_mask |= SV_M_SW;
    if (!(v <= tau)) results[c].flag = 1u;
  }
}

// A reference that is only known through its projections (kept up to date by sw_proj_ema_kernel): copy the L rows
// into the slot the sort works on, with the padding behind the T samples set to +inf.
__global__ __launch_bounds__(256) void sw_copy_pad_kernel(float* __restrict__ dst, const float* __restrict__ src, int64_t T, int64_t Tpad) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= Tpad) return;
  const int64_t i = (int64_t)blockIdx.y * Tpad + t;
  dst[i] = t < T ? src[i] : __builtin_huge_valf();
}

// The projection is linear, so the projections of m <- beta m + (1 - beta) mean_clean(x) are the same combination of
// the projections: pm <- beta pm + w sum_{c not skipped} P_c (index order, fp32), per direction and token.
__global__ __launch_bounds__(256) void sw_proj_ema_kernel(float* __restrict__ pm, const float* __restrict__ P, int n, uint32_t skip,
                                                          int64_t slot, int64_t T, int64_t Tpad, float beta, float w) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int64_t i = (int64_t)blockIdx.y * Tpad + t;
  float acc = 0.0f;
  for (int c = 0; c < n; ++c)
    if (((skip >> c) & 1u) == 0) acc += P[(int64_t)c * slot + i];
  pm[i] = beta * pm[i] + w * acc;
}

template <typename E, typename E2, int LB>
hipError_t project_launch(const void* X, int64_t stride, int count, const void* X2, int n2, const void* U, int D, int64_t T, int64_t Tpad,
                          float* P, float* P2, hipStream_t st) {
  auto kern = sw_project_kernel<E, E2, LB>;
  constexpr int lds = kSwDepth * (kSwTile + LB * 32 * 128);   // direction chunks of 128 (bf16 signal) or 64 bytes per row
  static bool configured = false;   // per process; the attribute is per function
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  dim3 grid((unsigned)((Tpad + 255) / 256), (unsigned)(count + n2));
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const E*)X, stride, (const E2*)X2, n2, (const bf16*)U, D, T, Tpad, P, P2);
  return hipGetLastError();
}

template <typename E, typename E2>
hipError_t project_dispatch(const void* X, int64_t stride, int count, const void* X2, int n2, const void* U, int L, int D, int64_t T,
                            int64_t Tpad, float* P, float* P2, hipStream_t st) {
  switch (L / 32) {
    case 1: return project_launch<E, E2, 1>(X, stride, count, X2, n2, U, D, T, Tpad, P, P2, st);
    case 2: return project_launch<E, E2, 2>(X, stride, count, X2, n2, U, D, T, Tpad, P, P2, st);
    case 3: return project_launch<E, E2, 3>(X, stride, count, X2, n2, U, D, T, Tpad, P, P2, st);
    default: return project_launch<E, E2, 4>(X, stride, count, X2, n2, U, D, T, Tpad, P, P2, st);
  }
}

}  // namespace

int64_t sw_padded_len(int64_t T) {
  int64_t p = 128;
  while (p < T) p <<= 1;
  return p;
}

hipError_t launch_sw_project(const void* X, int64_t stride, int count, int dtype, const void* U, int L, int D, int64_t T, int64_t Tpad,
                             float* P, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  return dtype == SV_BF16 ? project_dispatch<bf16, bf16>(X, stride, count, nullptr, 0, U, L, D, T, Tpad, P, nullptr, st)
                          : project_dispatch<float, float>(X, stride, count, nullptr, 0, U, L, D, T, Tpad, P, nullptr, st);
}

bool sw_project_with_ref_supported(int dtype, int ref_dtype) { return dtype == ref_dtype || (dtype == SV_BF16 && ref_dtype == SV_F32); }

hipError_t launch_sw_project_with_ref(const void* X, int64_t stride, int count, int dtype, const void* ref, int ref_dtype, const void* U,
                                      int L, int D, int64_t T, int64_t Tpad, float* P, float* Pref, hipStream_t st) {
  if (count <= 0 || !sw_project_with_ref_supported(dtype, ref_dtype)) return hipErrorInvalidValue;
  if (dtype == SV_BF16 && ref_dtype == SV_F32) return project_dispatch<bf16, float>(X, stride, count, ref, 1, U, L, D, T, Tpad, P, Pref, st);
  return dtype == SV_BF16 ? project_dispatch<bf16, bf16>(X, stride, count, ref, 1, U, L, D, T, Tpad, P, Pref, st)
                          : project_dispatch<float, float>(X, stride, count, ref, 1, U, L, D, T, Tpad, P, Pref, st);
}

hipError_t launch_sw_sort(float* P, int n_seg, int64_t T, int64_t Tpad, const float* ref, int ref_shared, int L, float* w1,
                          int first_seg, hipStream_t st) {
  if (n_seg <= 0) return hipSuccess;
  const int ch = (int)min(Tpad, (int64_t)kSortChunkMax);
  const int nt = max(64, min(512, ch / 32));      // a thread holds 32 elements in the register passes
  const size_t lds = (size_t)ch * sizeof(float);
  const dim3 grid((unsigned)(Tpad / ch), (unsigned)n_seg);
  if (Tpad == ch) {
    sw_sort_chunk_kernel<<<grid, nt, lds, st>>>(P, Tpad, ch, 2, Tpad, ref, ref_shared, L, T, w1, first_seg);
    return hipGetLastError();
  }
  sw_sort_chunk_kernel<<<grid, nt, lds, st>>>(P, Tpad, ch, 2, ch, nullptr, 0, L, T, nullptr, 0);
  for (int64_t k = 2 * (int64_t)ch; k <= Tpad; k <<= 1) {
    for (int64_t j = k >> 1; j >= ch; j >>= 1)
      sw_sort_global_kernel<<<dim3((unsigned)((Tpad / 2 + 255) / 256), (unsigned)n_seg), 256, 0, st>>>(P, Tpad, k, j);
    sw_sort_chunk_kernel<<<grid, nt, lds, st>>>(P, Tpad, ch, k, k, nullptr, 0, L, T, nullptr, 0);
  }
  if (ref) sw_w1_kernel<<<n_seg, 256, 0, st>>>(P, ref, ref_shared, L, T, Tpad, w1, first_seg);
  return hipGetLastError();
}

hipError_t launch_sw_copy_pad(float* dst, const float* src, int L, int64_t T, int64_t Tpad, hipStream_t st) {
  sw_copy_pad_kernel<<<dim3((unsigned)((Tpad + 255) / 256), (unsigned)L), 256, 0, st>>>(dst, src, T, Tpad);
  return hipGetLastError();
}

hipError_t launch_sw_proj_ema(float* pm, const float* P, int n, uint32_t skip, int L, int64_t T, int64_t Tpad, float beta, float w,
                              hipStream_t st) {
  sw_proj_ema_kernel<<<dim3((unsigned)((T + 255) / 256), (unsigned)L), 256, 0, st>>>(pm, P, n, skip, (int64_t)L * Tpad, T, Tpad, beta, w);
  return hipGetLastError();
}

hipError_t launch_sw_finalize(const float* w1, int n_claims, int L, int64_t T, float tau, float* sw_out, sv_result* results,
                              hipStream_t st) {
  if (n_claims <= 0) return hipSuccess;
  sw_finalize_kernel<<<(n_claims + 127) / 128, 128, 0, st>>>(w1, n_claims, L, T, tau, sw_out, results);
  return hipGetLastError();
}

}  // namespace sv
