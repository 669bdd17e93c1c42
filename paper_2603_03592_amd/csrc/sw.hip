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

constexpr int kSortChunkMax = 16384;   // floats sorted in LDS by one workgroup (64 KB)

// ---------------------------------------------------------------------------------------------
// Projection.  A workgroup of 4 waves owns 256 tokens (64 per wave, two blocks of 32) and all
// L = 32 * LB directions; the contraction runs over the feature axis in steps of 16 on
// v_mfma_f32_32x32x16_bf16 with the directions in the A slot, so a lane ends up with one token
// (lane & 31) and the directions 8q + 4 (lane >> 5) + r of each block of 32.
// The signal goes global -> register directly: inside a 64-feature chunk the k index is permuted
// (lane half h reads the 16-byte pieces 4h .. 4h+3, one per step) so that the four steps of a lane
// read 64 contiguous bytes of its row; the same permutation is applied to the directions, which
// leaves the dot product unchanged.  The directions' 64-feature chunk [L, 64] is staged through
// LDS once per workgroup (double buffered, 16-byte pieces XOR-swizzled by the row) so that L2 sees
// one read of it per 256 tokens, and the bf16 signal is prefetched one chunk ahead in registers.
// fp32 signals are split into three bf16 terms (x = hi + mid + lo exactly), three MFMAs per step:
// every product is exact in fp32, so the result has fp32-accumulation accuracy.
__device__ __forceinline__ int sw_swz(int row) { return (row ^ (row >> 3)) & 7; }

template <int LB>
__device__ __forceinline__ void mac_bf16(const bf16x8 (&u)[LB], const bf16x8& x, f32x16 (&acc)[LB]) {
#pragma unroll
  for (int b = 0; b < LB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u[b], x, acc[b], 0, 0, 0);
}

template <int LB>
__device__ __forceinline__ void mac_f32(const bf16x8 (&u)[LB], const float* p, f32x16 (&acc)[LB]) {
  float x[8];
  load8(p, x);
  bf16x8 hi, mid, lo;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const bf16 a = (bf16)x[i];
    const float r1 = x[i] - (float)a;
    const bf16 b = (bf16)r1;
    const float r2 = r1 - (float)b;
    hi[i] = a; mid[i] = b; lo[i] = (bf16)r2;
  }
  mac_bf16<LB>(u, lo, acc);
  mac_bf16<LB>(u, mid, acc);
  mac_bf16<LB>(u, hi, acc);
}

template <typename E, int LB>
__global__ __launch_bounds__(256) void sw_project_kernel(const E* __restrict__ X, int64_t x_stride, const bf16* __restrict__ U,
                                                         int D, int64_t T, int64_t Tpad, float* __restrict__ P) {
  constexpr bool kBf16 = sizeof(E) == 2;
  __shared__ __attribute__((aligned(16))) char us[2][LB * 32 * 128];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, lhi = lane >> 5;
  const int64_t t0 = ((int64_t)blockIdx.x * 4 + wave) * 64;
  const E* xp[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t row = min(t0 + tb * 32 + l31, T - 1);          // rows past the end re-read the last one
    xp[tb] = X + (int64_t)blockIdx.y * x_stride + row * D + lhi * 32;
  }
  // staging of the directions' chunk: thread e owns the 16-byte pieces e, e + 256, ... of the [L, 64] tile
  const bf16* ug[LB];
  int ul[LB];
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int e = tid + 256 * i, r = e >> 3, c = e & 7;
    ug[i] = U + (int64_t)r * D + c * 8;
    ul[i] = r * 128 + ((c ^ sw_swz(r)) << 4);
  }
  f32x16 acc[2][LB];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int b = 0; b < LB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tb][b][i] = 0.0f;

  bf16x8 ureg[LB];
  bf16x8 xcur[2][4], xnext[2][4];
#pragma unroll
  for (int i = 0; i < LB; ++i) *reinterpret_cast<bf16x8*>(us[0] + ul[i]) = *reinterpret_cast<const bf16x8*>(ug[i]);
  if (kBf16) {
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int s = 0; s < 4; ++s) xcur[tb][s] = *reinterpret_cast<const bf16x8*>((const bf16*)xp[tb] + s * 8);
  }
  __syncthreads();
  const int nchunk = D >> 6;
  for (int kc = 0; kc < nchunk; ++kc) {
    const int k0 = kc << 6;
    const bool more = kc + 1 < nchunk;
    if (more) {
#pragma unroll
      for (int i = 0; i < LB; ++i) ureg[i] = *reinterpret_cast<const bf16x8*>(ug[i] + k0 + 64);
      if (kBf16) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int s = 0; s < 4; ++s) xnext[tb][s] = *reinterpret_cast<const bf16x8*>((const bf16*)xp[tb] + k0 + 64 + s * 8);
      }
    }
    const char* ub = us[kc & 1];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 u[LB];
#pragma unroll
      for (int b = 0; b < LB; ++b) {
        const int r = b * 32 + l31;
        u[b] = *reinterpret_cast<const bf16x8*>(ub + r * 128 + (((lhi * 4 + s) ^ sw_swz(r)) << 4));
      }
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        if (kBf16) mac_bf16<LB>(u, xcur[tb][s], acc[tb]);
        else mac_f32<LB>(u, (const float*)xp[tb] + k0 + s * 8, acc[tb]);
      }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < LB; ++i) *reinterpret_cast<bf16x8*>(us[(kc + 1) & 1] + ul[i]) = ureg[i];
      if (kBf16) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int s = 0; s < 4; ++s) xcur[tb][s] = xnext[tb][s];
      }
    }
    __syncthreads();
  }
  float* out = P + (int64_t)blockIdx.y * (LB * 32) * Tpad;
  const float inf = __builtin_huge_valf();                       // padding sorts behind every real sample
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
__global__ __launch_bounds__(1024) void sw_sort_chunk_kernel(float* __restrict__ P, int64_t Tpad, int ch, int64_t k_first, int64_t k_last,
                                                             const float* __restrict__ ref, int ref_shared, int L, int64_t T,
                                                             float* __restrict__ w1, int first_seg) {
  extern __shared__ __attribute__((aligned(16))) float s[];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int64_t gbase = (int64_t)blockIdx.x * ch;
  float* row = P + (int64_t)blockIdx.y * Tpad + gbase;
  for (int i = tid * 4; i < ch; i += nt * 4) *reinterpret_cast<f32x4*>(s + i) = *reinterpret_cast<const f32x4*>(row + i);
  __syncthreads();
  const int half = ch >> 1;
  for (int64_t k = k_first; k <= k_last; k <<= 1) {
    for (int j = (int)min(k >> 1, (int64_t)half); j > 0; j >>= 1) {
      for (int p = tid; p < half; p += nt) {
        const int i = 2 * p - (p & (j - 1));
        const bool asc = ((gbase + i) & k) == 0;
        const float a = s[i], b = s[i + j];
        if ((a > b) == asc) { s[i] = b; s[i + j] = a; }
      }
      __syncthreads();
    }
  }
  if (ref == nullptr) {
    for (int i = tid * 4; i < ch; i += nt * 4) *reinterpret_cast<f32x4*>(row + i) = *reinterpret_cast<const f32x4*>(s + i);
    return;
  }
  const int seg = blockIdx.y;
  const float* rrow = ref + (int64_t)(ref_shared ? seg % L : seg) * Tpad;
  float sum = 0.0f;
  for (int64_t i = tid; i < T; i += nt) sum += fabsf(s[i] - rrow[i]);
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

template <typename E>
hipError_t project_dispatch(const void* X, int64_t stride, int count, const void* U, int L, int D, int64_t T, int64_t Tpad, float* P,
                            hipStream_t st) {
  dim3 grid((unsigned)((Tpad + 255) / 256), (unsigned)count);
  switch (L / 32) {
    case 1: sw_project_kernel<E, 1><<<grid, 256, 0, st>>>((const E*)X, stride, (const bf16*)U, D, T, Tpad, P); break;
    case 2: sw_project_kernel<E, 2><<<grid, 256, 0, st>>>((const E*)X, stride, (const bf16*)U, D, T, Tpad, P); break;
    case 3: sw_project_kernel<E, 3><<<grid, 256, 0, st>>>((const E*)X, stride, (const bf16*)U, D, T, Tpad, P); break;
    default: sw_project_kernel<E, 4><<<grid, 256, 0, st>>>((const E*)X, stride, (const bf16*)U, D, T, Tpad, P); break;
  }
  return hipGetLastError();
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
  return dtype == SV_BF16 ? project_dispatch<bf16>(X, stride, count, U, L, D, T, Tpad, P, st)
                          : project_dispatch<float>(X, stride, count, U, L, D, T, Tpad, P, st);
}

hipError_t launch_sw_sort(float* P, int n_seg, int64_t T, int64_t Tpad, const float* ref, int ref_shared, int L, float* w1,
                          int first_seg, hipStream_t st) {
  if (n_seg <= 0) return hipSuccess;
  const int ch = (int)min(Tpad, (int64_t)kSortChunkMax);
  const int nt = min(1024, ch / 2);
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

hipError_t launch_sw_finalize(const float* w1, int n_claims, int L, int64_t T, float tau, float* sw_out, sv_result* results,
                              hipStream_t st) {
  if (n_claims <= 0) return hipSuccess;
  sw_finalize_kernel<<<(n_claims + 127) / 128, 128, 0, st>>>(w1, n_claims, L, T, tau, sw_out, results);
  return hipGetLastError();
}

}  // namespace sv
