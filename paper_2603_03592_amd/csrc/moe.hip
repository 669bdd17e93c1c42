// Routing side of the mixture-of-experts MLP (the model family of the paper's "Alternative Architectures"
// paragraph): router scores and top-k choice, a stable counting sort of the (token, choice) pairs by expert,
// the gather of token rows into expert-contiguous buffers, and the weighted combination of the expert outputs
// (forward) or of their input gradients plus the gradient through the gate values (backward).  The expert
// feed-forward products themselves run on the GEMM kernels in their grouped form.
//
// Layout: the pairs of one expert occupy consecutive rows of the sorted buffers, in token order, and every
// expert's run is padded to a multiple of 256 rows (the GEMM row tile), so that one row tile never mixes experts.
// Everything here is bound by HBM traffic or by launch latency; there is no contraction worth the matrix cores
// (the router product has only n_experts <= 16 output columns).
#include "common.h"

namespace sv {
namespace {

constexpr int kME = kMoeMaxExperts, kMK = kMoeMaxTopK;

__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }

// ---------------------------------------------------------------------------------------------- route
// One wave per token: E dot products of length D in fp32, scores, top-k by repeated maximum of the LOGITS (both
// score functions increase with the logit, which unlike them does not saturate; strict '>' keeps the lower index on
// ties), gate values from the scores.
template <typename T>
__global__ __launch_bounds__(256) void moe_route_kernel(const T* __restrict__ n, const T* __restrict__ wr, int64_t Tn, int D, int E, int K,
                                                        int score_kind, int norm, int32_t* __restrict__ sel, float* __restrict__ gate,
                                                        float* __restrict__ score) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  float acc[kME];
#pragma unroll
  for (int e = 0; e < kME; ++e) acc[e] = 0.0f;
  for (int c = lane * 8; c < D; c += 512) {
    float x[8];
    load8(n + t * D + c, x);
#pragma unroll
    for (int e = 0; e < kME; ++e) {
      if (e < E) {
        float w[8];
        load8(wr + (int64_t)e * D + c, w);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[e] = fmaf(x[i], w[i], acc[e]);
      }
    }
  }
  float s[kME];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < kME; ++e) {
    acc[e] = e < E ? wave_sum(acc[e]) : -INFINITY;
    mx = fmaxf(mx, acc[e]);
  }
  if (score_kind == SV_ROUTER_SIGMOID) {
#pragma unroll
    for (int e = 0; e < kME; ++e) s[e] = e < E ? sigmoid_f(acc[e]) : -1.0f;
  } else {
    float z = 0.0f;
#pragma unroll
    for (int e = 0; e < kME; ++e) { s[e] = e < E ? expf(acc[e] - mx) : 0.0f; z += s[e]; }
#pragma unroll
    for (int e = 0; e < kME; ++e) s[e] = e < E ? s[e] / z : -1.0f;
  }
  uint32_t used = 0;
  int chosen[kMK];
  float g[kMK];
  float gsum = 0.0f;
#pragma unroll
  for (int j = 0; j < kMK; ++j) {
    chosen[j] = 0; g[j] = 0.0f;
    if (j < K) {
      int best = -1;
      float bl = 0.0f, bs = 0.0f;
#pragma unroll
      for (int e = 0; e < kME; ++e) {
        const bool free_ = e < E && !((used >> e) & 1u);
        if (free_ && (best < 0 || acc[e] > bl)) { best = e; bl = acc[e]; bs = s[e]; }
      }
      used |= 1u << best;
      chosen[j] = best; g[j] = bs; gsum += bs;
    }
  }
#pragma unroll
  for (int j = 0; j < kMK; ++j)
    if (j < K && lane == j) {
      sel[t * K + j] = chosen[j];
      gate[t * K + j] = norm ? g[j] / gsum : g[j];
    }
#pragma unroll
  for (int e = 0; e < kME; ++e)
    if (e < E && lane == 32 + e) score[t * E + e] = s[e];
}

// ---------------------------------------------------------------------------------------------- counting sort
__global__ __launch_bounds__(256) void moe_count_kernel(const int32_t* __restrict__ sel, int64_t n_entries, int E, int32_t* __restrict__ chunk_counts) {
  __shared__ int cnt[kME];
  if (threadIdx.x < kME) cnt[threadIdx.x] = 0;
  __syncthreads();
  const int64_t first = (int64_t)blockIdx.x * kMoeChunk;
#pragma unroll
  for (int r = 0; r < kMoeChunk / 256; ++r) {
    const int64_t i = first + r * 256 + threadIdx.x;
    if (i < n_entries) atomicAdd(&cnt[sel[i]], 1);
  }
  __syncthreads();
  if ((int)threadIdx.x < E) chunk_counts[(int64_t)blockIdx.x * E + threadIdx.x] = cnt[threadIdx.x];
}

// One workgroup: per expert the exclusive prefix of its chunk counts, the padded expert segments, the expert of
// every 256-row block (blocks behind the rows in use name expert 0; the products never reach them).  Thread
// (e, s) = (tid / 16, tid % 16) owns the s-th sixteenth of expert e's chunks: sum, prefix over s, then write.
__global__ __launch_bounds__(256) void moe_offsets_kernel(const int32_t* __restrict__ chunk_counts, int n_chunks, int E, int max_tiles,
                                                          int32_t* __restrict__ chunk_base, int32_t* __restrict__ meta,
                                                          int32_t* __restrict__ tile_expert) {
  __shared__ int part[kME][17], total[kME], start[kME + 1];
  const int tid = threadIdx.x, e = tid >> 4, sgm = tid & 15;
  const int per = (n_chunks + 15) / 16, c0 = sgm * per, c1 = min(n_chunks, c0 + per);
  int sum = 0;
  if (e < E)
    for (int c = c0; c < c1; ++c) sum += chunk_counts[(int64_t)c * E + e];
  part[e][sgm] = sum;
  __syncthreads();
  if (e < E) {
    int run = 0;
    for (int i = 0; i < sgm; ++i) run += part[e][i];
    for (int c = c0; c < c1; ++c) {
      chunk_base[(int64_t)c * E + e] = run;
      run += chunk_counts[(int64_t)c * E + e];
    }
    if (sgm == 15) total[e] = run;
  }
  __syncthreads();
  if (tid == 0) {
    int s = 0;
    for (int x = 0; x < E; ++x) { start[x] = s; s += (total[x] + 255) & ~255; }
    start[E] = s;
    meta[0] = s;
  }
  __syncthreads();
  if (tid < E) { meta[1 + tid] = start[tid]; meta[1 + E + tid] = total[tid]; }
  for (int tile = tid; tile < max_tiles; tile += 256) {
    int e_of = 0;
    for (int x = 0; x < E; ++x)
      if (tile * 256 >= start[x] && tile * 256 < start[x + 1]) e_of = x;
    tile_expert[tile] = e_of;
  }
}

// Stable placement: within an expert, pairs keep their (token, choice) order.
__global__ __launch_bounds__(256) void moe_scatter_kernel(const int32_t* __restrict__ sel, const float* __restrict__ gate, int64_t n_entries, int E,
                                                          int K, const int32_t* __restrict__ chunk_base, const int32_t* __restrict__ meta,
                                                          int32_t* __restrict__ pos, int32_t* __restrict__ row_token, float* __restrict__ row_gate) {
  __shared__ int run[kME], wcnt[4][kME];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < kME) run[tid] = tid < E ? meta[1 + tid] + chunk_base[(int64_t)blockIdx.x * E + tid] : 0;
  const int64_t first = (int64_t)blockIdx.x * kMoeChunk;
  for (int r = 0; r < kMoeChunk / 256; ++r) {
    const int64_t i = first + r * 256 + tid;
    const int x = i < n_entries ? sel[i] : -1;
    int rank = 0;
    for (int e = 0; e < E; ++e) {
      const unsigned long long mask = __ballot(x == e);
      if (x == e) rank = __popcll(mask & ((1ull << lane) - 1ull));
      if (lane == 0) wcnt[wave][e] = __popcll(mask);
    }
    __syncthreads();
    if (x >= 0) {
      int p = run[x] + rank;
      for (int w = 0; w < wave; ++w) p += wcnt[w][x];
      pos[i] = p;
      row_token[p] = (int32_t)(i / K);
      row_gate[p] = gate[i];
    }
    __syncthreads();
    if (tid < E) run[tid] += wcnt[0][tid] + wcnt[1][tid] + wcnt[2][tid] + wcnt[3][tid];
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------- gather
template <typename T>
__global__ __launch_bounds__(256) void moe_gather_kernel(const T* __restrict__ src, int D, int E, const int32_t* __restrict__ row_token,
                                                         const float* __restrict__ row_gate, const int32_t* __restrict__ meta,
                                                         const int32_t* __restrict__ tile_expert, int scaled, T* __restrict__ dst) {
  const int lane = threadIdx.x & 63;
  const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (p >= meta[0]) return;
  const int e = tile_expert[p >> 8];
  const bool live = p - meta[1 + e] < meta[1 + E + e];
  const int64_t t = live ? row_token[p] : 0;
  const float sc = live ? (scaled ? row_gate[p] : 1.0f) : 0.0f;
  for (int c = lane * 8; c < D; c += 512) {
    float v[8];
    load8(src + t * D + c, v);
    if (scaled || !live) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = live ? v[i] * sc : 0.0f;
    }
    store8(dst + p * D + c, v);
  }
}

// ---------------------------------------------------------------------------------------------- combine
template <typename T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T* base, const T* __restrict__ yp, int64_t Tn, int D, int K,
                                                          const int32_t* __restrict__ pos, const float* __restrict__ gate, T* y) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  int64_t p[kMK];
  float g[kMK];
#pragma unroll
  for (int j = 0; j < kMK; ++j) { p[j] = j < K ? pos[t * K + j] : 0; g[j] = j < K ? gate[t * K + j] : 0.0f; }
  for (int c = lane * 8; c < D; c += 512) {
    float v[8];
    load8(base + t * D + c, v);
#pragma unroll
    for (int j = 0; j < kMK; ++j)
      if (j < K) {
        float u[8];
        load8(yp + p[j] * D + c, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = fmaf(g[j], u[i], v[i]);
      }
    store8(y + t * D + c, v);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void moe_combine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ yp, const T* __restrict__ dxp,
                                                              const T* __restrict__ wr, int64_t Tn, int D, int E, int K, int score_kind,
                                                              int norm, const int32_t* __restrict__ pos, const int32_t* __restrict__ sel,
                                                              const float* __restrict__ gate, const float* __restrict__ score,
                                                              int accumulate, T* dn) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  int64_t p[kMK];
  int ex[kMK];
  float g[kMK], dg[kMK];
#pragma unroll
  for (int j = 0; j < kMK; ++j) {
    p[j] = j < K ? pos[t * K + j] : 0;
    ex[j] = j < K ? sel[t * K + j] : -1;
    g[j] = j < K ? gate[t * K + j] : 0.0f;
    dg[j] = 0.0f;
  }
  // gradient with respect to each gate value: <dy_t, y_e(t)>
  for (int c = lane * 8; c < D; c += 512) {
    float d[8];
    load8(dy + t * D + c, d);
#pragma unroll
    for (int j = 0; j < kMK; ++j)
      if (j < K) {
        float u[8];
        load8(yp + p[j] * D + c, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) dg[j] = fmaf(d[i], u[i], dg[j]);
      }
  }
  float s[kME], ds[kME], dl[kME];
#pragma unroll
  for (int e = 0; e < kME; ++e) { s[e] = e < E ? score[t * E + e] : 0.0f; ds[e] = 0.0f; }
  float z = 0.0f, dgg = 0.0f;
#pragma unroll
  for (int j = 0; j < kMK; ++j) {
    if (j < K) dg[j] = wave_sum(dg[j]);
    dgg += dg[j] * g[j];
#pragma unroll
    for (int e = 0; e < kME; ++e)
      if (ex[j] == e) z += s[e];
  }
#pragma unroll
  for (int j = 0; j < kMK; ++j) {
    const float dss = norm ? (dg[j] - dgg) / z : dg[j];
#pragma unroll
    for (int e = 0; e < kME; ++e)
      if (ex[j] == e) ds[e] = dss;
  }
  if (score_kind == SV_ROUTER_SIGMOID) {
#pragma unroll
    for (int e = 0; e < kME; ++e) dl[e] = ds[e] * s[e] * (1.0f - s[e]);
  } else {
    float dot = 0.0f;
#pragma unroll
    for (int e = 0; e < kME; ++e) dot += ds[e] * s[e];
#pragma unroll
    for (int e = 0; e < kME; ++e) dl[e] = s[e] * (ds[e] - dot);
  }
  for (int c = lane * 8; c < D; c += 512) {
    float v[8];
    if (accumulate) load8(dn + t * D + c, v);
    else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    }
#pragma unroll
    for (int j = 0; j < kMK; ++j)
      if (j < K) {
        float u[8];
        load8(dxp + p[j] * D + c, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] += u[i];
      }
#pragma unroll
    for (int e = 0; e < kME; ++e)
      if (e < E) {
        float w[8];
        load8(wr + (int64_t)e * D + c, w);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = fmaf(dl[e], w[i], v[i]);
      }
    store8(dn + t * D + c, v);
  }
}

}  // namespace

int64_t moe_padded_rows(int64_t T, int K, int E) { return ((T * K + 255) / 256 + E) * 256; }

hipError_t launch_moe_route(const void* n, const void* w_router, int64_t T, int D, int E, int K, int score_kind, int norm, int dtype,
                            const MoeRoute& r, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  if (E < 1 || E > kME || K < 1 || K > kMK || K > E || D % 8) return hipErrorInvalidValue;
  const unsigned tok_grid = (unsigned)((T + 3) / 4);
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(moe_route_kernel<bf16>, dim3(tok_grid), dim3(256), 0, st, (const bf16*)n, (const bf16*)w_router, T, D, E, K, score_kind, norm,
                       r.sel, r.gate, r.score);
  else
    hipLaunchKernelGGL(moe_route_kernel<float>, dim3(tok_grid), dim3(256), 0, st, (const float*)n, (const float*)w_router, T, D, E, K, score_kind,
                       norm, r.sel, r.gate, r.score);
  const int64_t n_entries = T * K;
  const int n_chunks = (int)((n_entries + kMoeChunk - 1) / kMoeChunk);
  const int max_tiles = (int)(moe_padded_rows(T, K, E) / 256);
  hipLaunchKernelGGL(moe_count_kernel, dim3(n_chunks), dim3(256), 0, st, r.sel, n_entries, E, r.chunk_counts);
  hipLaunchKernelGGL(moe_offsets_kernel, dim3(1), dim3(256), 0, st, r.chunk_counts, n_chunks, E, max_tiles, r.chunk_base, r.meta, r.tile_expert);
  hipLaunchKernelGGL(moe_scatter_kernel, dim3(n_chunks), dim3(256), 0, st, r.sel, r.gate, n_entries, E, K, r.chunk_base, r.meta, r.pos, r.row_token,
                     r.row_gate);
  return hipGetLastError();
}

hipError_t launch_moe_gather(const void* src, int D, int64_t Mp, int E, const MoeRoute& r, int scaled, void* dst, int dtype, hipStream_t st) {
  if (Mp <= 0) return hipSuccess;
  const unsigned grid = (unsigned)((Mp + 3) / 4);
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(moe_gather_kernel<bf16>, dim3(grid), dim3(256), 0, st, (const bf16*)src, D, E, r.row_token, r.row_gate, r.meta, r.tile_expert,
                       scaled, (bf16*)dst);
  else
    hipLaunchKernelGGL(moe_gather_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)src, D, E, r.row_token, r.row_gate, r.meta,
                       r.tile_expert, scaled, (float*)dst);
  return hipGetLastError();
}

hipError_t launch_moe_combine(const void* base, const void* yp, int64_t T, int D, int K, const MoeRoute& r, void* y, int dtype, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  const unsigned grid = (unsigned)((T + 3) / 4);
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(moe_combine_kernel<bf16>, dim3(grid), dim3(256), 0, st, (const bf16*)base, (const bf16*)yp, T, D, K, r.pos, r.gate, (bf16*)y);
  else
    hipLaunchKernelGGL(moe_combine_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)base, (const float*)yp, T, D, K, r.pos, r.gate,
                       (float*)y);
  return hipGetLastError();
}

hipError_t launch_moe_combine_bwd(const void* dy, const void* yp, const void* dxp, const void* w_router, int64_t T, int D, int E, int K,
                                  int score_kind, int norm, const MoeRoute& r, int accumulate, void* dn, int dtype, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  const unsigned grid = (unsigned)((T + 3) / 4);
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(moe_combine_bwd_kernel<bf16>, dim3(grid), dim3(256), 0, st, (const bf16*)dy, (const bf16*)yp, (const bf16*)dxp,
                       (const bf16*)w_router, T, D, E, K, score_kind, norm, r.pos, r.sel, r.gate, r.score, accumulate, (bf16*)dn);
  else
    hipLaunchKernelGGL(moe_combine_bwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)dy, (const float*)yp, (const float*)dxp,
                       (const float*)w_router, T, D, E, K, score_kind, norm, r.pos, r.sel, r.gate, r.score, accumulate, (float*)dn);
  return hipGetLastError();
}

}  // namespace sv
