// Plain kernels: every step of the block forward / input-gradient backward for any shape and
// for E = float or bf16 storage, all arithmetic in fp32 on the vector ALUs.  They are the
// product path for fp32 stages (the fp32 benchmark stage is tiny) and for the element-wise /
// row-wise steps of bf16 stages; bf16 contractions normally run on the MFMA kernels instead.
#include "common.h"

namespace sv {
namespace {

// ------------------------------------------------------------------------------------ GEMM
// 64x64 output tile, 16-deep K slices, 256 threads each owning a 4x4 micro-tile.
template <typename E, bool DUAL>
__global__ __launch_bounds__(256) void gemm_plain_kernel(GemmArgs a) {
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  __shared__ float Bs2[DUAL ? 16 : 1][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int M = a.m_dev ? *a.m_dev : a.M;   // grouped form: row count from device memory (the launch covers its bound)
  if (m0 >= M) return;
  const int64_t goff = a.tile_group ? (int64_t)a.tile_group[m0 >> 8] * a.group_stride : 0;
  float acc[4][4] = {}, acc2[4][4] = {};

  for (int s = 0; s < a.nseg; ++s) {
    const E* A = (const E*)a.seg[s].A;
    const E* B = (const E*)a.seg[s].B + goff;
    const E* B2 = a.B2 ? (const E*)a.B2 + goff : nullptr;
    const int64_t lda = a.seg[s].lda, ldb = a.seg[s].ldb;
    const int K = a.seg[s].K;
    for (int k0 = 0; k0 < K; k0 += 16) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = tid + i * 256;
        {
          const int r = e >> 4, k = e & 15;
          const bool ok = (m0 + r < M) && (k0 + k < K);
          As[k][r] = ok ? to_f32(A[(int64_t)(m0 + r) * lda + k0 + k]) : 0.0f;
        }
        if (!a.b_is_kn) {
          const int c = e >> 4, k = e & 15;
          const bool ok = (n0 + c < a.N) && (k0 + k < K);
          Bs[k][c] = ok ? to_f32(B[(int64_t)(n0 + c) * ldb + k0 + k]) : 0.0f;
          if (DUAL) Bs2[k][c] = ok ? to_f32(B2[(int64_t)(n0 + c) * a.ldb2 + k0 + k]) : 0.0f;
        } else {
          const int k = e >> 6, c = e & 63;
          const bool ok = (n0 + c < a.N) && (k0 + k < K);
          Bs[k][c] = ok ? to_f32(B[(int64_t)(k0 + k) * ldb + n0 + c]) : 0.0f;
          if (DUAL) Bs2[k][c] = ok ? to_f32(B2[(int64_t)(k0 + k) * a.ldb2 + n0 + c]) : 0.0f;
        }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        float av[4], bv[4], b2v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { av[i] = As[k][ty * 4 + i]; bv[i] = Bs[k][tx * 4 + i]; b2v[i] = DUAL ? Bs2[k][tx * 4 + i] : 0.0f; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
            if (DUAL) acc2[i][j] = fmaf(av[i], b2v[j], acc2[i][j]);
          }
      }
    }
  }

  E* C = (E*)a.C; E* C2 = (E*)a.C2; E* C3 = (E*)a.C3;
  const E* R = (const E*)a.R; const E* R2 = (const E*)a.R2;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = m0 + ty * 4 + i;
    if (r >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = n0 + tx * 4 + j;
      if (c >= a.N) continue;
      const int64_t ic = (int64_t)r * a.ldc + c, ir = (int64_t)r * a.ldr + c;
      const float v = acc[i][j];
      switch (a.epi) {
        case EPI_STORE: C[ic] = from_f32<E>(v); break;
        case EPI_RESID: C[ic] = from_f32<E>(v + to_f32(R[ir])); break;
        case EPI_GELU:
          C[ic] = from_f32<E>(gelu_f(v));
          if (C2) C2[ic] = from_f32<E>(v);
          break;
        case EPI_SWIGLU: {
          const float u = acc2[i][j];
          C[ic] = from_f32<E>(silu_f(v) * u);
          if (C2) C2[ic] = from_f32<E>(v);
          if (C3) C3[ic] = from_f32<E>(u);
        } break;
        case EPI_SWIGLU_BWD: {
          const float g = to_f32(R[ir]), u = to_f32(R2[ir]);
          C[ic] = from_f32<E>(v * u * silu_grad_f(g));
          C2[ic] = from_f32<E>(v * silu_f(g));
        } break;
        case EPI_GELU_BWD: C[ic] = from_f32<E>(v * gelu_grad_f(to_f32(R[ir]))); break;
      }
    }
  }
}

// ------------------------------------------------------------------------------------ norms
template <typename E>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const E* __restrict__ x, const E* __restrict__ g, const E* __restrict__ b,
                                                       E* __restrict__ out, int D, int kind, float eps) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const E* xr = x + row * D;
  E* orow = out + row * D;
  float mean = 0.0f;
  if (kind == SV_NORM_LN) {
    float s = 0.0f;
    for (int k = threadIdx.x * 8; k < D; k += 2048) { float v[8]; load8(xr + k, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) s += v[j]; }
    mean = block_sum_256(s, red) / (float)D;
  }
  float ss = 0.0f;
  for (int k = threadIdx.x * 8; k < D; k += 2048) { float v[8]; load8(xr + k, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float d = v[j] - mean; ss += d * d; } }
  const float rinv = rsqrtf(block_sum_256(ss, red) / (float)D + eps);
  for (int k = threadIdx.x * 8; k < D; k += 2048) {
    float v[8], gv[8], bv[8], o[8];
    load8(xr + k, v); load8(g + k, gv);
    if (kind == SV_NORM_LN) load8(b + k, bv);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (v[j] - mean) * rinv * gv[j] + (kind == SV_NORM_LN ? bv[j] : 0.0f);
    store8(orow + k, o);
  }
}

// The pieces of an RMSNorm that runs inside its neighbouring products.
__global__ __launch_bounds__(256) void rms_rstd_kernel(const bf16* __restrict__ x, float* __restrict__ rstd, int64_t T, int D, float eps) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);          // one wave per row
  if (row >= T) return;
  const bf16* xr = x + row * D;
  float ss = 0.0f;
  for (int k = (threadIdx.x & 63) * 8; k < D; k += 512) { float v[8]; load8(xr + k, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j]; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) rstd[row] = rsqrtf(ss / (float)D + eps);
}
__global__ __launch_bounds__(256) void rms_rstd_partials_kernel(const float* __restrict__ part, int P, int64_t ld, float* __restrict__ rstd,
                                                                int64_t T, int D, float eps) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= T) return;
  float ss = 0.0f;
  for (int j = 0; j < P; ++j) ss += part[j * ld + row];                        // fixed order: run-to-run identical
  rstd[row] = rsqrtf(ss / (float)D + eps);
}
__global__ __launch_bounds__(256) void fold_gain_kernel(const bf16* __restrict__ W, const bf16* __restrict__ g, bf16* __restrict__ out,
                                                        int64_t n8, int K) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;                  // one thread per 8 consecutive k
  if (i >= n8) return;
  const int k = (int)((i * 8) % K);
  float w[8], gv[8], o[8];
  load8(W + i * 8, w); load8(g + k, gv);
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = w[j] * gv[j];
  store8(out + i * 8, o);
}

// out = dres + J_norm(x)^T dn.  RMS: gd/r - x * sum(gd*x) / (D r^3).  LN: (gd - mean(gd) - xh*mean(gd*xh)) / sd.
template <typename E>
__global__ __launch_bounds__(256) void norm_bwd_add_kernel(const E* __restrict__ dn, const E* __restrict__ x, const E* __restrict__ g,
                                                           const E* __restrict__ dres, E* __restrict__ out, int D, int kind, float eps) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const E* xr = x + row * D; const E* dr = dn + row * D; const E* rr = dres + row * D;
  E* orow = out + row * D;
  float mean = 0.0f;
  if (kind == SV_NORM_LN) {
    float s = 0.0f;
    for (int k = threadIdx.x * 8; k < D; k += 2048) { float v[8]; load8(xr + k, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) s += v[j]; }
    mean = block_sum_256(s, red) / (float)D;
  }
  float ss = 0.0f;
  for (int k = threadIdx.x * 8; k < D; k += 2048) { float v[8]; load8(xr + k, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float d = v[j] - mean; ss += d * d; } }
  const float rinv = rsqrtf(block_sum_256(ss, red) / (float)D + eps);
  float s1 = 0.0f, s2 = 0.0f;   // sum gd, sum gd * xhat
  for (int k = threadIdx.x * 8; k < D; k += 2048) {
    float v[8], gv[8], dv[8];
    load8(xr + k, v); load8(g + k, gv); load8(dr + k, dv);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float gd = gv[j] * dv[j]; s1 += gd; s2 += gd * (v[j] - mean) * rinv; }
  }
  s1 = block_sum_256(s1, red) / (float)D;
  s2 = block_sum_256(s2, red) / (float)D;
  if (kind != SV_NORM_LN) s1 = 0.0f;
  for (int k = threadIdx.x * 8; k < D; k += 2048) {
    float v[8], gv[8], dv[8], rv[8], o[8];
    load8(xr + k, v); load8(g + k, gv); load8(dr + k, dv); load8(rr + k, rv);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float xh = (v[j] - mean) * rinv;
      o[j] = rv[j] + (gv[j] * dv[j] - s1 - xh * s2) * rinv;
    }
    store8(orow + k, o);
  }
}

// ------------------------------------------------------------------------------------ RoPE
template <typename E>
__global__ __launch_bounds__(256) void rope_kernel(E* __restrict__ qkv, int64_t ld, int64_t T, int S, int n_heads_total, int hd,
                                                   const float* __restrict__ cs, float sign) {
  const int half = hd >> 1;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_tok = (int64_t)n_heads_total * half;
  if (idx >= T * per_tok) return;
  const int64_t t = idx / per_tok;
  const int rem = (int)(idx - t * per_tok);
  const int head = rem / half, i = rem - head * half;
  const int p = (int)(t % S);
  const float c = cs[((int64_t)p * half + i) * 2], s = sign * cs[((int64_t)p * half + i) * 2 + 1];
  E* ptr = qkv + t * ld + (int64_t)head * hd + 2 * i;     // q heads then k heads are contiguous in a row
  const float a = to_f32(ptr[0]), b = to_f32(ptr[1]);
  ptr[0] = from_f32<E>(a * c - b * s);
  ptr[1] = from_f32<E>(a * s + b * c);
}

// ------------------------------------------------------------------------------------ attention
// 64 queries per workgroup, 4 threads per query each owning HD/4 of the head dimension;
// keys/values stream through LDS in tiles of 32 rows; softmax is the running (online) form.
constexpr int kKT = 32;

template <typename E, int HD>
__global__ __launch_bounds__(256) void attn_fwd_plain_kernel(const E* __restrict__ qkv, int64_t ld, E* __restrict__ o, float* __restrict__ lse,
                                                             int S, int H, int Hkv, int causal) {
  constexpr int DPT = HD / 4;
  __shared__ float Ks[kKT][HD];
  __shared__ float Vs[kKT][HD];
  const int h = blockIdx.y, b = blockIdx.z, kvh = h / (H / Hkv);
  const int qi = blockIdx.x * 64 + (threadIdx.x >> 2), part = threadIdx.x & 3;
  const bool valid = qi < S;
  const int Dq = H * HD, Dkv = Hkv * HD;
  const float scale = rsqrtf((float)HD);
  const E* qrow = qkv + (int64_t)(b * S + (valid ? qi : S - 1)) * ld + h * HD + part * DPT;
  float q[DPT], acc[DPT];
#pragma unroll
  for (int d = 0; d < DPT; ++d) { q[d] = to_f32(qrow[d]) * scale; acc[d] = 0.0f; }
  float m = -INFINITY, l = 0.0f;
  const int kend = causal ? min(S, (int)blockIdx.x * 64 + 64) : S;
  for (int k0 = 0; k0 < kend; k0 += kKT) {
    __syncthreads();
    for (int e = threadIdx.x; e < kKT * HD; e += 256) {
      const int r = e / HD, d = e - r * HD;
      const bool ok = k0 + r < S;
      const E* row = qkv + (int64_t)(b * S + (ok ? k0 + r : 0)) * ld + Dq + kvh * HD + d;
      Ks[r][d] = ok ? to_f32(row[0]) : 0.0f;
      Vs[r][d] = ok ? to_f32(row[Dkv]) : 0.0f;
    }
    __syncthreads();
    const int jmax = (causal ? min(qi + 1, S) : S) - k0;
    for (int j = 0; j < kKT; ++j) {
      float s = 0.0f;
#pragma unroll
      for (int d = 0; d < DPT; ++d) s = fmaf(q[d], Ks[j][part * DPT + d], s);
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      if (valid && j < jmax) {
        if (s > m) {
          const float c = expf(m - s);
          l *= c;
#pragma unroll
          for (int d = 0; d < DPT; ++d) acc[d] *= c;
          m = s;
        }
        const float p = expf(s - m);
        l += p;
#pragma unroll
        for (int d = 0; d < DPT; ++d) acc[d] = fmaf(p, Vs[j][part * DPT + d], acc[d]);
      }
    }
  }
  if (valid) {
    E* orow = o + (int64_t)(b * S + qi) * Dq + h * HD + part * DPT;
    const float inv = 1.0f / l;
#pragma unroll
    for (int d = 0; d < DPT; ++d) orow[d] = from_f32<E>(acc[d] * inv);
    if (part == 0) lse[((int64_t)b * H + h) * S + qi] = m + logf(l);
  }
}

// dq (and delta = rowsum(do * o)) for 64 queries per workgroup.
template <typename E, int HD>
__global__ __launch_bounds__(256) void attn_bwd_dq_plain_kernel(const E* __restrict__ qkv, int64_t ld, const E* __restrict__ o,
                                                                const E* __restrict__ dout, const float* __restrict__ lse,
                                                                float* __restrict__ delta, E* __restrict__ dqkv, int S, int H, int Hkv,
                                                                int causal) {
  constexpr int DPT = HD / 4;
  __shared__ float Ks[kKT][HD];
  __shared__ float Vs[kKT][HD];
  const int h = blockIdx.y, b = blockIdx.z, kvh = h / (H / Hkv);
  const int qi = blockIdx.x * 64 + (threadIdx.x >> 2), part = threadIdx.x & 3;
  const bool valid = qi < S;
  const int Dq = H * HD, Dkv = Hkv * HD;
  const float scale = rsqrtf((float)HD);
  const int64_t tok = (int64_t)b * S + (valid ? qi : S - 1);
  const E* qrow = qkv + tok * ld + h * HD + part * DPT;
  const E* orow = o + tok * Dq + h * HD + part * DPT;
  const E* drow = dout + tok * Dq + h * HD + part * DPT;
  float q[DPT], dov[DPT], dq[DPT];
  float dl = 0.0f;
#pragma unroll
  for (int d = 0; d < DPT; ++d) {
    q[d] = to_f32(qrow[d]) * scale; dov[d] = to_f32(drow[d]); dq[d] = 0.0f;
    dl = fmaf(dov[d], to_f32(orow[d]), dl);
  }
  dl += __shfl_xor(dl, 1, 64);
  dl += __shfl_xor(dl, 2, 64);
  const int64_t li = ((int64_t)b * H + h) * S + (valid ? qi : S - 1);
  const float L = lse[li];
  if (valid && part == 0) delta[li] = dl;
  const int kend = causal ? min(S, (int)blockIdx.x * 64 + 64) : S;
  for (int k0 = 0; k0 < kend; k0 += kKT) {
    __syncthreads();
    for (int e = threadIdx.x; e < kKT * HD; e += 256) {
      const int r = e / HD, d = e - r * HD;
      const bool ok = k0 + r < S;
      const E* row = qkv + (int64_t)(b * S + (ok ? k0 + r : 0)) * ld + Dq + kvh * HD + d;
      Ks[r][d] = ok ? to_f32(row[0]) : 0.0f;
      Vs[r][d] = ok ? to_f32(row[Dkv]) : 0.0f;
    }
    __syncthreads();
    const int jmax = (causal ? min(qi + 1, S) : S) - k0;
    for (int j = 0; j < kKT; ++j) {
      float s = 0.0f, dp = 0.0f;
#pragma unroll
      for (int d = 0; d < DPT; ++d) { s = fmaf(q[d], Ks[j][part * DPT + d], s); dp = fmaf(dov[d], Vs[j][part * DPT + d], dp); }
      s += __shfl_xor(s, 1, 64);  dp += __shfl_xor(dp, 1, 64);
      s += __shfl_xor(s, 2, 64);  dp += __shfl_xor(dp, 2, 64);
      if (valid && j < jmax) {
        const float ds = expf(s - L) * (dp - dl) * scale;
#pragma unroll
        for (int d = 0; d < DPT; ++d) dq[d] = fmaf(ds, Ks[j][part * DPT + d], dq[d]);
      }
    }
  }
  if (valid) {
    E* out = dqkv + ((int64_t)b * S + qi) * ld + h * HD + part * DPT;
#pragma unroll
    for (int d = 0; d < DPT; ++d) out[d] = from_f32<E>(dq[d]);
  }
}

// dk, dv for 64 keys per workgroup, summed over the query heads of the kv head's group.
constexpr int kQT = 16;
template <typename E, int HD>
__global__ __launch_bounds__(256) void attn_bwd_dkv_plain_kernel(const E* __restrict__ qkv, int64_t ld, const E* __restrict__ dout,
                                                                 const float* __restrict__ lse, const float* __restrict__ delta,
                                                                 E* __restrict__ dqkv, int S, int H, int Hkv, int causal) {
  constexpr int DPT = HD / 4;
  __shared__ float Qs[kQT][HD];
  __shared__ float Ds[kQT][HD];
  __shared__ float Ls[kQT], Dl[kQT];
  const int kvh = blockIdx.y, b = blockIdx.z, G = H / Hkv;
  const int kj = blockIdx.x * 64 + (threadIdx.x >> 2), part = threadIdx.x & 3;
  const bool valid = kj < S;
  const int Dq = H * HD, Dkv = Hkv * HD;
  const float scale = rsqrtf((float)HD);
  const E* krow = qkv + (int64_t)(b * S + (valid ? kj : S - 1)) * ld + Dq + kvh * HD + part * DPT;
  float k[DPT], v[DPT], dk[DPT], dv[DPT];
#pragma unroll
  for (int d = 0; d < DPT; ++d) { k[d] = to_f32(krow[d]) * scale; v[d] = to_f32(krow[Dkv + d]); dk[d] = 0.0f; dv[d] = 0.0f; }
  const int qstart = causal ? ((int)blockIdx.x * 64 / kQT) * kQT : 0;
  for (int g = 0; g < G; ++g) {
    const int h = kvh * G + g;
    for (int q0 = qstart; q0 < S; q0 += kQT) {
      __syncthreads();
      for (int e = threadIdx.x; e < kQT * HD; e += 256) {
        const int r = e / HD, d = e - r * HD;
        const bool ok = q0 + r < S;
        const int64_t tok = (int64_t)b * S + (ok ? q0 + r : 0);
        Qs[r][d] = ok ? to_f32(qkv[tok * ld + h * HD + d]) : 0.0f;
        Ds[r][d] = ok ? to_f32(dout[tok * Dq + h * HD + d]) : 0.0f;
      }
      if (threadIdx.x < kQT) {
        const bool ok = q0 + (int)threadIdx.x < S;
        const int64_t li = ((int64_t)b * H + h) * S + (ok ? q0 + threadIdx.x : 0);
        Ls[threadIdx.x] = ok ? lse[li] : 0.0f;
        Dl[threadIdx.x] = ok ? delta[li] : 0.0f;
      }
      __syncthreads();
      for (int i = 0; i < kQT; ++i) {
        float s = 0.0f, dp = 0.0f;
#pragma unroll
        for (int d = 0; d < DPT; ++d) { s = fmaf(k[d], Qs[i][part * DPT + d], s); dp = fmaf(v[d], Ds[i][part * DPT + d], dp); }
        s += __shfl_xor(s, 1, 64);  dp += __shfl_xor(dp, 1, 64);
        s += __shfl_xor(s, 2, 64);  dp += __shfl_xor(dp, 2, 64);
        const int qi = q0 + i;
        if (valid && qi < S && (!causal || qi >= kj)) {
          const float p = expf(s - Ls[i]);
          const float ds = p * (dp - Dl[i]) * scale;
#pragma unroll
          for (int d = 0; d < DPT; ++d) {
            dv[d] = fmaf(p, Ds[i][part * DPT + d], dv[d]);
            dk[d] = fmaf(ds, Qs[i][part * DPT + d], dk[d]);
          }
        }
      }
    }
  }
  if (valid) {
    E* out = dqkv + ((int64_t)b * S + kj) * ld + Dq + kvh * HD + part * DPT;
#pragma unroll
    for (int d = 0; d < DPT; ++d) { out[d] = from_f32<E>(dk[d]); out[Dkv + d] = from_f32<E>(dv[d]); }
  }
}

// ------------------------------------------------------------------------------------ transpose
// dst[c][r] = src[r][c] for a row-major [R, C] matrix: 64x64 tiles through LDS (row pitch 65).
template <typename E>
__global__ __launch_bounds__(256) void transpose_kernel(const E* __restrict__ src, E* __restrict__ dst, int R, int C) {
  __shared__ E tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4)
    if (r0 + i < R && c0 + tx < C) tile[i][tx] = src[(int64_t)(r0 + i) * C + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 64; i += 4)
    if (c0 + i < C && r0 + tx < R) dst[(int64_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

// Head-dimension padding for the matrix-core attention kernels: [T, n_heads * hd] <-> [T, n_heads * hd_pad], bf16, 8 elements per
// thread.  widen: the columns hd .. hd_pad of every head are zero.
__global__ __launch_bounds__(256) void pad_heads_kernel(const bf16* __restrict__ src, int64_t ld_src, bf16* __restrict__ dst, int64_t ld_dst,
                                                        int64_t T, int n_heads, int hd, int hd_pad, int widen) {
  const int cp = hd_pad / 8, cs = hd / 8;                         // 16-byte chunks per head
  const int per_row = n_heads * (widen ? cp : cs);
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= T * per_row) return;
  const int64_t t = i / per_row;
  const int r = (int)(i % per_row), h = r / (widen ? cp : cs), c = r % (widen ? cp : cs);
  bf16x8 v;
#pragma unroll
  for (int k = 0; k < 8; ++k) v[k] = (bf16)0.0f;
  if (widen) {
    if (c < cs) v = *reinterpret_cast<const bf16x8*>(src + t * ld_src + h * hd + c * 8);
    *reinterpret_cast<bf16x8*>(dst + t * ld_dst + h * hd_pad + c * 8) = v;
  } else {
    v = *reinterpret_cast<const bf16x8*>(src + t * ld_src + h * hd_pad + c * 8);
    *reinterpret_cast<bf16x8*>(dst + t * ld_dst + h * hd + c * 8) = v;
  }
}

}  // namespace

hipError_t plain_pad_heads(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int n_heads, int hd, int hd_pad, int widen,
                           hipStream_t st) {
  if (T <= 0 || n_heads <= 0) return hipSuccess;
  if (hd % 8 || hd_pad % 8 || hd > hd_pad || ld_src % 8 || ld_dst % 8) return hipErrorInvalidValue;
  const int64_t n = T * n_heads * ((widen ? hd_pad : hd) / 8);
  hipLaunchKernelGGL(pad_heads_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const bf16*)src, ld_src, (bf16*)dst, ld_dst, T,
                     n_heads, hd, hd_pad, widen);
  return hipGetLastError();
}

hipError_t plain_transpose(const void* src, void* dst, int R, int C, int dtype, hipStream_t st) {
  if (R <= 0 || C <= 0) return hipSuccess;
  const dim3 grid((C + 63) / 64, (R + 63) / 64), block(256);
  if (dtype == SV_BF16) hipLaunchKernelGGL(transpose_kernel<bf16>, grid, block, 0, st, (const bf16*)src, (bf16*)dst, R, C);
  else hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, st, (const float*)src, (float*)dst, R, C);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------ launchers
hipError_t plain_gemm(const GemmArgs& a, int dtype, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  const dim3 grid((a.N + 63) / 64, (a.M + 63) / 64), block(256);
  const bool dual = a.epi == EPI_SWIGLU;
  if (dtype == SV_BF16) {
    if (dual) hipLaunchKernelGGL((gemm_plain_kernel<bf16, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((gemm_plain_kernel<bf16, false>), grid, block, 0, st, a);
  } else {
    if (dual) hipLaunchKernelGGL((gemm_plain_kernel<float, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((gemm_plain_kernel<float, false>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

hipError_t plain_norm_fwd(const void* x, const void* g, const void* b, void* out, int64_t T, int D, int kind, float eps, int dtype,
                          hipStream_t st) {
  if (T <= 0) return hipSuccess;
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(norm_fwd_kernel<bf16>, dim3((unsigned)T), dim3(256), 0, st, (const bf16*)x, (const bf16*)g, (const bf16*)b, (bf16*)out, D, kind, eps);
  else
    hipLaunchKernelGGL(norm_fwd_kernel<float>, dim3((unsigned)T), dim3(256), 0, st, (const float*)x, (const float*)g, (const float*)b, (float*)out, D, kind, eps);
  return hipGetLastError();
}

hipError_t rms_rstd(const void* x, float* rstd, int64_t T, int D, float eps, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  if (D % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rms_rstd_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, st, (const bf16*)x, rstd, T, D, eps);
  return hipGetLastError();
}
hipError_t rms_rstd_from_partials(const float* part, int P, int64_t ld, float* rstd, int64_t T, int D, float eps, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  hipLaunchKernelGGL(rms_rstd_partials_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, part, P, ld, rstd, T, D, eps);
  return hipGetLastError();
}
hipError_t fold_gain(const void* W, const void* g, void* out, int64_t N, int K, hipStream_t st) {
  if (N <= 0) return hipSuccess;
  if (K % 8) return hipErrorInvalidValue;
  const int64_t n8 = N * K / 8;
  hipLaunchKernelGGL(fold_gain_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st, (const bf16*)W, (const bf16*)g, (bf16*)out, n8, K);
  return hipGetLastError();
}

hipError_t plain_norm_bwd_add(const void* dn, const void* x, const void* g, const void* dres, void* out, int64_t T, int D, int kind,
                              float eps, int dtype, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  if (dtype == SV_BF16)
    hipLaunchKernelGGL(norm_bwd_add_kernel<bf16>, dim3((unsigned)T), dim3(256), 0, st, (const bf16*)dn, (const bf16*)x, (const bf16*)g, (const bf16*)dres, (bf16*)out, D, kind, eps);
  else
    hipLaunchKernelGGL(norm_bwd_add_kernel<float>, dim3((unsigned)T), dim3(256), 0, st, (const float*)dn, (const float*)x, (const float*)g, (const float*)dres, (float*)out, D, kind, eps);
  return hipGetLastError();
}

hipError_t plain_rope(void* qkv, int64_t ld, int64_t T, int S, int n_q_heads, int n_kv_heads, int hd, const float* cs_table, int inverse,
                      int dtype, hipStream_t st) {
  const int heads = n_q_heads + n_kv_heads;
  const int64_t n = T * heads * (hd / 2);
  if (n <= 0) return hipSuccess;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  const float sign = inverse ? -1.0f : 1.0f;
  if (dtype == SV_BF16) hipLaunchKernelGGL(rope_kernel<bf16>, grid, block, 0, st, (bf16*)qkv, ld, T, S, heads, hd, cs_table, sign);
  else hipLaunchKernelGGL(rope_kernel<float>, grid, block, 0, st, (float*)qkv, ld, T, S, heads, hd, cs_table, sign);
  return hipGetLastError();
}

#define SV_HD_DISPATCH(HDV, CALL)            \
  switch (HDV) {                             \
    case 8: { constexpr int HD = 8; CALL; } break;     \
    case 16: { constexpr int HD = 16; CALL; } break;   \
    case 32: { constexpr int HD = 32; CALL; } break;   \
    case 64: { constexpr int HD = 64; CALL; } break;   \
    case 128: { constexpr int HD = 128; CALL; } break; \
    default: return hipErrorInvalidValue;    \
  }

hipError_t plain_attn_fwd(const void* qkv, int64_t ld, void* o, float* lse, int B, int S, int H, int Hkv, int hd, int causal, int dtype,
                          hipStream_t st) {
  if (B <= 0 || S <= 0) return hipSuccess;
  const dim3 grid((S + 63) / 64, H, B), block(256);
  if (dtype == SV_BF16) {
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_fwd_plain_kernel<bf16, HD>), grid, block, 0, st, (const bf16*)qkv, ld, (bf16*)o, lse, S, H, Hkv, causal))
  } else {
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_fwd_plain_kernel<float, HD>), grid, block, 0, st, (const float*)qkv, ld, (float*)o, lse, S, H, Hkv, causal))
  }
  return hipGetLastError();
}

hipError_t plain_attn_bwd(const void* qkv, int64_t ld, const void* o, const void* dout, const float* lse, float* delta, void* dqkv, int B,
                          int S, int H, int Hkv, int hd, int causal, int dtype, hipStream_t st) {
  if (B <= 0 || S <= 0) return hipSuccess;
  const dim3 gq((S + 63) / 64, H, B), gk((S + 63) / 64, Hkv, B), block(256);
  if (dtype == SV_BF16) {
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_bwd_dq_plain_kernel<bf16, HD>), gq, block, 0, st, (const bf16*)qkv, ld, (const bf16*)o, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, H, Hkv, causal))
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_bwd_dkv_plain_kernel<bf16, HD>), gk, block, 0, st, (const bf16*)qkv, ld, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, H, Hkv, causal))
  } else {
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_bwd_dq_plain_kernel<float, HD>), gq, block, 0, st, (const float*)qkv, ld, (const float*)o, (const float*)dout, lse, delta, (float*)dqkv, S, H, Hkv, causal))
    SV_HD_DISPATCH(hd, hipLaunchKernelGGL((attn_bwd_dkv_plain_kernel<float, HD>), gk, block, 0, st, (const float*)qkv, ld, (const float*)dout, lse, delta, (float*)dqkv, S, H, Hkv, causal))
  }
  return hipGetLastError();
}

}  // namespace sv
