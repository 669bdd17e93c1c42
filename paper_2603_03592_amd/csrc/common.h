// Shared device helpers for the stage-verifier kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stageverify.h"

namespace sv {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
template <typename E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return static_cast<bf16>(v); }  // RNE

// 8 consecutive elements (16-byte aligned for bf16, 32-byte for float) as floats.
__device__ __forceinline__ void load8(const bf16* p, float (&o)[8]) {
  bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = static_cast<float>(v[i]);
}
__device__ __forceinline__ void load8(const float* p, float (&o)[8]) {
  f32x4 a = *reinterpret_cast<const f32x4*>(p);
  f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = static_cast<bf16>(v[i]);
  *reinterpret_cast<bf16x8*>(p) = o;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  f32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Workgroup barrier that orders LDS accesses only: waits for this wave's LDS operations, then s_barrier.  Unlike
// __syncthreads() it does not wait for global loads in flight (a workgroup fence drains the vector memory counter),
// so loads prefetched into registers stay in flight across it.  Use only where nothing but LDS is shared between waves.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Sum over a 256-thread workgroup; every thread gets the result.  `red` holds >= 4 floats.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// sigmoid through the hardware reciprocal (1 ulp) instead of a full-precision division (ten instructions): the SiLU
// epilogues evaluate it for every output element, which at small K is a visible share of a GEMM tile's time
__device__ __forceinline__ float sigmoid_fast_f(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_fast_f(z); }
__device__ __forceinline__ float silu_grad_f(float z) {
  const float s = sigmoid_fast_f(z);
  return s * (1.0f + z * (1.0f - s));
}
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
  return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * __expf(-0.5f * z * z) * 0.39894228040143268f;
}

}  // namespace sv

// ----------------------------------------------------------------------------------------
// Host-side launch interfaces between the translation units (all enqueue on `st`).
namespace sv {

struct ScorePartial {   // per (claim, token tile)
  double s[8];          // sum c, sum r, sum c^2, sum r^2, sum d, sum |d|, sum d^2, #sign mismatches
  float max_rel;        // max over the tile's tokens of the per-token relative L2
  int32_t argmax;       // token index of that maximum (lowest on ties)
  int32_t bad;          // a non-finite per-token value was seen
  int32_t pad;
};
constexpr int kScoreTokensPerWG = 16;

// score.hip
hipError_t launch_score(const void* claims, int64_t claim_stride, int n_claims, const void* ref, int64_t ref_stride,
                        int claim_dtype, int ref_dtype, int64_t T, int D, uint32_t mask, const float* tau4,
                        int reduce, float* token_scores, sv_result* results, ScorePartial* scratch,
                        int64_t scratch_elems, hipStream_t st, uint32_t skip = 0, float* sum_out = nullptr);
// api.hip: error text for entry points without a context (sv_last_error(NULL) returns it on the same thread)
void set_global_error(const char* fmt, ...);
// With sum_out the score pass also writes sum_out[t, :] = sum of the submissions whose bit in `skip` is clear (fp32, index
// order); only for the cases score_sum_supported names (one shared reference, at most 32 submissions, rows of a multiple of 2 KB).
bool score_sum_supported(int n_claims, int64_t ref_stride, int claim_dtype, int D);
hipError_t launch_ema_from_sum(float* m, const float* sum, int n_summed, int64_t T, int D, float beta, hipStream_t st);
hipError_t launch_ema(float* m, const void* claims, int64_t claim_stride, int n_claims, int claim_dtype,
                      const uint8_t* flags, int64_t T, int D, float beta, hipStream_t st);

hipError_t launch_replace(void* signals, int64_t stride, int n, int dtype, const uint8_t* mask, const float* m, int64_t T, int D,
                          hipStream_t st);

// sw.hip: sliced Wasserstein.  P holds rows of Tpad = sw_padded_len(T) floats, L rows per tensor.
int64_t sw_padded_len(int64_t T);
hipError_t launch_sw_project(const void* X, int64_t stride, int count, int dtype, const void* U, int L, int D, int64_t T, int64_t Tpad,
                             float* P, hipStream_t st);
// One launch for a single reference tensor (into Pref) and `count` submissions (into P); only for the dtype pairs
// sw_project_with_ref_supported names.
bool sw_project_with_ref_supported(int dtype, int ref_dtype);
hipError_t launch_sw_project_with_ref(const void* X, int64_t stride, int count, int dtype, const void* ref, int ref_dtype, const void* U,
                                      int L, int D, int64_t T, int64_t Tpad, float* P, float* Pref, hipStream_t st);
// Sort n_seg rows; with ref != nullptr also w1[first_seg + s] = sum_t |row_s[t] - ref_row[t]| (ref rows already sorted).
hipError_t launch_sw_sort(float* P, int n_seg, int64_t T, int64_t Tpad, const float* ref, int ref_shared, int L, float* w1,
                          int first_seg, hipStream_t st);
hipError_t launch_sw_copy_pad(float* dst, const float* src, int L, int64_t T, int64_t Tpad, hipStream_t st);
hipError_t launch_sw_proj_ema(float* pm, const float* P, int n, uint32_t skip, int L, int64_t T, int64_t Tpad, float beta, float w,
                              hipStream_t st);
constexpr int64_t kSwSortChunkMax = 16384;   // longest row one workgroup sorts in LDS (longer rows are sorted in place in global memory)
hipError_t launch_sw_finalize(const float* w1, int n_claims, int L, int64_t T, float tau, float* sw_out, sv_result* results,
                              hipStream_t st);

// One K-segment of a (possibly multi-segment) product  C = sum_seg A_seg * op(B_seg).
struct GemmSeg {
  const void* A; int64_t lda;   // [M, K] row-major
  const void* B; int64_t ldb;   // NT: [N, K] row-major;  NN: [K, N] row-major
  int K;
};
enum EpiMode {
  EPI_STORE = 0,        // C = acc
  EPI_RESID = 1,        // C = acc + R
  EPI_GELU = 2,         // C = gelu(acc); if C2: C2 = acc (pre-activation)
  EPI_SWIGLU = 3,       // dual product (B, B2): C = silu(g) * u; if C2/C3: C2 = g, C3 = u
  EPI_SWIGLU_BWD = 4,   // da = acc: C = da * U * silu'(G), C2 = da * silu(G)   (G = R, U = R2)
  EPI_GELU_BWD = 5,     // C = acc * gelu'(R)
  EPI_ROPE = 6          // C = acc with columns < rope_cols rotated pairwise by the RoPE angle of token (row % rope_S)
};
struct GemmArgs {
  int M, N;               // output [M, N]
  int nseg; GemmSeg seg[3];
  const void* B2; int64_t ldb2;   // second weight of the dual product (EPI_SWIGLU), same shape as seg[0].B
  int b_is_kn;            // 0: NT (B stored [N,K]);  1: NN (B stored [K,N])
  int epi;
  void* C; int64_t ldc;
  void* C2; void* C3;     // same leading dimension as C
  const void* R; const void* R2; int64_t ldr;
  // optional: output columns split over up to 3 weight matrices (single K segment, [N,K] weights):
  // columns [0, ncol[0]) use Bcol[0], the next ncol[1] use Bcol[1], ... (all with leading dimension seg[0].ldb)
  int nbcol; const void* Bcol[3]; int ncol[3];
  // EPI_ROPE: (cos, sin) table [rope_S][rope_hd / 2][2] of floats
  const float* rope_cs; int rope_S, rope_hd, rope_cols;
  // optional grouped form (mixture of experts): rows [256 i, 256 i + 256) of the product use the weight matrices of
  // group tile_group[i], found group_stride elements apart behind every seg[].B and B2; with m_dev the row count is
  // read from device memory (*m_dev <= M, a multiple of 256) and M only bounds the launch
  const int32_t* tile_group; int64_t group_stride;
  const int32_t* m_dev;
  // optional: fp32 scratch for split-k partial products (small row counts against a long k); none = never split
  float* split_ws; int64_t split_ws_floats;
  // optional, the two ends of an RMSNorm that runs inside its neighbouring products (its gain folded into the weights of
  // the product that follows):
  //   rscale: row m of the accumulators is multiplied by rscale[m] -- the row's 1 / rms -- before the epilogue's own
  //           function (EPI_STORE, EPI_GELU, EPI_SWIGLU, EPI_ROPE)
  //   rowsq : EPI_RESID on the 256 x 256 direct-to-LDS kernel (mfma_gemm_emits_rowsq) also writes, for every row m and
  //           every 128 columns j, rowsq[j * rowsq_ld + m] = the sum of squares of the 128 values it stored (rowsq_ld >= M)
  const float* rscale;
  float* rowsq; int rowsq_ld;
};

// kernels_plain.hip: any shape, fp32 math, E = float | bf16 by `dtype`
hipError_t plain_gemm(const GemmArgs& a, int dtype, hipStream_t st);
hipError_t plain_norm_fwd(const void* x, const void* g, const void* b, void* out, int64_t T, int D, int kind, float eps,
                          int dtype, hipStream_t st);
// RMSNorm in pieces, bf16 rows: rstd[t] = 1 / sqrt(mean_k x[t][k]^2 + eps) straight from the rows, or from the P partial sums of
// squares per row that a product's epilogue left (GemmArgs::rowsq: P planes of ld floats); out[n][k] = W[n][k] * g[k] folds the gain into the [N, K]
// weights of the product that follows the norm
hipError_t rms_rstd(const void* x, float* rstd, int64_t T, int D, float eps, hipStream_t st);
hipError_t rms_rstd_from_partials(const float* part, int P, int64_t ld, float* rstd, int64_t T, int D, float eps, hipStream_t st);
hipError_t fold_gain(const void* W, const void* g, void* out, int64_t N, int K, hipStream_t st);
// out = dres + d/dx [ Norm(x) ] applied to dn
hipError_t plain_norm_bwd_add(const void* dn, const void* x, const void* g, const void* dres, void* out, int64_t T, int D,
                              int kind, float eps, int dtype, hipStream_t st);
// in-place rotation of the q and k parts of qkv [T, ld]; positions = token index mod S
hipError_t plain_rope(void* qkv, int64_t ld, int64_t T, int S, int n_q_heads, int n_kv_heads, int hd, const float* cs_table,
                      int inverse, int dtype, hipStream_t st);
hipError_t plain_attn_fwd(const void* qkv, int64_t ld, void* o, float* lse, int B, int S, int H, int Hkv, int hd, int causal,
                          int dtype, hipStream_t st);
hipError_t plain_attn_bwd(const void* qkv, int64_t ld, const void* o, const void* dout, const float* lse, float* delta,
                          void* dqkv, int B, int S, int H, int Hkv, int hd, int causal, int dtype, hipStream_t st);

hipError_t plain_transpose(const void* src, void* dst, int R, int C, int dtype, hipStream_t st);
// bf16 [T, n_heads * hd] (row stride ld_src) -> [T, n_heads * hd_pad] with zero columns (widen = 1), or back (widen = 0:
// src has hd_pad columns per head, dst hd); hd, hd_pad and the strides are multiples of 8
hipError_t plain_pad_heads(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int n_heads, int hd, int hd_pad, int widen,
                           hipStream_t st);

// moe.hip: routing of a mixture-of-experts MLP.  All buffers are device memory of one block.
constexpr int kMoeMaxExperts = 16, kMoeMaxTopK = 8, kMoeChunk = 1024;
struct MoeRoute {
  int32_t* sel;          // [T, K] chosen experts, decreasing score
  float* gate;           // [T, K] their weights
  float* score;          // [T, E] router scores
  int32_t* pos;          // [T, K] row of (token, choice) in the expert-sorted buffers
  int32_t* row_token;    // [Mp]   token of a row (rows of one expert are contiguous, padded to a multiple of 256)
  float* row_gate;       // [Mp]   gate of a row
  int32_t* tile_expert;  // [Mp / 256] expert of each 256-row block
  int32_t* meta;         // [0] rows in use (multiple of 256), [1 + e] first row of expert e, [1 + E + e] its row count
  int32_t* chunk_counts; // [n_chunks, E] scratch of the counting sort, n_chunks = ceil(T K / kMoeChunk)
  int32_t* chunk_base;   // [n_chunks, E]
};
int64_t moe_padded_rows(int64_t T, int K, int E);   // upper bound Mp of the rows in use
hipError_t launch_moe_route(const void* n, const void* w_router, int64_t T, int D, int E, int K, int score_kind, int norm, int dtype,
                            const MoeRoute& r, hipStream_t st);
// dst[p, :] = scale_p * src[row_token[p], :] for the rows in use (zeros for padding rows); scale_p = row_gate[p] if scaled
hipError_t launch_moe_gather(const void* src, int D, int64_t Mp, int E, const MoeRoute& r, int scaled, void* dst, int dtype, hipStream_t st);
// y[t, :] = base[t, :] + sum_j gate[t, j] * yp[pos[t, j], :]      (y may alias base)
hipError_t launch_moe_combine(const void* base, const void* yp, int64_t T, int D, int K, const MoeRoute& r, void* y, int dtype, hipStream_t st);
// dn[t, :] = (accumulate ? dn[t, :] : 0) + sum_j dxp[pos[t, j], :] + sum_e dlogit[t, e] Wr[e, :], where dlogit follows
// from dgate[t, j] = <dy[t, :], yp[pos[t, j], :]> through the gate normalisation and the score function
hipError_t launch_moe_combine_bwd(const void* dy, const void* yp, const void* dxp, const void* w_router, int64_t T, int D, int E, int K,
                                  int score_kind, int norm, const MoeRoute& r, int accumulate, void* dn, int dtype, hipStream_t st);

// gemm_mfma.hip: bf16 only; returns hipErrorInvalidValue if the shape is outside its limits
bool mfma_gemm_supported(const GemmArgs& a);
bool mfma_gemm_emits_rowsq(const GemmArgs& a);          // would mfma_gemm(a, st) fill a.rowsq?
hipError_t mfma_gemm(const GemmArgs& a, hipStream_t st, int tile = 0);   // tile: 0 auto, 1 = 256x256, 2 = 128x128

// attn_mfma.hip: bf16, head_dim 64 | 128.  scale_hd (0 = hd): the head dimension the softmax scale 1/sqrt(.) is taken from,
// for inputs whose heads were zero-padded from scale_hd to hd columns
bool mfma_attn_supported(int S, int H, int Hkv, int hd, int64_t ld);
hipError_t mfma_attn_fwd(const void* qkv, int64_t ld, void* o, float* lse, int B, int S, int H, int Hkv, int hd, int causal,
                         hipStream_t st, int scale_hd = 0);
// the dk / dv kernel gives every query head of a group its own workgroup when one workgroup per (batch, kv head, key
// tile of 64 -- two tiles under the causal mask) would be fewer than this many: two per CU
constexpr int kDkvSplitWorkgroups = 512;
// rope_cs != nullptr: dq and dk are rotated back (inverse RoPE) before they are stored.  part_ws: optional fp32 scratch of
// part_floats floats; with G * B * S * 2 * Hkv * hd of them and few (batch, kv head, key tile) triples the dk / dv kernel
// runs one workgroup per query head and a second kernel adds each group's heads in a fixed order
hipError_t mfma_attn_bwd(const void* qkv, int64_t ld, const void* o, const void* dout, const float* lse, float* delta, void* dqkv,
                         int B, int S, int H, int Hkv, int hd, int causal, const float* rope_cs, hipStream_t st, int scale_hd = 0,
                         float* part_ws = nullptr, int64_t part_floats = 0);

}  // namespace sv
