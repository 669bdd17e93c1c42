// bf16 GEMMs of the block recompute on the gfx950 matrix cores.
//
//   C[M,N] = sum_seg A_seg[M,K_seg] * op(B_seg)   fp32 accumulation, fused epilogue
//
// op(B) = B^T with B stored [N,K] (forward: activations times [out,in] weights) or B stored
// [K,N] (backward: gradients times the same [out,in] weights, contraction over "out").
//
// Kernel shape: a BM x BN output tile per workgroup, K walked in slices of 64.  Both operand
// slices are staged in LDS as rows of 64 bf16 (128 bytes) whose eight 16-byte chunks are
// XOR-swizzled by the row index, so that the 16-byte fragment reads of v_mfma_f32_32x32x16_bf16
// (a lane reads 8 consecutive k of one row) and the 16-byte staging writes are bank-conflict
// free.  LDS is double buffered: the global loads of slice k+1 are in flight while slice k is
// multiplied.  A [K,N] operand is transposed in registers (8x8 blocks, v_perm) on its way into
// LDS, so both layouts feed the same multiply loop.
//
// The weight tile takes the MFMA "A" slot and the activation tile the "B" slot: each lane then
// owns one token row and groups of 4 consecutive output features, which makes every epilogue
// access an 8-byte vector (4 bf16) and keeps SwiGLU's gate/up pair in the same lane.
//
// Workgroup ids are remapped so that each XCD (ids congruent mod 8) works on a contiguous run
// of tiles, ordered in groups of GROUP_M row tiles, to keep operand panels hot in its L2.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace sv {
namespace {

constexpr int BK = 64;
constexpr int kGroupM = 4;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ swz(row)) << 4); }

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

template <int BM, int BN, int WAVES_M, int WAVES_N, bool KN, bool DUAL>
struct Cfg {
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int XCH = BM * 8 / NT;      // 16-byte chunks per thread, activation tile
  static constexpr int WCH = BN * 8 / NT;      // weight tile
  static constexpr int STAGE = (BM + BN) * 128;
  static constexpr int LDS = 2 * STAGE;
  static constexpr int NOUT = DUAL ? BN / 2 : BN;   // output columns per tile
  static_assert(!DUAL || !KN, "the dual product is forward only");
  static_assert(!KN || WCH % 8 == 0, "a [K,N] operand is staged in whole 8x8 blocks per thread");
};

// x of the lane N places further on in its row of 16 lanes (cyclic)
template <int N> __device__ __forceinline__ float dpp_row_ror(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + N, 0xf, 0xf, false));
}

// Epilogue on 4 consecutive output features of one token row, in two phases so that a caller can
// issue all loads of a row block before the first store (the output and the residual / gate / up
// buffers may alias as far as the compiler knows, so loads are never hoisted over stores for us).
struct EpiIn { bf16x4 r, r2; f32x4 cs; };

template <int EPI>
__device__ __forceinline__ void epilogue_load4(const GemmArgs& a, int m, int n, EpiIn& in) {
  const int64_t ir = (int64_t)m * a.ldr + n;
  if (EPI == EPI_RESID || EPI == EPI_SWIGLU_BWD || EPI == EPI_GELU_BWD) in.r = *reinterpret_cast<const bf16x4*>((const bf16*)a.R + ir);
  if (EPI == EPI_SWIGLU_BWD) in.r2 = *reinterpret_cast<const bf16x4*>((const bf16*)a.R2 + ir);
  if (EPI == EPI_ROPE && n < a.rope_cols) {      // cos_i, sin_i, cos_i+1, sin_i+1 of the two feature pairs
    const int half = a.rope_hd >> 1, p = m % a.rope_S, i0 = (n % a.rope_hd) >> 1;
    in.cs = *reinterpret_cast<const f32x4*>(a.rope_cs + ((int64_t)p * half + i0) * 2);
  }
}

// rs multiplies the accumulators first (GemmArgs::rscale; the kinds that can follow a norm).  put(w, p) stores the four bf16
// values p into output w (0: C, 1: C2, 2: C3) at the place this call stands for; roped: the features are rotated (EPI_ROPE).
// Returns the sum of squares of the four values as stored in C.
template <int EPI, class Put>
__device__ __forceinline__ float epilogue_math4(const GemmArgs& a, bool roped, const float (&v_in)[4], const float (&u_in)[4], const EpiIn& in,
                                                float rs, Put&& put) {
  const bf16x4& r = in.r;
  const bf16x4& r2 = in.r2;
  constexpr bool kScaled = EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_SWIGLU || EPI == EPI_ROPE;
  float v[4], u[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = kScaled ? v_in[i] * rs : v_in[i]; u[i] = kScaled ? u_in[i] * rs : u_in[i]; }
  float o[4];
  switch (EPI) {
    case EPI_STORE:
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i];
      break;
    case EPI_RESID:
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i] + (float)r[i];
      break;
    case EPI_GELU: {
      if (a.C2) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)v[i]; put(1, p); }
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = gelu_f(v[i]);
    } break;
    case EPI_SWIGLU: {
      if (a.C2) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)v[i]; put(1, p); }
      if (a.C3) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)u[i]; put(2, p); }
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = silu_f(v[i]) * u[i];
    } break;
    case EPI_SWIGLU_BWD: {
      bf16x4 p;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gf = (float)r[i];
        o[i] = v[i] * (float)r2[i] * silu_grad_f(gf);
        p[i] = (bf16)(v[i] * silu_f(gf));
      }
      put(1, p);
    } break;
    case EPI_ROPE: {
      if (roped) {
        const f32x4 cs = in.cs;
        o[0] = v[0] * cs[0] - v[1] * cs[1];
        o[1] = v[0] * cs[1] + v[1] * cs[0];
        o[2] = v[2] * cs[2] - v[3] * cs[3];
        o[3] = v[2] * cs[3] + v[3] * cs[2];
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = v[i];
      }
    } break;
    default:  // EPI_GELU_BWD
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i] * gelu_grad_f((float)r[i]);
      break;
  }
  bf16x4 p;
  float sq = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) { p[i] = (bf16)o[i]; sq = fmaf((float)p[i], (float)p[i], sq); }
  put(0, p);
  return sq;
}

// the same on the output element (m, n), through plain pointers
template <int EPI>
__device__ __forceinline__ float epilogue_apply4(const GemmArgs& a, int m, int n, const float (&v_in)[4], const float (&u_in)[4], const EpiIn& in,
                                                 float rs = 1.0f) {
  const int64_t ic = (int64_t)m * a.ldc + n;
  return epilogue_math4<EPI>(a, EPI == EPI_ROPE && n < a.rope_cols, v_in, u_in, in, rs, [&](int w, bf16x4 p) {
    *reinterpret_cast<bf16x4*>((bf16*)(w == 0 ? a.C : w == 1 ? a.C2 : a.C3) + ic) = p;
  });
}

// How many trips ahead of its stores the direct-to-LDS kernel's epilogue reads its inputs (a trip: two rows per lane).  One trip
// of work is shorter than a memory round trip, so one trip ahead leaves the epilogue waiting once per trip.
template <int EPI> constexpr int kEpiAhead = EPI == EPI_ROPE ? 2 : EPI == EPI_SWIGLU_BWD ? 3 : 4;   // as far as the registers go

// does this kind of epilogue take GemmArgs::rscale?
template <int EPI> constexpr bool kEpiScaled = EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_SWIGLU || EPI == EPI_ROPE;

// The accumulators of one 32-row block of a wave tile: NIO feature blocks of 32 (the second half of the
// accumulator blocks is the `up` product of a dual launch).  Per feature block: its four loads first,
// then compute and store.
template <int EPI, int NIO, int NI, int MI>
__device__ __forceinline__ void epilogue_rows(const GemmArgs& a, int M, const f32x16 (&acc)[NI][MI], int mi, int m, int nbase) {
  if (m >= M) return;
  const float rs = kEpiScaled<EPI> && a.rscale ? a.rscale[m] : 1.0f;
#pragma unroll
  for (int ni = 0; ni < NIO; ++ni) {
    EpiIn in[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) epilogue_load4<EPI>(a, m, nbase + ni * 32 + q * 8, in[q]);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = acc[ni][mi][q * 4 + i];
        u[i] = (EPI == EPI_SWIGLU) ? acc[ni + (NIO < NI ? NIO : 0)][mi][q * 4 + i] : 0.0f;
      }
      epilogue_apply4<EPI>(a, m, nbase + ni * 32 + q * 8, v, u, in[q], rs);
    }
  }
}

// SPLIT: blockIdx.y takes one of gridDim.y contiguous runs of k slices and leaves its fp32 partial product in
// a.split_ws[blockIdx.y][M][N]; splitk_reduce_kernel adds the runs in a fixed order and applies the epilogue.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool KN, int EPI, bool SPLIT = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_mfma_kernel(GemmArgs a, int tiles_m, int tiles_n) {
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  static_assert(!SPLIT || (!DUAL && !KN && BM * BN <= 128 * 128), "split-k serves the small [N,K] tiles");
  using C = Cfg<BM, BN, WAVES_M, WAVES_N, KN, DUAL>;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // grouped form: the row count lives in device memory and the launch covers its bound
  const int M = a.m_dev ? *a.m_dev : a.M;
  if (a.m_dev) tiles_m = (M + BM - 1) / BM;
  // ---- tile assignment (XCD-contiguous, grouped raster)
  const int nblk = tiles_m * tiles_n;
  const int per_xcd = (nblk + 7) >> 3;
  const int pid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (pid >= nblk) return;
  const int in_group = kGroupM * tiles_n;
  const int first_m = (pid / in_group) * kGroupM;
  const int gsz = min(tiles_m - first_m, kGroupM);
  const int tile_m = first_m + (pid % in_group) % gsz;
  const int tile_n = (pid % in_group) / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * C::NOUT;
  const int64_t goff = a.tile_group ? (int64_t)a.tile_group[m0 >> 8] * a.group_stride : 0;   // this row block's weight matrices

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  // ---- global -> register staging
  // Small tiles keep TWO slices in flight in registers (PF2): with at most two workgroups of four waves on a CU, one
  // slice of multiplies (~500 cycles) does not cover a global load's latency.  Large tiles have no registers for that.
  constexpr bool PF2 = BM * BN <= 128 * 128;
  constexpr int NSET = PF2 ? 2 : 1;
  bf16x8 xregs[NSET][C::XCH], wregs[NSET][C::WCH];
  int seg = 0, kin = 0;       // position of the slice being loaded
  auto load_slice = [&](auto set_tag) {
    bf16x8 (&xreg)[C::XCH] = xregs[decltype(set_tag)::value];
    bf16x8 (&wreg)[C::WCH] = wregs[decltype(set_tag)::value];
    const bf16* A = (const bf16*)a.seg[seg].A;
    const int64_t lda = a.seg[seg].lda, ldb = a.seg[seg].ldb;
#pragma unroll
    for (int i = 0; i < C::XCH; ++i) {
      const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
      const int m = min(m0 + r, M - 1);
      xreg[i] = *reinterpret_cast<const bf16x8*>(A + (int64_t)m * lda + kin + c * 8);
    }
    if (!KN) {
#pragma unroll
      for (int i = 0; i < C::WCH; ++i) {
        const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
        const bf16* B;
        int n;
        if (DUAL && r >= BN / 2) { B = (const bf16*)a.B2 + goff; n = n0 + r - BN / 2; }
        else { B = (const bf16*)a.seg[seg].B + goff; n = n0 + r; }
        const int64_t ld = (DUAL && r >= BN / 2) ? a.ldb2 : ldb;
        wreg[i] = *reinterpret_cast<const bf16x8*>(B + (int64_t)n * ld + kin + c * 8);
      }
    } else {
      // thread owns 8x8 blocks: 8 consecutive k rows x 8 consecutive n columns
      const bf16* B = (const bf16*)a.seg[seg].B + goff;
#pragma unroll
      for (int b = 0; b < C::WCH / 8; ++b) {
        const int blk = tid + b * C::NT, ng = blk % (BN / 8), kg = blk / (BN / 8);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          wreg[b * 8 + j] = *reinterpret_cast<const bf16x8*>(B + (int64_t)(kin + kg * 8 + j) * ldb + n0 + ng * 8);
      }
    }
    if (PF2) {                 // branch-free callers load past the end: stay on the last slice then
      if (kin + BK < a.seg[seg].K) kin += BK;
      else if (seg + 1 < a.nseg) { kin = 0; ++seg; }
    } else {
      kin += BK;
      if (kin >= a.seg[seg].K) { kin = 0; ++seg; }
    }
  };
  auto store_slice = [&](int stage, auto set_tag) {
    bf16x8 (&xreg)[C::XCH] = xregs[decltype(set_tag)::value];
    bf16x8 (&wreg)[C::WCH] = wregs[decltype(set_tag)::value];
    char* xs = smem + stage * C::STAGE;
    char* ws = xs + BM * 128;
#pragma unroll
    for (int i = 0; i < C::XCH; ++i) {
      const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
      *reinterpret_cast<bf16x8*>(xs + lds_off(r, c)) = xreg[i];
    }
    if (!KN) {
#pragma unroll
      for (int i = 0; i < C::WCH; ++i) {
        const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
        *reinterpret_cast<bf16x8*>(ws + lds_off(r, c)) = wreg[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < C::WCH / 8; ++b) {
        const int blk = tid + b * C::NT, ng = blk % (BN / 8), kg = blk / (BN / 8);
        u32x4 in[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) in[j] = __builtin_bit_cast(u32x4, wreg[b * 8 + j]);
#pragma unroll
        for (int n = 0; n < 8; ++n) {
          // column n of the block: element n of rows 0..7 -> one 16-byte chunk (8 consecutive k)
          u32x4 o;
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const uint32_t lo = in[2 * p][n >> 1], hi = in[2 * p + 1][n >> 1];
            o[p] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
          }
          *reinterpret_cast<u32x4*>(ws + lds_off(ng * 8 + n, kg)) = o;
        }
      }
    }
  };

  int nslices = 0;
  for (int s = 0; s < a.nseg; ++s) nslices += a.seg[s].K / BK;
  if (SPLIT) {                                       // this workgroup's run of slices; the loads start at its first
    const int first = (int)((int64_t)nslices * blockIdx.y / gridDim.y);
    nslices = (int)((int64_t)nslices * (blockIdx.y + 1) / gridDim.y) - first;
    int skip = first;
    while (skip >= a.seg[seg].K / BK) { skip -= a.seg[seg].K / BK; ++seg; }
    kin = skip * BK;
  }

  f32x16 acc[C::NI][C::MI];
#pragma unroll
  for (int i = 0; i < C::NI; ++i)
#pragma unroll
    for (int j = 0; j < C::MI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // per-lane fragment rows
  const int l31 = lane & 31, lhi = lane >> 5;
  int wrow[C::NI];
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    if (DUAL) wrow[ni] = (ni < C::NI / 2 ? wn * (C::WTN / 2) + ni * 32 : BN / 2 + wn * (C::WTN / 2) + (ni - C::NI / 2) * 32) + l31;
    else wrow[ni] = wn * C::WTN + ni * 32 + l31;
  }

  auto multiply = [&](int stage) {
    const char* xs = smem + stage * C::STAGE;
    const char* ws = xs + BM * 128;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 xf[C::MI], wf[C::NI];
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
        xf[mi] = *reinterpret_cast<const bf16x8*>(xs + lds_off(wm * C::WTM + mi * 32 + l31, kk * 2 + lhi));
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        wf[ni] = *reinterpret_cast<const bf16x8*>(ws + lds_off(wrow[ni], kk * 2 + lhi));
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
          acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, NSET - 1>;
  if constexpr (PF2) {
    // Slice kt is multiplied from LDS stage kt & 1 while slice kt + 1 sits in register set (kt + 1) & 1 (stored to the
    // other stage at the end of the step) and slice kt + 2 is being loaded into set kt & 1.  No branch in a step: loads
    // past the end re-read the last slice, the store after the last multiply fills a stage nobody reads -- so the
    // compiler's wait before a store counts exactly the newer loads still in flight.
    load_slice(Set0{});
    load_slice(Set1{});
    store_slice(0, Set0{});
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < nslices; kt += 2) {
      load_slice(Set0{});
      __builtin_amdgcn_sched_barrier(0);     // the loads stay at the top of the step: sunk below the multiply they
      multiply(0);                           // would be issued one step late
      __builtin_amdgcn_sched_barrier(0);
      store_slice(1, Set1{});
      __syncthreads();
      load_slice(Set1{});
      __builtin_amdgcn_sched_barrier(0);
      multiply(1);
      __builtin_amdgcn_sched_barrier(0);
      store_slice(0, Set0{});
      __syncthreads();
    }
    if (kt < nslices) multiply(0);
  } else {
    load_slice(Set0{});
    store_slice(0, Set0{});
    __syncthreads();
    for (int kt = 0; kt < nslices; ++kt) {
      const bool more = kt + 1 < nslices;
      if (more) load_slice(Set0{});
      multiply(kt & 1);
      if (more) store_slice((kt + 1) & 1, Set0{});
      __syncthreads();
    }
  }

  // ---- epilogue: lane owns token row (lane & 31) of each 32-row block and, per register
  // quad q, output features 8q + 4*(lane>>5) .. +3 of each 32-feature block.
  constexpr int NIO = DUAL ? C::NI / 2 : C::NI;
  if constexpr (SPLIT) {
    float* part = a.split_ws + (int64_t)blockIdx.y * M * a.N;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
      const int m = m0 + wm * C::WTM + mi * 32 + l31;
      if (m >= M) continue;
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = acc[ni][mi][q * 4 + i];
          *reinterpret_cast<f32x4*>(part + (int64_t)m * a.N + n0 + wn * C::WTN + ni * 32 + q * 8 + lhi * 4) = v;
        }
    }
  } else {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
      epilogue_rows<EPI, NIO, C::NI, C::MI>(a, M, acc, mi, m0 + wm * C::WTM + mi * 32 + l31, n0 + wn * (DUAL ? C::WTN / 2 : C::WTN) + lhi * 4);
  }
}

// Sum of the split-k partial products, in the order of the splits, then the epilogue: one thread per 4 consecutive
// output features of a row.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs a, int nsplit) {
  const int n4 = a.N >> 2;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)a.M * n4) return;
  const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
  const float* p = a.split_ws + (int64_t)m * a.N + n;
  f32x4 sum = *reinterpret_cast<const f32x4*>(p);
  for (int s = 1; s < nsplit; ++s) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(p + (int64_t)s * a.M * a.N);
#pragma unroll
    for (int i = 0; i < 4; ++i) sum[i] += v[i];
  }
  float v[4], u[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = sum[i];
  EpiIn in;
  epilogue_load4<EPI>(a, m, n, in);
  epilogue_apply4<EPI>(a, m, n, v, u, in, kEpiScaled<EPI> && a.rscale ? a.rscale[m] : 1.0f);
}

// ------------------------------------------------------------------------------------------
// 256x256x64 NT kernel with direct global->LDS loads (buffer_load_dwordx4 ... lds, 16 bytes per lane).
//
// Each wave instruction copies 64 x 16 bytes to one contiguous 1 KB block of LDS = 8 tile rows;
// the XOR swizzle is applied by choosing WHICH global chunk each lane fetches, so the LDS image
// is the same swizzled layout the fragment reads expect and no VGPR staging or ds_write is
// needed.  The loads are buffer loads: a descriptor per operand panel in scalar registers, the
// lane's byte offset in one vector register, the slice's k offset as the scalar offset -- no
// 64-bit address arithmetic per slice.  Two LDS stages; the 16 loads a wave owes for slice k+1 and
// the 8 fragment reads of the next 16-wide k step are issued ONE AT A TIME BEHIND AN MFMA, in the
// 32 cycles the matrix pipe is busy with it (one wave per SIMD: whatever is issued between two
// MFMAs after the pipe has drained idles it; grouping them between blocks of four MFMAs measured
// 1-3 % slower), fragments double buffered in registers.  The loop is rotated so that the one
// full wait + barrier per slice sits at the loop top: after it the compiler's counter tracking
// is exact and no other wait stalls the MFMA stream.
//
// GROUPED: the grouped form (per-row-block weight group, row count from device memory) as its own instantiation, so
// that the dense form's code -- in particular its waits, which scalar loads in the tile-change path would disturb
// (they share a counter with the LDS reads) -- is unaffected by it.
//
// NF: the forms that stand at the two ends of an RMSNorm run inside the products (their own instantiations, for the same
// reason): the kinds that can follow a norm multiply every row by GemmArgs::rscale, EPI_RESID also writes GemmArgs::rowsq.
// SPLIT: a tile's k slices are dealt to nsplit workgroups in contiguous runs (virtual block = (run, tile), the tiles of one run
// next to each other so that an XCD's workgroups share operand panels); each leaves its fp32 partial product in
// a.split_ws[run][M][N] and splitk_reduce_kernel adds the runs in a fixed order and applies the epilogue.
template <int EPI, bool GROUPED, bool NF = false, bool SPLIT = false>
__global__ __launch_bounds__(256) void gemm_mfma_dma_kernel(GemmArgs a, int tiles_m, int tiles_n, int nsplit) {
  static_assert(!SPLIT || (EPI == EPI_STORE && !GROUPED && !NF), "a split run stores bare partial products");
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  constexpr bool RS = NF && kEpiScaled<EPI>, SQ = NF && EPI == EPI_RESID;
  constexpr int BM = 256, BN = 256, STAGE = (BM + BN) * 128, MI = 4, NI = 4;
  constexpr int NOUT = DUAL ? 128 : 256;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // grouped form: the row count lives in device memory and the launch covers its bound
  const int M = GROUPED ? *a.m_dev : a.M;
  if (GROUPED) tiles_m = (M + BM - 1) / BM;
  // Persistent workgroups: workgroup b works on the virtual block ids b, b + gridDim.x, ...; a virtual id
  // maps to a tile so that ids congruent mod 8 (one XCD) walk a contiguous run of tiles in groups of
  // kGroupM row tiles.  gridDim.x is a multiple of 8, so a workgroup stays on its XCD's run.
  const int nblk = tiles_m * tiles_n, nvb = SPLIT ? nblk * nsplit : nblk;
  const int per_xcd = (nvb + 7) >> 3;
  auto tile_of = [&](int vb, int& m0, int& n0, int& run) -> bool {
    if (vb >= per_xcd * 8) return false;
    int pid = (vb & 7) * per_xcd + (vb >> 3);
    if (pid >= nvb) return false;
    run = 0;
    if (SPLIT) { run = pid / nblk; pid -= run * nblk; }
    const int in_group = kGroupM * tiles_n;
    const int first_m = (pid / in_group) * kGroupM;
    const int gsz = min(tiles_m - first_m, kGroupM);
    m0 = (first_m + (pid % in_group) % gsz) * BM;
    n0 = ((pid % in_group) / gsz) * NOUT;
    return true;
  };

  const int tid = threadIdx.x, lane = tid & 63, l31 = lane & 31, lhi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave & 1, wn = wave >> 1;

  // ---- DMA side: one continuous stream of slices across this workgroup's tiles, always one slice
  // ahead of the multiply.  State: virtual block d_vb (tile d_m0, d_n0), segment dseg, offset dk.
  int d_vb = blockIdx.x, d_m0 = 0, d_n0 = 0, d_run = 0, d_left = 0, dseg = 0, dk = 0, d_K = 0;   // d_K: length of segment dseg, kept in a register
                                                                           // (a per-slice kernel-argument load would share
                                                                           // its wait counter with the LDS reads)
  bool d_valid = tile_of(d_vb, d_m0, d_n0, d_run);
  int nslices = 0;
  for (int s = 0; s < a.nseg; ++s) nslices += a.seg[s].K / BK;
  // SPLIT: run r of a tile takes the slices [r * nslices / nsplit, (r + 1) * nslices / nsplit) of its segments laid end to end
  auto start_run = [&]() {                                    // the stream's position at the first slice of run d_run
    const int ks = d_run * nslices / nsplit;
    d_left = (d_run + 1) * nslices / nsplit - ks;
    dseg = 0;
    int k = ks * BK;
    while (k >= a.seg[dseg].K) { k -= a.seg[dseg].K; ++dseg; }
    dk = k;
  };
  const char *gA, *gB, *gB2;
  __amdgpu_buffer_rsrc_t rA, rB, rB2;     // buffer descriptors of the panels the stream reads: base = first row, no bound
  unsigned voffA[8], voffB[8];
  auto set_segment = [&]() {
    const GemmSeg& sg = a.seg[dseg];
    d_K = sg.K;
    gA = (const char*)((const bf16*)sg.A + (int64_t)d_m0 * sg.lda);
    const int64_t goff = GROUPED ? (int64_t)a.tile_group[d_m0 >> 8] * a.group_stride : 0;
    if (!DUAL && a.nbcol > 0) {
      int start = 0, j = 0;
      while (j + 1 < a.nbcol && d_n0 >= start + a.ncol[j]) { start += a.ncol[j]; ++j; }
      gB = (const char*)((const bf16*)a.Bcol[j] + (int64_t)(d_n0 - start) * sg.ldb);
    } else {
      gB = (const char*)((const bf16*)sg.B + goff + (int64_t)d_n0 * sg.ldb);
    }
    gB2 = DUAL ? (const char*)((const bf16*)a.B2 + goff + (int64_t)d_n0 * a.ldb2) : gB;
    rA = __builtin_amdgcn_make_buffer_rsrc((void*)gA, (short)0, -1, 0x00020000);
    rB = __builtin_amdgcn_make_buffer_rsrc((void*)gB, (short)0, -1, 0x00020000);
    rB2 = __builtin_amdgcn_make_buffer_rsrc((void*)gB2, (short)0, -1, 0x00020000);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (wave + 4 * i) * 8 + (lane >> 3), c = (lane & 7) ^ swz(r);
      const int ra = min(r, M - 1 - d_m0);                  // ragged row tail: re-read the last row
      voffA[i] = (unsigned)((int64_t)ra * sg.lda + c * 8) * 2u;
      if (DUAL) voffB[i] = (unsigned)((int64_t)(r & 127) * (i >= 4 ? a.ldb2 : sg.ldb) + c * 8) * 2u;
      else voffB[i] = (unsigned)((int64_t)r * sg.ldb + c * 8) * 2u;
    }
  };
  auto dma = [&](int stage, int j) {                          // j: 0..7 activation rows, 8..15 weight rows
    const int i = j & 7;
    const unsigned off = j < 8 ? voffA[i] : voffB[i];
    char* dst = smem + stage * STAGE + (j < 8 ? 0 : BM * 128) + (wave + 4 * i) * 1024;
    // buffer form of the direct-to-LDS load: per-lane byte offset in a register, the slice's offset k * 2 as the scalar offset
    __builtin_amdgcn_raw_ptr_buffer_load_lds(j < 8 ? rA : ((DUAL && i >= 4) ? rB2 : rB), (__attribute__((address_space(3))) void*)dst, 16,
                                             (int)off, dk * 2, 0, 0);
  };
  auto advance = [&]() {                                      // to the next slice of the stream
    dk += BK;
    if (SPLIT) {
      if (--d_left == 0) {                                    // the run is through: on to the next virtual block
        d_vb += gridDim.x;
        d_valid = tile_of(d_vb, d_m0, d_n0, d_run);
        if (d_valid) { start_run(); set_segment(); }
        else dk -= BK;                                        // a finished stream re-reads its last slice
        return;
      }
      if (dk < d_K) return;
      dk = 0; ++dseg; set_segment();
      return;
    }
    if (dk < d_K) return;
    dk = 0;
    if (dseg + 1 < a.nseg) { ++dseg; set_segment(); return; }
    dseg = 0;
    d_vb += gridDim.x;
    d_valid = tile_of(d_vb, d_m0, d_n0, d_run);
    if (d_valid) set_segment();
  };

  int xrow[MI], wrow[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) xrow[mi] = wm * 128 + mi * 32 + l31;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) wrow[ni] = (DUAL ? (ni < 2 ? wn * 64 + ni * 32 : 128 + wn * 64 + (ni - 2) * 32) : wn * 128 + ni * 32) + l31;

  f32x16 acc[NI][MI];

#define SV_SB __builtin_amdgcn_sched_barrier(0)
  // One 16-wide k step: MFMAs on (xc, wc); fragments (rstage, rkk) are read into (xn, wn_) and the
  // DMAs [d0, d0 + 8) of the stream's next slice are issued into dstage, both spread over the four MFMA groups.
  auto step = [&](bf16x8 (&xc)[MI], bf16x8 (&wc)[NI], bf16x8 (&xn)[MI], bf16x8 (&wn_)[NI], bool do_read, int rstage, int rkk,
                  bool do_dma, int dstage, int d0) {
    const char* xs = smem + rstage * STAGE;
    const char* ws = xs + BM * 128;
    // The fragments this step multiplies were requested during the previous step, the youngest of them four MFMAs
    // ago: wait for them here, before this step's own requests are queued behind them.
    __builtin_amdgcn_s_waitcnt(0xc07f);
    SV_SB;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // every other instruction of the group is issued behind an MFMA, in the 32 cycles the matrix pipe is busy with it
      acc[g][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[g], xc[0], acc[g][0], 0, 0, 0);
      SV_SB;
      if (do_read) xn[g] = *reinterpret_cast<const bf16x8*>(xs + lds_off(xrow[g], rkk * 2 + lhi));
      SV_SB;
      acc[g][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[g], xc[1], acc[g][1], 0, 0, 0);
      SV_SB;
      if (do_read) wn_[g] = *reinterpret_cast<const bf16x8*>(ws + lds_off(wrow[g], rkk * 2 + lhi));
      SV_SB;
      acc[g][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[g], xc[2], acc[g][2], 0, 0, 0);
      SV_SB;
      if (do_dma) dma(dstage, d0 + 2 * g);
      SV_SB;
      acc[g][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[g], xc[3], acc[g][3], 0, 0, 0);
      SV_SB;
      if (do_dma) dma(dstage, d0 + 2 * g + 1);
      SV_SB;
    }
  };

  if (!d_valid) return;
  bf16x8 xf0[MI], wf0[NI], xf1[MI], wf1[NI];
  if (SPLIT) start_run();
  set_segment();
#pragma unroll
  for (int j = 0; j < 16; ++j) dma(0, j);                     // slice 0 of the first tile
  advance();
  int par = 0;                                                // LDS stage of the current tile's slice 0

  int m0, n0, run;
  for (int vb = blockIdx.x; tile_of(vb, m0, n0, run); vb += gridDim.x) {
    const int nsl = SPLIT ? (run + 1) * nslices / nsplit - run * nslices / nsplit : nslices;   // slices of this virtual block
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < MI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    // ---- what the epilogue's global accesses need, set up here because a full tile asks for its first inputs a slice early.
    // In the read-back of the epilogue a lane serves row er of each group of 4 rows, 16-byte chunk ec4 (and 16 + ec4).
    // One buffer descriptor per tensor, based at the tile's first row and the wave's first column; inside it a lane's
    // byte offset is (row * ld + column) * 2, of which the lane's part never changes and the row block's part is a scalar:
    // no 64-bit address arithmetic per access.
    constexpr bool kHasInputs = EPI == EPI_RESID || EPI == EPI_SWIGLU_BWD || EPI == EPI_GELU_BWD || EPI == EPI_ROPE;
    constexpr int PD = kEpiAhead<EPI>;                   // trips the epilogue's global reads run ahead of its stores
    const int er = lane >> 4, ec4 = lane & 15;
    const int ncol0 = n0 + wn * (DUAL ? 64 : 128);
    auto desc = [&](const void* base, int ld) {
      return __builtin_amdgcn_make_buffer_rsrc((void*)((const bf16*)base + (int64_t)m0 * ld + ncol0), (short)0, -1, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t bC = desc(a.C, a.ldc), bC2 = desc(a.C2, a.ldc), bC3 = desc(a.C3, a.ldc);
    const __amdgpu_buffer_rsrc_t bR = desc(a.R, a.ldr), bR2 = desc(a.R2, a.ldr);
    const int vC = ((wm * 128 + er) * a.ldc + ec4 * 4) * 2, vR = ((wm * 128 + er) * a.ldr + ec4 * 4) * 2;
    // SPLIT: the run's partial product, fp32 [M][N]
    const __amdgpu_buffer_rsrc_t bW = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.split_ws + ((int64_t)run * M + m0) * a.N + ncol0), (short)0, -1, 0x00020000);
    const int vW = ((wm * 128 + er) * a.N + ec4 * 4) * 4;
    // offsets of row block rb (rows rb .. rb + 3 of the wave's 128): per lane (vo) and scalar (so).  A ragged tile
    // re-reads its last row for the rows past the end, which takes the row into the lane's part.
    auto place = [&](auto check_tag, int rb, int ld, int vlane, int& vo, int& so) {
      if (decltype(check_tag)::value) { vo = (min(wm * 128 + rb + er, M - 1 - m0) * ld + ec4 * 4) * 2; so = 0; }
      else { vo = vlane; so = rb * ld * 2; }
    };
    int rope_p0 = 0, rope_v_lo = 0, rope_v_hi = 0;      // first row's position; byte offsets of the lane's feature pairs in a table row
    if (EPI == EPI_ROPE) {
      rope_p0 = (m0 + wm * 128) % a.rope_S;
      rope_v_lo = (((ncol0 + ec4 * 4) % a.rope_hd) >> 1) * 8;
      rope_v_hi = (((ncol0 + 64 + ec4 * 4) % a.rope_hd) >> 1) * 8 - rope_v_lo;
    }
    const __amdgpu_buffer_rsrc_t bT = __builtin_amdgcn_make_buffer_rsrc((void*)a.rope_cs, (short)0, -1, 0x00020000);
    auto ld8 = [&](__amdgpu_buffer_rsrc_t b, int vo, int so) { return __builtin_bit_cast(bf16x4, __builtin_amdgcn_raw_buffer_load_b64(b, vo, so, 0)); };
    // the inputs of trip `trip` (two rows of row block mi = trip / 4 per lane): residual, gate / up, RoPE table
    auto load_inputs = [&](auto check_tag, int trip, EpiIn (&lo)[2], EpiIn (&hi)[2]) {
      const int mi = trip >> 2, it = (trip & 3) * 2;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int rb = mi * 32 + (it + k) * 4;
        if (EPI == EPI_ROPE) {
          // position of the row in its sequence without a division per row: the wave's first row is reduced once
          // per tile, the rows of the tile follow it consecutively
          int p = rope_p0 + rb + er;
          if (a.rope_S >= 256) p -= p >= a.rope_S ? a.rope_S : 0; else p %= a.rope_S;
          const int vo = p * (a.rope_hd >> 1) * 8 + rope_v_lo;      // the table entry (position p, feature pair) is 8 bytes
          lo[k].cs = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(bT, vo, 0, 0));
          hi[k].cs = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(bT, vo + rope_v_hi, 0, 0));
        } else if (kHasInputs) {
          int vo, so;
          place(check_tag, rb, a.ldr, vR, vo, so);
          lo[k].r = ld8(bR, vo, so);
          hi[k].r = ld8(bR, vo + 128, so);
          if (EPI == EPI_SWIGLU_BWD) { lo[k].r2 = ld8(bR2, vo, so); hi[k].r2 = ld8(bR2, vo + 128, so); }
        }
      }
    };
    EpiIn in_lo[PD][2], in_hi[PD][2];                    // [trip mod PD][row of the pair]
    const bool full_tile = m0 + 256 <= M;
    auto first_inputs = [&]() {                          // of a full tile, a slice before the epilogue
      if (kHasInputs && full_tile) {
#pragma unroll
        for (int t = 0; t < PD; ++t) load_inputs(std::false_type{}, t, in_lo[t], in_hi[t]);
      }
    };
    // ---- slice 0 (its loads were issued during the previous tile's last slice, or above)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    SV_SB;
    // the row factors of the wave's 128 rows are asked for here, a whole k loop before the epilogue wants them (its
    // first loads would otherwise start with a memory round trip per tile); the next wait for memory is a slice away
    float rs_pre0 = 1.0f, rs_pre1 = 1.0f;
    if (RS) {
      rs_pre0 = a.rscale[min(m0 + wm * 128 + lane, M - 1)];
      rs_pre1 = a.rscale[min(m0 + wm * 128 + 64 + lane, M - 1)];
    }
    if (nsl == 1) first_inputs();
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      xf0[g] = *reinterpret_cast<const bf16x8*>(smem + par * STAGE + lds_off(xrow[g], lhi));
      wf0[g] = *reinterpret_cast<const bf16x8*>(smem + par * STAGE + BM * 128 + lds_off(wrow[g], lhi));
    }
    step(xf0, wf0, xf1, wf1, true, par, 1, true, par ^ 1, 0);
    step(xf1, wf1, xf0, wf0, true, par, 2, true, par ^ 1, 8);
    if (d_valid) advance();
    step(xf0, wf0, xf1, wf1, true, par, 3, false, 0, 0);
    for (int kt = 1; kt < nsl; ++kt) {
      const int st = (par + kt) & 1;
      __builtin_amdgcn_s_waitcnt(0);   // my DMAs of slice kt have landed, my fragment reads of slice kt-1 are done
      __syncthreads();                 // ... and so have everybody's: stage st is complete, stage st^1 is free
      SV_SB;
      if (kt == nsl - 1) first_inputs();     // their round trip hides behind the last slice's products
      SV_SB;
      step(xf1, wf1, xf0, wf0, true, st, 0, true, st ^ 1, 0);     // MFMAs of (kt-1, k step 3)
      step(xf0, wf0, xf1, wf1, true, st, 1, true, st ^ 1, 8);
      if (d_valid) advance();
      step(xf1, wf1, xf0, wf0, true, st, 2, false, 0, 0);
      step(xf0, wf0, xf1, wf1, true, st, 3, false, 0, 0);
    }
    step(xf1, wf1, xf0, wf0, false, 0, 0, false, 0, 0);

    // ---- epilogue through LDS (the next tile's slice 0 is landing in the other stage meanwhile).
    // In the accumulator layout a lane owns one token row and scattered groups of 4 features, so a
    // store instruction would touch 32 rows with 16 bytes each; the memory pipeline then takes ~11 us
    // per tile.  Each wave instead writes its 32 x 128 fp32 block into its own 16 KB patch of the
    // stage that was just consumed (16-byte chunks XOR-swizzled by the row: conflict-free both ways)
    // and reads it back so that 16 consecutive lanes cover 128 contiguous bytes of an output row;
    // every global access of the epilogue (result, residual, gate / up) becomes a full-line run.
    const int sl = (par + nsl - 1) & 1;
    par = (par + nsl) & 1;
    __syncthreads();                                   // everybody is done reading stage sl
    char* patch = smem + sl * STAGE + wave * 16384;
    // per wave, behind the two stages: the row factors of its 128 rows (each lane of the read-back needs those of the
    // rows it serves) and the rows' sums of squares (stored in one piece when the tile is done)
    float* rsbuf = reinterpret_cast<float*>(smem + 2 * STAGE) + wave * 256;
    float* sqbuf = rsbuf + 128;
    if (RS) { rsbuf[lane] = rs_pre0; rsbuf[64 + lane] = rs_pre1; }
    // Sixteen trips per tile: row block mi = trip / 4, two rows per lane and trip.  The epilogue's global reads (residual,
    // gate / up, RoPE table) run kEpiAhead trips ahead of its stores; the first of them were asked for when the last slice
    // began.  (The memory counter retires in order: a read is waited for together with every store issued before it, so
    // the reads of a trip are issued before the stores they must not wait for have piled up.)  Tiles that lie
    // inside the M rows run without any per-lane condition (CHECK = false): around divergent branches the compiler's
    // wait insertion falls back to waiting for (nearly) everything in flight, one memory round trip per store.
    auto run_epilogue = [&](auto check_tag) {
      constexpr bool CHECK = decltype(check_tag)::value;
      if constexpr (DUAL) {
        if (!a.C2 && !a.C3) {
          // Forward-only check (no stash of g and u).  Gate and up of one feature sit in the same lane and register
          // index, so SiLU(g) * u is taken in the accumulator layout and only its bf16 result goes through the patch:
          // 128 token rows x 64 features x 2 bytes = the 16 KB patch in one piece (16-byte chunks XOR-swizzled by bits
          // 1..3 of the row), a quarter of the fp32 way's LDS traffic, and the read-back gives every lane 16 bytes of a
          // row, so 8 lanes store one full 128-byte line.  (With the stashes, three such passes measured slower than
          // the fp32 way below, which serves them.)
          // The lane's row and chunk numbers are made opaque once per tile: otherwise every address below is loop
          // invariant, gets hoisted out of the tile loop and spilled, and its reloads cost a memory round trip each.
          int r31 = l31, rhi = lhi, ln = lane;
          asm volatile("" : "+v"(r31), "+v"(rhi), "+v"(ln));
          // The accumulators are read where they are, in the accumulation registers, by an instruction the compiler
          // cannot merge with the reads of the other way: left to it, it keeps copies of whole accumulator blocks in
          // ordinary registers from one use to the next and spills them.  The matrix pipe's last write is long
          // finished (a workgroup barrier lies in between); the wait states make that formal, since the compiler's
          // own hazard handling does not look into assembly.
          float rsv[MI];
          if (RS) { __builtin_amdgcn_s_waitcnt(0xc07f); __builtin_amdgcn_wave_barrier(); }   // the factors are in LDS
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) rsv[mi] = RS ? rsbuf[mi * 32 + r31] : 1.0f;
          asm volatile("s_nop 15\n\ts_nop 15");
          auto rd = [&](int ni, int mi, int r) {
            float x;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(acc[ni][mi][r]));
            return x;
          };
#pragma unroll
          for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                bf16x4 pk;
#pragma unroll
                for (int i = 0; i < 4; ++i) pk[i] = (bf16)(silu_f(rd(ni, mi, q * 4 + i) * rsv[mi]) * (rd(ni + 2, mi, q * 4 + i) * rsv[mi]));
                const int row = mi * 32 + r31;
                *reinterpret_cast<bf16x4*>(patch + row * 128 + (((ni * 4 + q) ^ ((r31 >> 1) & 7)) << 4) + rhi * 8) = pk;
                if (q == 3) SV_SB;                       // one feature block at a time
              }
          __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0): the patch is complete before it is read back
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int it = 0; it < 16; ++it) {
            const int row = it * 8 + (ln >> 3), cc = ln & 7;
            const bf16x8 v = *reinterpret_cast<const bf16x8*>(patch + row * 128 + ((cc ^ ((row >> 1) & 7)) << 4));
            const int m = m0 + wm * 128 + row;
            if (CHECK && m >= M) continue;
            *reinterpret_cast<bf16x8*>((bf16*)a.C + (int64_t)m * a.ldc + n0 + wn * 64 + cc * 8) = v;
            if ((it & 3) == 3) SV_SB;
          }
          return;
        }
      }
      // The lane's row and chunk numbers in the patch are made opaque once per tile, as above: the patch addresses below
      // are the same for every tile, and kept in registers across the k loop they crowd the epilogue's inputs out.
      int e31 = l31, eer = er, ec = ec4;
      asm volatile("" : "+v"(e31), "+v"(eer), "+v"(ec));
      if (kHasInputs && CHECK) {                         // a ragged tile asks for its first inputs here, a full one did so a slice ago
#pragma unroll
        for (int t = 0; t < PD; ++t) load_inputs(check_tag, t, in_lo[t], in_hi[t]);
      }
#pragma unroll
      for (int trip = 0; trip < 16; ++trip) {
        const int mi = trip >> 2, it = (trip & 3) * 2;
        if ((trip & 3) == 0) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              f32x4 v;
#pragma unroll
              for (int i = 0; i < 4; ++i) v[i] = acc[ni][mi][q * 4 + i];
              const int chunk = ni * 8 + q * 2 + lhi;    // features 4*chunk .. +3 of the wave's 128
              *reinterpret_cast<f32x4*>(patch + e31 * 512 + ((chunk ^ e31) << 4)) = v;
            }
          __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0): the patch is complete before it is read back
          __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          const int row = (it + k) * 4 + eer, rb = mi * 32 + (it + k) * 4;
          const f32x4 a_lo = *reinterpret_cast<const f32x4*>(patch + row * 512 + ((ec ^ row) << 4));
          const f32x4 a_hi = *reinterpret_cast<const f32x4*>(patch + row * 512 + (((16 + ec) ^ row) << 4));
          float lo[4], hi[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) { lo[i] = a_lo[i]; hi[i] = a_hi[i]; }
          const bool ok = !CHECK || wm * 128 + rb + er < M - m0;
          if constexpr (SPLIT) {                       // the bare accumulators: 16 lanes x 16 bytes = 256 contiguous bytes of a row, twice
            int vo = vW, so = rb * a.N * 4;
            if (CHECK) { vo = (min(wm * 128 + rb + er, M - 1 - m0) * a.N + ec4 * 4) * 4; so = 0; }
            if (ok) {
              __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, a_lo), bW, vo, so, 0);
              __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, a_hi), bW, vo + 256, so, 0);
            }
            continue;
          }
          int vo, so;
          place(check_tag, rb, a.ldc, vC, vo, so);
          auto put_lo = [&](int w, bf16x4 pk) {
            if (ok) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, pk), w == 0 ? bC : w == 1 ? bC2 : bC3, vo, so, 0);
          };
          auto put_hi = [&](int w, bf16x4 pk) {
            if (ok) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, pk), w == 0 ? bC : w == 1 ? bC2 : bC3, vo + 128, so, 0);
          };
          const float rs = RS ? rsbuf[mi * 32 + row] : 1.0f;
          const EpiIn& i_lo = in_lo[trip % PD][k];
          const EpiIn& i_hi = in_hi[trip % PD][k];
          if (DUAL) epilogue_math4<EPI>(a, false, lo, hi, i_lo, rs, put_lo);   // patch columns 0..63: gate, 64..127: up
          else {
            float sq = epilogue_math4<EPI>(a, EPI == EPI_ROPE && ncol0 + ec4 * 4 < a.rope_cols, lo, hi, i_lo, rs, put_lo);
            sq += epilogue_math4<EPI>(a, EPI == EPI_ROPE && ncol0 + 64 + ec4 * 4 < a.rope_cols, hi, lo, i_hi, rs, put_hi);
            if (SQ) {
              // the 16 lanes of a row hold its 128 stored values: rotate-and-add within the row of 16 lanes leaves the
              // sum in all of them, and all of them write it (one LDS address per row, no per-lane condition)
              sq += dpp_row_ror<8>(sq); sq += dpp_row_ror<4>(sq); sq += dpp_row_ror<2>(sq); sq += dpp_row_ror<1>(sq);
              if (ok) sqbuf[mi * 32 + row] = sq;
            }
          }
        }
        if (kHasInputs && trip + PD < 16) load_inputs(check_tag, trip + PD, in_lo[trip % PD], in_hi[trip % PD]);
      }
      if (SQ) {                                          // 128 consecutive floats of plane (n0 / 128 + wn): two full-line stores
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_wave_barrier();
        float* plane = a.rowsq + (int64_t)((n0 >> 7) + wn) * a.rowsq_ld + m0 + wm * 128;
        if (!CHECK || m0 + wm * 128 + lane < M) plane[lane] = sqbuf[lane];
        if (!CHECK || m0 + wm * 128 + 64 + lane < M) plane[64 + lane] = sqbuf[64 + lane];
      }
    };
    if (m0 + 256 <= M) run_epilogue(std::false_type{});
    else run_epilogue(std::true_type{});
  }
  // A finished stream keeps re-reading its last slice into the free stage (the loop has no branch for it): every
  // such load must have landed before the workgroup gives its LDS back.
  __builtin_amdgcn_s_waitcnt(0);
#undef SV_SB
}

template <int EPI, bool GROUPED, bool NF = false>
hipError_t launch_dma(const GemmArgs& a, hipStream_t st) {
  auto kern = gemm_mfma_dma_kernel<EPI, GROUPED, NF>;
  constexpr int lds = 2 * 512 * 128 + 4 * 1024;           // two stages, and per wave 128 row factors + 128 row sums
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (a.M + 255) / 256, tiles_n = a.N / (EPI == EPI_SWIGLU ? 128 : 256);
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  static int n_cu = 0;                                   // one persistent workgroup per CU (128 KB of LDS each)
  if (n_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorUnknown;
    n_cu = (prop.multiProcessorCount / 8) * 8;
    if (n_cu < 8) n_cu = 8;
  }
  const int grid = per_xcd * 8 < n_cu ? per_xcd * 8 : n_cu;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, a, tiles_m, tiles_n, 1);
  return hipGetLastError();
}

// the 256 x 256 kernel over nsplit runs of k slices per tile, then the reduction with the epilogue
template <int EPI>
hipError_t launch_dma_split(const GemmArgs& a, int nsplit, hipStream_t st) {
  auto kern = gemm_mfma_dma_kernel<EPI_STORE, false, false, true>;
  constexpr int lds = 2 * 512 * 128 + 4 * 1024;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (a.M + 255) / 256, tiles_n = a.N / 256;
  const int per_xcd = (tiles_m * tiles_n * nsplit + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(256), lds, st, a, tiles_m, tiles_n, nsplit);   // at most one workgroup per CU
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t threads = (int64_t)a.M * (a.N / 4);
  hipLaunchKernelGGL(splitk_reduce_kernel<EPI>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, a, nsplit);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool KN, int EPI>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t st) {
  using C = Cfg<BM, BN, WAVES_M, WAVES_N, KN, EPI == EPI_SWIGLU>;
  auto kern = gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, KN, EPI>;
  static bool configured = false;   // per process; the attribute is per function
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = a.N / C::NOUT;
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(C::NT), C::LDS, st, a, tiles_m, tiles_n);
  return hipGetLastError();
}

// 128 x 64 tiles, nsplit runs of k slices each, then the reduction with the epilogue
template <int EPI>
hipError_t launch_split(const GemmArgs& a, int nsplit, hipStream_t st) {
  using C = Cfg<128, 64, 2, 2, false, false>;
  auto kern = gemm_mfma_kernel<128, 64, 2, 2, false, EPI_STORE, true>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (a.M + 127) / 128, tiles_n = a.N / 64;
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8, nsplit), dim3(C::NT), C::LDS, st, a, tiles_m, tiles_n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t threads = (int64_t)a.M * (a.N / 4);
  hipLaunchKernelGGL(splitk_reduce_kernel<EPI>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, a, nsplit);
  return hipGetLastError();
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Tile choice: the 256x256 tile has the best LDS-traffic-to-MFMA ratio; fall back to 128x128
// when the large tile would leave most of the 256 CUs without work.
bool use_big_tile(const GemmArgs& a) {
  const int nout = a.epi == EPI_SWIGLU ? 128 : 256;
  if (a.N % nout) return false;
  const int64_t tiles = (int64_t)((a.M + 255) / 256) * (a.N / nout);
  return tiles >= 192;
}


// Few tiles of 256 x 256 (few tokens against a wide projection): how many runs of k slices per tile bring the direct-to-LDS
// kernel to about one workgroup per CU, or 0 where that form does not apply (no scratch for the partial products, the
// dual or grouped product, fewer than 4 slices per run).  A 256-CU part is assumed: the rule only shapes the launch.
int dma_split_runs(const GemmArgs& a) {
  if (!a.split_ws || a.b_is_kn || a.tile_group || a.epi == EPI_SWIGLU || a.rowsq || a.N % 256) return 0;
  const int64_t tiles = (int64_t)((a.M + 255) / 256) * (a.N / 256);
  if (tiles >= 192) return 0;
  int slices = 0;
  for (int s = 0; s < a.nseg; ++s) {
    slices += a.seg[s].K / BK;
    if (!(256 * a.seg[s].lda * 2 < (int64_t)1 << 32 && 256 * a.seg[s].ldb * 2 < (int64_t)1 << 32)) return 0;
  }
  int64_t n = std::min<int64_t>(std::min<int64_t>(8, 256 / tiles), slices / 4);
  n = std::min<int64_t>(n, a.split_ws_floats / ((int64_t)a.M * a.N));
  return n >= 2 ? (int)n : 0;
}

}  // namespace

namespace {
// the 256 x 256 direct-to-LDS kernel serves this product (the DMA offsets are 32-bit byte offsets within a 256-row panel)
bool takes_dma_kernel(const GemmArgs& a) {
  if (a.b_is_kn || !use_big_tile(a)) return false;
  for (int s = 0; s < a.nseg; ++s)
    if (!(256 * a.seg[s].lda * 2 < (int64_t)1 << 32 && 256 * a.seg[s].ldb * 2 < (int64_t)1 << 32)) return false;
  return !(a.epi == EPI_SWIGLU && a.ldc % 8);            // its epilogue stores 16 bytes per lane
}
}  // namespace

bool mfma_gemm_emits_rowsq(const GemmArgs& a) {
  return a.rowsq && a.epi == EPI_RESID && !a.tile_group && mfma_gemm_supported(a) && takes_dma_kernel(a);
}

bool mfma_gemm_supported(const GemmArgs& a) {
  if (a.M < 1 || a.nseg < 1 || a.nseg > 3) return false;
  if (a.rscale && (a.tile_group || (a.epi != EPI_STORE && a.epi != EPI_GELU && a.epi != EPI_SWIGLU && a.epi != EPI_ROPE))) return false;
  if (a.rowsq && (a.epi != EPI_RESID || a.rowsq_ld < a.M)) return false;
  const bool dual = a.epi == EPI_SWIGLU;
  if (dual && (a.b_is_kn || a.nseg != 1 || !a.B2 || a.ldb2 % 8 || !aligned16(a.B2))) return false;
  if (a.epi < EPI_STORE || a.epi > EPI_ROPE) return false;
  if (a.nbcol > 0 || a.epi == EPI_ROPE) {
    // fused QKV form: served by the 256x256 direct-to-LDS kernel only (whole tiles, or runs of k slices for few tiles)
    if (a.b_is_kn || a.nseg != 1 || a.nbcol > 3 || a.N % 256 || !(use_big_tile(a) || dma_split_runs(a))) return false;
    int tot = 0;
    for (int j = 0; j < a.nbcol; ++j) { if (a.ncol[j] % 256 || !aligned16(a.Bcol[j])) return false; tot += a.ncol[j]; }
    if (a.nbcol > 0 && tot != a.N) return false;
    if (a.epi == EPI_ROPE && (!a.rope_cs || a.rope_hd % 4 || a.rope_cols % 4 || a.rope_S < 1)) return false;
  }
  if ((a.tile_group != nullptr) != (a.m_dev != nullptr)) return false;      // the grouped form needs both
  if (a.tile_group && (a.nbcol > 0 || a.group_stride % 8 || a.M % 256)) return false;
  if (a.tile_group && a.epi != EPI_STORE && a.epi != EPI_SWIGLU && a.epi != EPI_SWIGLU_BWD) return false;
  if (a.b_is_kn && (a.epi == EPI_RESID || a.epi == EPI_GELU || a.epi == EPI_SWIGLU)) return false;
  if ((a.epi == EPI_RESID || a.epi == EPI_SWIGLU_BWD || a.epi == EPI_GELU_BWD) && !a.R) return false;
  if (a.epi == EPI_SWIGLU_BWD && (!a.R2 || !a.C2)) return false;
  if (a.N % (dual ? 64 : 128)) return false;
  if (a.ldc % 4 || !aligned16(a.C)) return false;
  if ((a.C2 && !aligned16(a.C2)) || (a.C3 && !aligned16(a.C3))) return false;
  if ((a.R || a.R2) && (a.ldr % 4 || !aligned16(a.R) || (a.R2 && !aligned16(a.R2)))) return false;
  for (int s = 0; s < a.nseg; ++s) {
    const GemmSeg& g = a.seg[s];
    if (g.K < BK || g.K % BK || g.lda % 8 || g.ldb % 8 || !aligned16(g.A) || !aligned16(g.B)) return false;
  }
  return true;
}

hipError_t mfma_gemm(const GemmArgs& a, hipStream_t st, int tile) {
  if (!mfma_gemm_supported(a)) return hipErrorInvalidValue;
  if ((tile == 1 || tile == 3) && a.N % (a.epi == EPI_SWIGLU ? 128 : 256)) return hipErrorInvalidValue;
  const bool big = tile == 1 || tile == 3 || (tile == 0 && use_big_tile(a));
  if (!a.b_is_kn && big && tile != 3) {
    bool fits = true;                                      // as in takes_dma_kernel, for a forced tile too
    for (int s = 0; s < a.nseg; ++s) fits = fits && 256 * a.seg[s].lda * 2 < (int64_t)1 << 32 && 256 * a.seg[s].ldb * 2 < (int64_t)1 << 32;
    if (a.epi == EPI_SWIGLU && a.ldc % 8) fits = false;       // its epilogue stores 16 bytes per lane
    if (fits) {
      if (a.tile_group) {
        switch (a.epi) {                                   // the epilogues the mixture-of-experts products use
          case EPI_STORE: return launch_dma<EPI_STORE, true>(a, st);
          case EPI_SWIGLU: return launch_dma<EPI_SWIGLU, true>(a, st);
          case EPI_SWIGLU_BWD: return launch_dma<EPI_SWIGLU_BWD, true>(a, st);
          default: return hipErrorInvalidValue;
        }
      }
      if (a.rscale || a.rowsq) {
        switch (a.epi) {                                   // the ends of a norm that runs inside the products
          case EPI_STORE: return launch_dma<EPI_STORE, false, true>(a, st);
          case EPI_RESID: return launch_dma<EPI_RESID, false, true>(a, st);
          case EPI_GELU: return launch_dma<EPI_GELU, false, true>(a, st);
          case EPI_SWIGLU: return launch_dma<EPI_SWIGLU, false, true>(a, st);
          case EPI_ROPE: return launch_dma<EPI_ROPE, false, true>(a, st);
          default: return hipErrorInvalidValue;
        }
      }
      switch (a.epi) {
        case EPI_STORE: return launch_dma<EPI_STORE, false>(a, st);
        case EPI_RESID: return launch_dma<EPI_RESID, false>(a, st);
        case EPI_GELU: return launch_dma<EPI_GELU, false>(a, st);
        case EPI_SWIGLU: return launch_dma<EPI_SWIGLU, false>(a, st);
        case EPI_SWIGLU_BWD: return launch_dma<EPI_SWIGLU_BWD, false>(a, st);
        case EPI_GELU_BWD: return launch_dma<EPI_GELU_BWD, false>(a, st);
        case EPI_ROPE: return launch_dma<EPI_ROPE, false>(a, st);
        default: return hipErrorInvalidValue;
      }
    }
  }
  if (tile == 0) {
    // few tokens: the large tile over runs of k slices, about one workgroup per CU, instead of small tiles
    const int runs = dma_split_runs(a);
    if (runs) {
      switch (a.epi) {
        case EPI_STORE: return launch_dma_split<EPI_STORE>(a, runs, st);
        case EPI_RESID: return launch_dma_split<EPI_RESID>(a, runs, st);
        case EPI_GELU: return launch_dma_split<EPI_GELU>(a, runs, st);
        case EPI_SWIGLU_BWD: return launch_dma_split<EPI_SWIGLU_BWD>(a, runs, st);
        case EPI_GELU_BWD: return launch_dma_split<EPI_GELU_BWD>(a, runs, st);
        case EPI_ROPE: return launch_dma_split<EPI_ROPE>(a, runs, st);
        default: return hipErrorInvalidValue;
      }
    }
  }
  if (a.nbcol > 0 || a.epi == EPI_ROPE) return hipErrorInvalidValue;   // only the direct-to-LDS kernel implements these
  if (!a.b_is_kn) {
    // Few rows (a 512-token micro-batch against a 4096-wide projection is 128 tiles of 128 x 128 for 256 CUs):
    // 128 x 64 tiles double the workgroups.
    const bool narrow = !big && !a.tile_group && a.epi != EPI_SWIGLU &&
                        (tile == 4 || (tile == 0 && (int64_t)((a.M + 127) / 128) * (a.N / 128) < 160));
    if (narrow) {
      // Long k with few workgroups (the down-projection of a 512-token micro-batch: 256 workgroups x 224 slices):
      // split k so that about three workgroups share a CU and cover each other's load-to-multiply latency.
      int slices = 0;
      for (int s = 0; s < a.nseg; ++s) slices += a.seg[s].K / BK;
      const int64_t wgs = (int64_t)((a.M + 127) / 128) * (a.N / 64);
      int nsplit = (int)std::min<int64_t>(std::min<int64_t>(8, slices / 8), (768 + wgs - 1) / wgs);
      if (a.split_ws) nsplit = (int)std::min<int64_t>(nsplit, a.split_ws_floats / ((int64_t)a.M * a.N));
      if (a.split_ws && tile == 0 && nsplit >= 2) {
        switch (a.epi) {
          case EPI_STORE: return launch_split<EPI_STORE>(a, nsplit, st);
          case EPI_RESID: return launch_split<EPI_RESID>(a, nsplit, st);
          case EPI_GELU: return launch_split<EPI_GELU>(a, nsplit, st);
          case EPI_SWIGLU_BWD: return launch_split<EPI_SWIGLU_BWD>(a, nsplit, st);
          case EPI_GELU_BWD: return launch_split<EPI_GELU_BWD>(a, nsplit, st);
          default: return hipErrorInvalidValue;
        }
      }
      switch (a.epi) {
        case EPI_STORE: return launch_cfg<128, 64, 2, 2, false, EPI_STORE>(a, st);
        case EPI_RESID: return launch_cfg<128, 64, 2, 2, false, EPI_RESID>(a, st);
        case EPI_GELU: return launch_cfg<128, 64, 2, 2, false, EPI_GELU>(a, st);
        case EPI_SWIGLU_BWD: return launch_cfg<128, 64, 2, 2, false, EPI_SWIGLU_BWD>(a, st);
        case EPI_GELU_BWD: return launch_cfg<128, 64, 2, 2, false, EPI_GELU_BWD>(a, st);
        default: return hipErrorInvalidValue;
      }
    }
    switch (a.epi) {
      case EPI_STORE: return big ? launch_cfg<256, 256, 2, 2, false, EPI_STORE>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_STORE>(a, st);
      case EPI_RESID: return big ? launch_cfg<256, 256, 2, 2, false, EPI_RESID>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_RESID>(a, st);
      case EPI_GELU: return big ? launch_cfg<256, 256, 2, 2, false, EPI_GELU>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_GELU>(a, st);
      case EPI_SWIGLU: return big ? launch_cfg<256, 256, 2, 2, false, EPI_SWIGLU>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_SWIGLU>(a, st);
      case EPI_SWIGLU_BWD: return big ? launch_cfg<256, 256, 2, 2, false, EPI_SWIGLU_BWD>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_SWIGLU_BWD>(a, st);
      case EPI_GELU_BWD: return big ? launch_cfg<256, 256, 2, 2, false, EPI_GELU_BWD>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_GELU_BWD>(a, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (a.epi) {
    case EPI_STORE: return big ? launch_cfg<256, 256, 2, 2, true, EPI_STORE>(a, st) : launch_cfg<128, 128, 2, 1, true, EPI_STORE>(a, st);
    case EPI_SWIGLU_BWD: return big ? launch_cfg<256, 256, 2, 2, true, EPI_SWIGLU_BWD>(a, st) : launch_cfg<128, 128, 2, 1, true, EPI_SWIGLU_BWD>(a, st);
    case EPI_GELU_BWD: return big ? launch_cfg<256, 256, 2, 2, true, EPI_GELU_BWD>(a, st) : launch_cfg<128, 128, 2, 1, true, EPI_GELU_BWD>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sv
