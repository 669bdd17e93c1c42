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
#include "common.h"

namespace sv {
namespace {

constexpr int BK = 64;
constexpr int kGroupM = 4;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ swz(row)) << 4); }

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

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

// 4 consecutive output features of one token row.
template <int EPI>
__device__ __forceinline__ void epilogue4(const GemmArgs& a, int m, int n, const float (&v)[4], const float (&u)[4]) {
  const int64_t ic = (int64_t)m * a.ldc + n, ir = (int64_t)m * a.ldr + n;
  float o[4];
  switch (EPI) {
    case EPI_STORE:
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i];
      break;
    case EPI_RESID: {
      const bf16x4 r = *reinterpret_cast<const bf16x4*>((const bf16*)a.R + ir);
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i] + (float)r[i];
    } break;
    case EPI_GELU: {
      if (a.C2) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)v[i]; *reinterpret_cast<bf16x4*>((bf16*)a.C2 + ic) = p; }
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = gelu_f(v[i]);
    } break;
    case EPI_SWIGLU: {
      if (a.C2) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)v[i]; *reinterpret_cast<bf16x4*>((bf16*)a.C2 + ic) = p; }
      if (a.C3) { bf16x4 p; for (int i = 0; i < 4; ++i) p[i] = (bf16)u[i]; *reinterpret_cast<bf16x4*>((bf16*)a.C3 + ic) = p; }
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = silu_f(v[i]) * u[i];
    } break;
    case EPI_SWIGLU_BWD: {
      const bf16x4 g = *reinterpret_cast<const bf16x4*>((const bf16*)a.R + ir);
      const bf16x4 w = *reinterpret_cast<const bf16x4*>((const bf16*)a.R2 + ir);
      bf16x4 p;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gf = (float)g[i];
        o[i] = v[i] * (float)w[i] * silu_grad_f(gf);
        p[i] = (bf16)(v[i] * silu_f(gf));
      }
      *reinterpret_cast<bf16x4*>((bf16*)a.C2 + ic) = p;
    } break;
    default: {  // EPI_GELU_BWD
      const bf16x4 r = *reinterpret_cast<const bf16x4*>((const bf16*)a.R + ir);
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = v[i] * gelu_grad_f((float)r[i]);
    } break;
  }
  bf16x4 p;
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = (bf16)o[i];
  *reinterpret_cast<bf16x4*>((bf16*)a.C + ic) = p;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool KN, int EPI>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_mfma_kernel(GemmArgs a, int tiles_m, int tiles_n) {
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  using C = Cfg<BM, BN, WAVES_M, WAVES_N, KN, DUAL>;
  extern __shared__ __attribute__((aligned(16))) char smem[];

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

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  // ---- global -> register staging
  bf16x8 xreg[C::XCH], wreg[C::WCH];
  int seg = 0, kin = 0;       // position of the slice being loaded
  auto load_slice = [&]() {
    const bf16* A = (const bf16*)a.seg[seg].A;
    const int64_t lda = a.seg[seg].lda, ldb = a.seg[seg].ldb;
#pragma unroll
    for (int i = 0; i < C::XCH; ++i) {
      const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
      const int m = min(m0 + r, a.M - 1);
      xreg[i] = *reinterpret_cast<const bf16x8*>(A + (int64_t)m * lda + kin + c * 8);
    }
    if (!KN) {
#pragma unroll
      for (int i = 0; i < C::WCH; ++i) {
        const int e = tid + i * C::NT, r = e >> 3, c = e & 7;
        const bf16* B;
        int n;
        if (DUAL && r >= BN / 2) { B = (const bf16*)a.B2; n = n0 + r - BN / 2; }
        else { B = (const bf16*)a.seg[seg].B; n = n0 + r; }
        const int64_t ld = (DUAL && r >= BN / 2) ? a.ldb2 : ldb;
        wreg[i] = *reinterpret_cast<const bf16x8*>(B + (int64_t)n * ld + kin + c * 8);
      }
    } else {
      // thread owns 8x8 blocks: 8 consecutive k rows x 8 consecutive n columns
      const bf16* B = (const bf16*)a.seg[seg].B;
#pragma unroll
      for (int b = 0; b < C::WCH / 8; ++b) {
        const int blk = tid + b * C::NT, ng = blk % (BN / 8), kg = blk / (BN / 8);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          wreg[b * 8 + j] = *reinterpret_cast<const bf16x8*>(B + (int64_t)(kin + kg * 8 + j) * ldb + n0 + ng * 8);
      }
    }
    kin += BK;
    if (kin >= a.seg[seg].K) { kin = 0; ++seg; }
  };
  auto store_slice = [&](int stage) {
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

  load_slice();
  store_slice(0);
  __syncthreads();

  for (int kt = 0; kt < nslices; ++kt) {
    const bool more = kt + 1 < nslices;
    if (more) load_slice();
    const char* xs = smem + (kt & 1) * C::STAGE;
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
    if (more) store_slice((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: lane owns token row (lane & 31) of each 32-row block and, per register
  // quad q, output features 8q + 4*(lane>>5) .. +3 of each 32-feature block.
  constexpr int NIO = DUAL ? C::NI / 2 : C::NI;
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi) {
    const int m = m0 + wm * C::WTM + mi * 32 + l31;
    if (m >= a.M) continue;
#pragma unroll
    for (int ni = 0; ni < NIO; ++ni) {
      const int nb = n0 + wn * (DUAL ? C::WTN / 2 : C::WTN) + ni * 32 + lhi * 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4], u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = acc[ni][mi][q * 4 + i];
          u[i] = DUAL ? acc[ni + NIO][mi][q * 4 + i] : 0.0f;
        }
        epilogue4<EPI>(a, m, nb + q * 8, v, u);
      }
    }
  }
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

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Tile choice: the 256x256 tile has the best LDS-traffic-to-MFMA ratio; fall back to 128x128
// when the large tile would leave most of the 256 CUs without work.
bool use_big_tile(const GemmArgs& a) {
  const int nout = a.epi == EPI_SWIGLU ? 128 : 256;
  if (a.N % nout) return false;
  const int64_t tiles = (int64_t)((a.M + 255) / 256) * (a.N / nout);
  return tiles >= 192;
}

}  // namespace

bool mfma_gemm_supported(const GemmArgs& a) {
  if (a.M < 1 || a.nseg < 1 || a.nseg > 3) return false;
  const bool dual = a.epi == EPI_SWIGLU;
  if (dual && (a.b_is_kn || a.nseg != 1 || !a.B2 || a.ldb2 % 8 || !aligned16(a.B2))) return false;
  if (a.b_is_kn ? (a.epi != EPI_STORE && a.epi != EPI_SWIGLU_BWD && a.epi != EPI_GELU_BWD)
                : (a.epi != EPI_STORE && a.epi != EPI_RESID && a.epi != EPI_GELU && a.epi != EPI_SWIGLU)) return false;
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
  if (tile == 1 && a.N % (a.epi == EPI_SWIGLU ? 128 : 256)) return hipErrorInvalidValue;
  const bool big = tile == 1 || (tile == 0 && use_big_tile(a));
  if (!a.b_is_kn) {
    switch (a.epi) {
      case EPI_STORE: return big ? launch_cfg<256, 256, 2, 2, false, EPI_STORE>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_STORE>(a, st);
      case EPI_RESID: return big ? launch_cfg<256, 256, 2, 2, false, EPI_RESID>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_RESID>(a, st);
      case EPI_GELU: return big ? launch_cfg<256, 256, 2, 2, false, EPI_GELU>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_GELU>(a, st);
      case EPI_SWIGLU: return big ? launch_cfg<256, 256, 2, 2, false, EPI_SWIGLU>(a, st) : launch_cfg<128, 128, 2, 2, false, EPI_SWIGLU>(a, st);
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
