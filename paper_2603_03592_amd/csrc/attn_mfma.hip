// Causal / full softmax attention of the block recompute on the gfx950 matrix cores
// (bf16 inputs, fp32 scores, softmax statistics and accumulation; head_dim 64 or 128; GQA).
//
// Forward: one workgroup = 128 queries of one (sequence, query head); each of its 4 waves owns
// 32 queries.  Keys/values stream through LDS in tiles of 64, double buffered.  Per tile a wave
// computes the TRANSPOSED score block S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (keys in the
// MFMA row dimension, queries in the column dimension), so every lane owns one query column:
// the running maximum, the running sum and the rescale factor of the online softmax are
// per-lane scalars and only one cross-lane exchange (lane ^ 32) per tile is needed.  The
// probabilities then feed O^T += V^T P^T directly from registers: the accumulator layout of
// S^T is a valid B-operand layout once the 16 keys of an MFMA are taken in the order
// {0-3, 8-11 | 4-7, 12-15}; the V^T fragments come out of the row-major V tile in exactly that key
// order by transposing LDS reads.  The 64 keys of a tile are taken as two halves whose matrix and
// vector instructions are interleaved in the wave's instruction stream (see the tile body).
#include "common.h"
#include <type_traits>

namespace sv {
namespace {

constexpr int BQ = 128, BKV = 64;

// Workgroup id -> (batch, head, tile) for the kernels that stream the keys / values of one (batch, kv head) pair.
// Workgroup ids go round-robin over the 8 XCDs, each with its own L2; ids congruent mod 8 are therefore given whole
// (batch, kv head) pairs, so that the G query heads and all tiles that read one pair's K / V run on ONE XCD and find
// them in its L2 (1 MB per pair at S = 2048, head_dim 128) instead of every XCD streaming every pair from HBM.  Within
// a pair: tiles in descending order (the longest causal rows first), the G heads of a tile next to each other.
// Returns false for the padding ids of an XCD with fewer pairs.
__device__ __forceinline__ bool xcd_map(int w, int n_tiles, int G, int Hkv, int B, int& tile_rank, int& h, int& b) {
  const int xcd = w & 7, i = w >> 3, per_pair = G * n_tiles;
  const int pair = (i / per_pair) * 8 + xcd;
  if (pair >= B * Hkv) return false;
  const int rem = i % per_pair;
  tile_rank = rem / G;
  h = (pair % Hkv) * G + rem % G;
  b = pair / Hkv;
  return true;
}
inline int xcd_grid(int n_tiles, int G, int Hkv, int B) { return 8 * ((B * Hkv + 7) / 8) * G * n_tiles; }

// Under the causal mask the work of a tile grows linearly with its index, and a launch of one workgroup per tile ends
// with most CUs waiting for the few longest ones (at 8 x 1024 tokens, 16 heads, half of the wave slots were empty on
// average).  A workgroup therefore takes TWO tiles, r and n - 1 - r, one after the other, so that every workgroup does
// the same amount of work.  Workgroups per (batch, head) -- the middle tile of an odd count stands alone -- and tiles
// of workgroup r:
inline bool pair_tiles(int causal, int n_tiles) { return causal && n_tiles > 1; }
__host__ __device__ __forceinline__ int paired_tiles(bool pair, int n) { return pair ? (n + 1) / 2 : n; }
__device__ __forceinline__ int n_passes(bool pair, int n, int r) { return pair && 2 * r != n - 1 ? 2 : 1; }

typedef __attribute__((ext_vector_type(4))) short s16x4;
#define LDS __attribute__((address_space(3)))

// Position of 16-byte chunk c inside row `row` of a row-major LDS tile (an involution in c, so the staging side uses
// the same function to pick the chunk that belongs at a position).  The LDS serves 256 bytes per clock, and a tile is
// read in two ways: fragments along the rows (16 consecutive rows, one chunk index, 16 bytes per lane) and transposed
// fragments through ds_read_b64_tr_b16 (32 lanes: 4 consecutive rows x 4 consecutive chunks, 8 bytes per lane).  With
// the two 2-bit fields of the row number swapped into the XOR mask both patterns fall into 16 different 16-byte slots
// modulo 256 bytes (rows of 128 bytes, head_dim 64: the row parity is one slot bit, the mask has three bits; rows of
// 64 bytes, head_dim 32: two slot bits, two mask bits).
//
// SW = 1 is the layout of the kernel on the 16x16x32 shape, whose reads group the lanes differently: fragments along the
// rows take 16 consecutive rows x one chunk per 16 lanes, and a transposing read takes, per 32 lanes, 8 consecutive rows x
// 2 consecutive chunks.  There the row's low bits go to the mask's upper bits (bit 0 of the chunk index tells the two
// chunks of a transposing read apart and must not meet a row bit that varies among its 8 rows) and row bit 3 to bit 0.
template <int HD, int SW = 0> __device__ __forceinline__ int rm_pos(int c, int row) {
  if (SW == 1) {
    if (HD == 128) return c ^ (((row & 7) << 1) | ((row >> 3) & 1));
    if (HD == 64) return c ^ ((((row >> 1) & 3) << 1) | ((row >> 3) & 1));     // rows of 128 bytes: row bit 0 is a slot bit
    return c ^ ((((row >> 2) & 1) << 1) | ((row >> 3) & 1));                    // rows of 64 bytes: row bits 0, 1 are slot bits
  }
  if (HD == 32) return c ^ ((row >> 2) & 3);        // rows of 64 bytes: the low two row bits are slot bits already
  return HD == 128 ? (c ^ (((row & 3) << 2) | ((row >> 2) & 3))) : (c ^ ((((row >> 1) & 1) << 2) | ((row >> 2) & 3)));
}

// One direct-to-LDS load of 16 bytes per lane: lane l's bytes go to lds + 16 l (lds wave-uniform).  Issued as inline
// assembly so that it stays outside the compiler's model of memory: with the builtin, the compiler makes every
// transposing LDS read wait (vmcnt(0)) for all direct-to-LDS loads in flight -- it cannot tell that they fill the OTHER
// stage -- and the next tile's loads, issued at the top of a tile, were waited for in the middle of that tile's work.
// The kernels wait for these loads themselves (dma_wait_all) before the barrier that hands a stage over; waits the
// compiler computes for its own loads can only become stricter by loads it does not know of.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"      // m0 is a reserved register: nothing else in these kernels uses it
__device__ __forceinline__ void dma16(const char* g, unsigned off, char* lds) {       // g wave-uniform, off per lane
  const unsigned l = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) char*)lds);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(g), "s"(l) : "memory", "m0");
}
__device__ __forceinline__ void dma16(const char* g_lane, char* lds) {                // per-lane address
  const unsigned l = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) char*)lds);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g_lane), "s"(l) : "memory", "m0");
}
#pragma clang diagnostic pop
// Every direct-to-LDS load of this wave has landed (to be followed by the barrier that publishes the stage).  The builtin,
// not assembly: the compiler then also knows that its own earlier loads have landed and plans no waits for them later,
// which the loads it does not know of would turn into waits for the next tile.
__device__ __forceinline__ void dma_wait_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }     // vmcnt(0) only

// Two 64-row tiles (rows r0 .. r0 + 63 of a and of b, HD bf16 each, row pitches lda / ldb, clamped to the last valid
// row) go global -> LDS
// row-major with global_load_lds: no registers, no LDS write instructions.  One wave instruction moves 1 KB = RPI rows;
// lane (row, position p) fetches the 16-byte chunk that belongs at position p of its row under rm_pos.  256 threads.
template <int HD, int SW = 0>
__device__ __forceinline__ void stage_two_tiles(const bf16* a, int64_t lda, const bf16* b, int64_t ldb, int r0, int last_row, char* ta,
                                                char* tb, int wave, int lane) {
  constexpr int KCH = HD / 8, KROW = HD * 2, RPI = 1024 / KROW, IPW = (64 / RPI) / 4;
  const int s_row = lane / KCH, s_pos = lane % KCH;
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int ii = wave * IPW + i, r = ii * RPI + s_row;
    const int rr = min(r, last_row - r0);                       // row within the tile, clamped to the last valid one
    const int col = rm_pos<HD, SW>(s_pos, r) * 8;
    dma16((const char*)(a + (int64_t)r0 * lda), (unsigned)((int64_t)rr * lda + col) * 2u, ta + ii * 1024);
    dma16((const char*)(b + (int64_t)r0 * ldb), (unsigned)((int64_t)rr * ldb + col) * 2u, tb + ii * 1024);
  }
}

// The same transfer for tiles that lie inside the valid rows, with the per-lane part of the addresses made once per
// kernel: 32-bit byte offsets (row within the tile, swizzled chunk) that are added to a wave-uniform tile pointer, so a
// tile costs its load instructions and a few scalar adds instead of a 64-bit multiply chain per load.
template <int HD, int NW = 4, int SW = 0>
struct TileOffsets {
  static constexpr int KCH = HD / 8, KROW = HD * 2, RPI = 1024 / KROW, IPW = (64 / RPI) / NW;
  unsigned off[IPW];
  __device__ __forceinline__ void init(int64_t ld, int wave, int lane) {
    const int s_row = lane / KCH, s_pos = lane % KCH;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int r = (wave * IPW + i) * RPI + s_row;
      off[i] = (unsigned)((int64_t)r * ld + rm_pos<HD, SW>(s_pos, r) * 8) * 2u;
    }
  }
};
template <int HD, int NW = 4, int SW = 0>
__device__ __forceinline__ void stage_tile_fast(const bf16* tile_rows, const TileOffsets<HD, NW, SW>& o, char* dst, int wave) {
  const char* g = (const char*)tile_rows;           // wave-uniform: first row of the tile
#pragma unroll
  for (int i = 0; i < TileOffsets<HD, NW, SW>::IPW; ++i)
    dma16(g, o.off[i], dst + (wave * TileOffsets<HD, NW, SW>::IPW + i) * 1024);
}

// A-operand fragment of the TRANSPOSE of a row-major 64-row tile, for MFMA g (0..3) of the tile's 64 rows and feature
// block db: the lane gets features db * 32 + (lane & 31) of 8 rows, in the order the score accumulators hold them
// ({0-3, 8-11} of the 16 rows for the lower lane half, {4-7, 12-15} for the upper one).  Transposing LDS read: in each
// group of 16 lanes, lane 4 e + q names 8 bytes (4 features) of row e, and lane i of the group receives feature i of the
// four rows.  Group (lane >> 4): feature sub-block (group & 1) * 16, row half group >> 1 -- the operand's own lane map.
template <int HD>
__device__ __forceinline__ bf16x8 tr_fragment(const char* tile, int g, int db, int lane) {
  const int tr_e = (lane & 15) >> 2, tr_q = lane & 3, tr_nb = (lane >> 4) & 1, half = lane >> 5;
  bf16x8 f;
#pragma unroll
  for (int r2 = 0; r2 < 2; ++r2) {
    const int row = (g >> 1) * 32 + (g & 1) * 16 + r2 * 8 + half * 4 + tr_e;
    const int chunk = db * 4 + tr_nb * 2 + (tr_q >> 1);
    const bf16x4 t4 = __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(tile + row * (HD * 2) + (rm_pos<HD>(chunk, row) << 4) + (tr_q & 1) * 8)));
#pragma unroll
    for (int i = 0; i < 4; ++i) f[r2 * 4 + i] = t4[i];
  }
  return f;
}

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv, int64_t ld, bf16* __restrict__ o,
                                                            float* __restrict__ lse, int B, int S, int H, int Hkv, float scale_log2e, int pair) {
  constexpr int KCH = HD / 8;                       // 16-byte chunks per K row
  constexpr int KROW = HD * 2;                      // bytes per K row in LDS
  constexpr int KSTAGE = BKV * KROW, VSTAGE = BKV * KROW, STAGE = KSTAGE + VSTAGE;
  constexpr int NKK = HD / 16, NDB = HD / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int nqt = (S + BQ - 1) / BQ;
  int rank, h, b;
  if (!xcd_map((int)blockIdx.x, paired_tiles(pair, nqt), H / Hkv, Hkv, B, rank, h, b)) return;
  const int kvh = h / (H / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, half = lane >> 5;
  const int Dq = H * HD, Dkv = Hkv * HD;
  TileOffsets<HD> toff;
  toff.init(ld, wave, lane);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // Per-lane LDS byte offsets of the fragment reads, made once: the swizzle only looks at the low four bits of a row, so
  // the second 32 keys of a K fragment and the MFMA index of a V^T fragment are immediate offsets from these.
  LDS char* const lds0 = (LDS char*)smem;
  unsigned kbase_l[NKK], vbase_l[NDB][2];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) kbase_l[kk] = l31 * KROW + (rm_pos<HD>(kk * 2 + half, l31) << 4);
  {
    const int tr_e = (lane & 15) >> 2, tr_q = lane & 3, tr_nb = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r2 = 0; r2 < 2; ++r2) {
        const int row = r2 * 8 + half * 4 + tr_e, chunk = db * 4 + tr_nb * 2 + (tr_q >> 1);
        vbase_l[db][r2] = row * KROW + (rm_pos<HD>(chunk, row) << 4) + (tr_q & 1) * 8;
      }
  }
  for (int pass = 0; pass < n_passes(pair, nqt, rank); ++pass) {
  const int qt = pass == 0 ? nqt - 1 - rank : rank;
  const int q0 = qt * BQ, wq0 = q0 + wave * 32;
  const bf16* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * HD;
  const bf16* kbase = qkv + (int64_t)b * S * ld + Dq + (int64_t)kvh * HD;
  const bf16* vbase = kbase + Dkv;

  bf16x8 qf[NKK];
  {
    const int qrow = min(wq0 + l31, S - 1);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qbase + (int64_t)qrow * ld + kk * 16 + half * 8);
  }

  const int nkv = (S + BKV - 1) / BKV;
  const int ntiles = CAUSAL ? min((q0 + BQ + BKV - 1) / BKV, nkv) : nkv;

  auto stage_tile = [&](int j, int stage) {
    char* ks = smem + stage * STAGE;
    if ((j + 1) * BKV <= S) {                        // whole tile inside the sequence (uniform)
      stage_tile_fast<HD>(kbase + (int64_t)j * BKV * ld, toff, ks, wave_u);
      stage_tile_fast<HD>(vbase + (int64_t)j * BKV * ld, toff, ks + KSTAGE, wave_u);
    } else {
      stage_two_tiles<HD>(kbase, ld, vbase, ld, j * BKV, S - 1, ks, ks + KSTAGE, wave, lane);   // keys past the end: masked later
    }
  };

  f32x16 oacc[NDB];
#pragma unroll
  for (int i = 0; i < NDB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;             // in units of log2: scores are scaled by scale*log2(e)
  const int myq = wq0 + l31;

  stage_tile(0, 0);
  dma_wait_all();
  __syncthreads();

  for (int j = 0; j < ntiles; ++j) {
    const bool more = j + 1 < ntiles;
    const int k0 = j * BKV;
    const bool wave_active = !CAUSAL || k0 <= wq0 + 31;
    // The next tile's loads: a wave that computes issues them one behind each MFMA of its first phase, where it would
    // otherwise wait for the matrix pipe (issued in a row they held the wave for some 450 cycles per tile: the
    // instruction stream of a wave is in order, and the load path takes a 1 KB instruction every 16 cycles at best).
    // Causal kernels only: the unmasked kernel's loop is laid out differently by the compiler, and there the second
    // copy of the tile body that this takes costs registers it does not have (spills inside the loop).
    const bool spread = CAUSAL && more && wave_active && (j + 2) * BKV <= S;
    if (more && !spread) stage_tile(j + 1, (j + 1) & 1);
    auto tile_body = [&](auto spread_c) {
      constexpr bool SPREAD = decltype(spread_c)::value;
      const unsigned so = (unsigned)(j & 1) * STAGE;   // this tile's stage: K at so, V at so + KSTAGE
      const bool need_mask = (CAUSAL && k0 + BKV - 1 > wq0) || (k0 + BKV > S);
      // The tile's 64 keys are taken as two halves t of 32, and a wave issues its instructions in order, so the vector
      // work of one half is written BETWEEN the matrix instructions of the other: each MFMA (32 cycles in the matrix
      // pipe) is followed by a slice of about as many cycles of softmax, with scheduling barriers that keep this order.
      //   phase 0: S(0)                      with the next tile's global -> LDS loads
      //   phase A: S(1)  | softmax(0)        with the V^T reads of PV(0)
      //   phase B: PV(0) | softmax(1)        with the V^T reads of PV(1)
      //   phase 3: PV(1)
      // K fragments run two MFMAs ahead through phases 0 and A.
      auto kread = [&](int i) {                        // i = t * NKK + kk
        return *reinterpret_cast<const LDS bf16x8*>(lds0 + (kbase_l[i % NKK] + so + (i / NKK) * 32 * KROW));
      };
      auto vread = [&](int g, int db) {                // the V^T fragment of MFMA g, feature block db (see tr_fragment)
        bf16x8 f;
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2) {
          const bf16x4 t4 = __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (LDS s16x4*)(lds0 + (vbase_l[db][r2] + so + KSTAGE + g * 16 * KROW))));
#pragma unroll
          for (int e = 0; e < 4; ++e) f[r2 * 4 + e] = t4[e];
        }
        return f;
      };
      f32x16 s[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[t][r] = 0.0f;
      bf16x8 pf[4];
      float psum = 0.0f;
      // slice i of NS of the softmax of half t: slice 0 masks, takes the maximum and moves the reference if it must,
      // the others take the exponentials of an even share of the 8 element pairs
      float corr = 1.0f;
      auto soft_slice = [&](int t, int i, int NS) {
        if (i == 0) {
          if (need_mask) {                             // one uniform branch: tiles below the diagonal skip all of it
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = k0 + t * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
              if ((CAUSAL && key > myq) || key >= S) s[t][r] = -INFINITY;
            }
          }
          float mx = s[t][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
          const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, mx), __builtin_bit_cast(unsigned, mx), false, false);
          mx = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));     // both lane halves of the query
          // Lazy reference: the running reference m only moves when the maximum grew by more than 2^8 (probabilities
          // then reach at most 256, harmless in bf16 and in the fp32 sums; O / l does not depend on the reference).
          // With the exact maximum some query of the wave moves it in most tiles and all output registers get rescaled.
          const float mx_s = mx * scale_log2e;
          const bool moved = mx_s > m_run + 8.0f;
          corr = 1.0f;
          if (__builtin_amdgcn_ballot_w64(moved) != 0) {
            const float m_new = moved ? mx_s : m_run;
            corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
          }
          psum = 0.0f;
        } else {
          const int p_lo = (8 * (i - 1)) / (NS - 1), p_hi = (8 * i) / (NS - 1);
#pragma unroll
          for (int r = 2 * p_lo; r < 2 * p_hi; ++r) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[t][r], scale_log2e, -m_run));
            psum += p;
            pf[t * 2 + (r >> 3)][r & 7] = (bf16)p;
          }
        }
        // Arithmetic has no place of its own in the instruction order the compiler starts from, and the scheduling
        // barriers only hold what already sits between them: the slice is tied down by passing what it made, and what
        // the next slice reads, through an empty volatile statement.
        asm volatile("" : "+v"(m_run), "+v"(psum));
      };
      // after the phase: the products that were issued between the slices belong to the old reference
      auto soft_end = [&]() {
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
          l_run *= corr;
#pragma unroll
          for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
        l_run += psum;
      };
      constexpr int NPV = 2 * NDB;                    // MFMAs of one half's P V product
      constexpr int KD = 2;                           // K fragments this many MFMAs ahead
      bf16x8 kf[KD + 1], vf[2][NPV];
#pragma unroll
      for (int i = 0; i < KD; ++i) kf[i] = kread(i);
      // phase 0
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        kf[(kk + KD) % (KD + 1)] = kread(kk + KD);
        __builtin_amdgcn_sched_barrier(0);
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk % (KD + 1)], qf[kk], s[0], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (SPREAD) {                                  // NKK = the wave's load instructions per tile: K then V
          constexpr int IPW = TileOffsets<HD>::IPW;
          const bf16* src = (kk / IPW ? vbase : kbase) + (int64_t)(j + 1) * BKV * ld;
          dma16((const char*)src, toff.off[kk % IPW], smem + ((j + 1) & 1) * STAGE + (kk / IPW) * KSTAGE + (wave_u * IPW + kk % IPW) * 1024);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // phase A
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        if (kk + KD < NKK) kf[(NKK + kk + KD) % (KD + 1)] = kread(NKK + kk + KD);
        __builtin_amdgcn_sched_barrier(0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(NKK + kk) % (KD + 1)], qf[kk], s[1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = kk * NPV / NKK; u < (kk + 1) * NPV / NKK; ++u) vf[0][u] = vread(u / NDB, u % NDB);
        soft_slice(0, kk, NKK);
        __builtin_amdgcn_sched_barrier(0);
      }
      soft_end();
      // phase B
#pragma unroll
      for (int u = 0; u < NPV; ++u) {
        oacc[u % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[0][u], pf[u / NDB], oacc[u % NDB], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        vf[1][u] = vread(2 + u / NDB, u % NDB);
        soft_slice(1, u, NPV);
        __builtin_amdgcn_sched_barrier(0);
      }
      soft_end();
      // phase 3
#pragma unroll
      for (int u = 0; u < NPV; ++u)
        oacc[u % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[1][u], pf[2 + u / NDB], oacc[u % NDB], 0, 0, 0);
    };
    if (wave_active) {
      if (spread) tile_body(std::true_type{}); else tile_body(std::false_type{});
    }
    dma_wait_all();
    __syncthreads();                                  // fence + barrier: the next tile has landed for everybody
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  {
    // O leaves through LDS.  In the accumulators a lane holds scattered groups of 4 features of ONE query, so a store from
    // there touches 32 rows with 16 bytes each (512 requests per wave and tile of queries: ~5 k cycles per pass).  The
    // wave's 32 x HD block goes, normalised and in bf16, into its own patch of the second stage (free after the loop's last
    // barrier; the next pass loads its first tile into the first stage), 16-byte chunks XOR-swizzled by the row, and comes
    // back so that HD / 8 consecutive lanes hold one whole row.
    constexpr int NCH = HD / 8, RPO = 64 / NCH;       // chunks per row; rows per store instruction
    LDS char* const patch = lds0 + STAGE + wave_u * (32 * KROW);
    const float inv = 1.0f / l_tot;
    // the lane numbers are made opaque here: the patch addresses are the same in every pass, and computed ahead of the
    // tile loop they would live (or spill) across it
    int e31 = l31, ehalf = half, elane = lane;
    asm volatile("" : "+v"(e31), "+v"(ehalf), "+v"(elane));
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = (bf16)(oacc[db][g4 * 4 + i] * inv);
        *reinterpret_cast<LDS bf16x4*>(patch + e31 * KROW + (((db * 4 + g4) ^ (e31 & (NCH - 1))) << 4) + ehalf * 8) = pk;
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);               // lgkmcnt(0): the patch is complete before it is read back
    __builtin_amdgcn_wave_barrier();
    const int orow = elane / NCH, ochunk = elane % NCH;
#pragma unroll
    for (int it = 0; it < 32 / RPO; ++it) {
      const int row = it * RPO + orow, q = wq0 + row;
      const bf16x8 v = *reinterpret_cast<const LDS bf16x8*>(patch + row * KROW + ((ochunk ^ (row & (NCH - 1))) << 4));
      if (q < S) *reinterpret_cast<bf16x8*>(o + ((int64_t)b * S + q) * Dq + (int64_t)h * HD + ochunk * 8) = v;
    }
    if (myq < S && half == 0) lse[((int64_t)b * H + h) * S + myq] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994531f;
  }
  }  // pass
}


// ------------------------------------------------------------------------------------------
// Backward.  With P = softmax(S), dP = dO V^T, dS = P o (dP - delta), delta_i = sum_d dO_id O_id:
//   dQ = dS K / sqrt(hd),  dK = dS^T Q / sqrt(hd),  dV = P^T dO.
// Two kernels, no atomics (results are run-to-run identical):
//   dq kernel : one workgroup per 128 queries, walks the key tiles like the forward.  S^T and
//               dP^T = V dO^T are formed with keys in the MFMA row dimension so that lse and
//               delta are per-lane scalars; dS^T feeds dQ^T += K^T dS^T from registers (K is
//               also kept transposed in LDS, same key order trick as V in the forward).
//   dkv kernel: one workgroup per 64 keys of a kv head (16 per wave, v_mfma_f32_16x16x32_bf16), walks
//               the query tiles of every query head of the group.  Here S = Q K^T and dP = dO V^T
//               are formed with QUERIES in the row dimension, so each lane owns a key column and
//               P, dS feed dV^T += dO^T P and dK^T += Q^T dS from registers.
// Both stream their tiles (K and V; Q and dO) global -> LDS row-major with direct-to-LDS loads and take
// the transposed operands out of the same tiles with transposing LDS reads.

// byte offset of 16-byte chunk `chunk` of row `row` in a row-major tile
template <int HD, int SW = 0>
__device__ __forceinline__ int rm_off(int row, int chunk) { return row * (HD * 2) + (rm_pos<HD, SW>(chunk, row) << 4); }

// Inverse RoPE of 4 consecutive features d..d+3 (two pairs) of the token at in-sequence position p:
// (a, b) -> (a cos + b sin, -a sin + b cos), the transpose of the forward rotation.
template <int HD>
__device__ __forceinline__ void unrope4(float (&v)[4], const float* __restrict__ cs, int p, int d) {
  const f32x4 t = *reinterpret_cast<const f32x4*>(cs + ((int64_t)p * (HD / 2) + (d >> 1)) * 2);
  const float a0 = v[0], b0 = v[1], a1 = v[2], b1 = v[3];
  v[0] = a0 * t[0] + b0 * t[1];
  v[1] = b0 * t[0] - a0 * t[1];
  v[2] = a1 * t[2] + b1 * t[3];
  v[3] = b1 * t[2] - a1 * t[3];
}

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_mfma_kernel(const bf16* __restrict__ qkv, int64_t ld, const bf16* __restrict__ o,
                                                               const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                               float* __restrict__ delta, bf16* __restrict__ dqkv, int B, int S, int H, int Hkv,
                                                               float scale, const float* __restrict__ rope_cs, int pair) {
  constexpr int KCH = HD / 8, NKK = HD / 16, NDB = HD / 32;
  constexpr int TILE = BKV * HD * 2;                 // bytes of one 64-row tile (row-major or transposed)
  constexpr int STAGE = 2 * TILE;                    // K and V, both row-major (K is read along its rows and transposed)
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nqt = (S + BQ - 1) / BQ;
  int rank, h, b;
  if (!xcd_map((int)blockIdx.x, paired_tiles(pair, nqt), H / Hkv, Hkv, B, rank, h, b)) return;
  const int kvh = h / (H / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, half = lane >> 5;
  const int Dq = H * HD, Dkv = Hkv * HD;
  const float c2 = scale * 1.4426950408889634f;
  const bf16* kbase = qkv + (int64_t)b * S * ld + Dq + (int64_t)kvh * HD;
  const bf16* vbase = kbase + Dkv;
  TileOffsets<HD> toff;
  toff.init(ld, wave, lane);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  for (int pass = 0; pass < n_passes(pair, nqt, rank); ++pass) {
  const int qt = pass == 0 ? nqt - 1 - rank : rank;
  const int q0 = qt * BQ, wq0 = q0 + wave * 32, myq = wq0 + l31;
  const int qrow = min(myq, S - 1);

  bf16x8 qf[NKK], dof[NKK];
  float dl = 0.0f;
  {
    const bf16* qp = qkv + ((int64_t)b * S + qrow) * ld + (int64_t)h * HD;
    const bf16* op = o + ((int64_t)b * S + qrow) * Dq + (int64_t)h * HD;
    const bf16* dp = dout + ((int64_t)b * S + qrow) * Dq + (int64_t)h * HD;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + half * 8);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dp + kk * 16 + half * 8);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(op + kk * 16 + half * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) dl = fmaf((float)dof[kk][e], (float)of[e], dl);
    }
  }
  dl += __shfl_xor(dl, 32, 64);
  const int64_t li = ((int64_t)b * H + h) * S + qrow;
  const float lse2 = lse[li] * 1.4426950408889634f;
  if (myq < S && half == 0) delta[li] = dl;

  const int nkv = (S + BKV - 1) / BKV;
  const int ntiles = CAUSAL ? min((q0 + BQ + BKV - 1) / BKV, nkv) : nkv;
  auto stage_tile = [&](int j, int stage) {
    char* base = smem + stage * STAGE;
    if ((j + 1) * BKV <= S) {                        // whole tile inside the sequence (uniform)
      stage_tile_fast<HD>(kbase + (int64_t)j * BKV * ld, toff, base, wave_u);
      stage_tile_fast<HD>(vbase + (int64_t)j * BKV * ld, toff, base + TILE, wave_u);
    } else {
      stage_two_tiles<HD>(kbase, ld, vbase, ld, j * BKV, S - 1, base, base + TILE, wave, lane);
    }
  };

  f32x16 dq[NDB];
#pragma unroll
  for (int i = 0; i < NDB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.0f;

  stage_tile(0, 0);
  dma_wait_all();
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const bool more = j + 1 < ntiles;
    if (more) stage_tile(j + 1, (j + 1) & 1);
    const int k0 = j * BKV;
    if (!CAUSAL || k0 <= wq0 + 31) {
      const char* ks = smem + (j & 1) * STAGE;
      const char* vs = ks + TILE;
      const bool need_mask = (CAUSAL && k0 + BKV - 1 > wq0) || (k0 + BKV > S);
      // one 32-key block at a time, to keep only 32 score registers live
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.0f; dp[r] = 0.0f; }
        const int krow = t * 32 + l31;
        // fragments one k step ahead of the MFMAs that use them: a read issued right before its MFMA exposes the LDS latency
        bf16x8 kf[2], vf[2];
        kf[0] = *reinterpret_cast<const bf16x8*>(ks + rm_off<HD>(krow, half));
        vf[0] = *reinterpret_cast<const bf16x8*>(vs + rm_off<HD>(krow, half));
  #pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          if (kk + 1 < NKK) {
            kf[(kk + 1) & 1] = *reinterpret_cast<const bf16x8*>(ks + rm_off<HD>(krow, (kk + 1) * 2 + half));
            vf[(kk + 1) & 1] = *reinterpret_cast<const bf16x8*>(vs + rm_off<HD>(krow, (kk + 1) * 2 + half));
          }
          __builtin_amdgcn_sched_barrier(0);           // the scheduler would otherwise sink the reads back to their uses
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk & 1], qf[kk], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk & 1], dof[kk], dp, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
          bf16x8 dsf[2];
        if (need_mask) {                             // one uniform branch; a masked score of -inf gives p = 0 below
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + t * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if ((CAUSAL && key > myq) || key >= S) s[r] = -INFINITY;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lse2));
          dsf[r >> 3][r & 7] = (bf16)(p * (dp[r] - dl));
        }
  #pragma unroll
        for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
          for (int db = 0; db < NDB; ++db) {
            const bf16x8 ktf = tr_fragment<HD>(ks, t * 2 + g2, db, lane);
            dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf[g2], dq[db], 0, 0, 0);
          }
        }
    }
    dma_wait_all();
    __syncthreads();                                  // fence + barrier: the next tile has landed for everybody
  }
  {
    // dq leaves through LDS as whole rows, like the forward kernel's output: the wave's 32 x HD block, scaled, rotated back
    // and in bf16, goes into its patch of the second stage (free after the loop's last barrier) and comes back so that
    // HD / 8 consecutive lanes hold one row.
    constexpr int RPO = 64 / KCH;                     // rows per store instruction
    LDS char* const patch = (LDS char*)smem + STAGE + wave_u * (32 * HD * 2);
    int e31 = l31, ehalf = half, elane = lane;        // opaque: the patch addresses are not to live across the tile loop
    asm volatile("" : "+v"(e31), "+v"(ehalf), "+v"(elane));
    const int pq = min(myq, S - 1);                   // rows past the end are made and never stored
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = dq[db][g4 * 4 + i] * scale;
        if (rope_cs) unrope4<HD>(v, rope_cs, pq, db * 32 + g4 * 8 + half * 4);
        bf16x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = (bf16)v[i];
        *reinterpret_cast<LDS bf16x4*>(patch + e31 * (HD * 2) + (((db * 4 + g4) ^ (e31 & (KCH - 1))) << 4) + ehalf * 8) = pk;
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);               // lgkmcnt(0): the patch is complete before it is read back
    __builtin_amdgcn_wave_barrier();
    const int orow = elane / KCH, ochunk = elane % KCH;
#pragma unroll
    for (int it = 0; it < 32 / RPO; ++it) {
      const int row = it * RPO + orow, q = wq0 + row;
      const bf16x8 v = *reinterpret_cast<const LDS bf16x8*>(patch + row * (HD * 2) + ((ochunk ^ (row & (KCH - 1))) << 4));
      if (q < S) *reinterpret_cast<bf16x8*>(dqkv + ((int64_t)b * S + q) * ld + (int64_t)h * HD + ochunk * 8) = v;
    }
  }
  }  // pass
}

// A-operand fragment of v_mfma_f32_16x16x32_bf16 for the TRANSPOSE of a row-major 64-row tile: 16 features
// (16 fb .. 16 fb + 15) in the row dimension, the 32 rows 32 jj .. 32 jj + 31 in the contraction.  Lane (feature lane & 15,
// group g = lane >> 4) gets the feature's values in rows 4 g .. 4 g + 3 of the first and then of the second 16-row block
// -- the order in which a lane of the score blocks holds its 8 probabilities (two blocks of 16 rows x 16 keys, rows
// 4 g + r).  Two transposing reads: each group of 16 lanes takes a block of 4 rows x 16 features.
template <int HD>
__device__ __forceinline__ bf16x8 tr16_fragment(const char* tile, int jj, int fb, int lane) {
  const int tr_e = (lane & 15) >> 2, tr_q = lane & 3, g = lane >> 4;
  bf16x8 f;
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2) {
    const int row = 32 * jj + 16 * h2 + 4 * g + tr_e;
    const int chunk = 2 * fb + (tr_q >> 1);
    const bf16x4 t4 = __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(tile + row * (HD * 2) + (rm_pos<HD, 1>(chunk, row) << 4) + (tr_q & 1) * 8)));
#pragma unroll
    for (int i = 0; i < 4; ++i) f[h2 * 4 + i] = t4[i];
  }
  return f;
}

// dk / dv kernel.  One workgroup = 64 keys of one (sequence, kv head), 16 per wave, on v_mfma_f32_16x16x32_bf16: the
// accumulators dK^T, dV^T of 16 keys x head_dim are 2 x head_dim / 4 registers (64 at head_dim 128), so two workgroups
// share a CU and one wave's exponentials and LDS waits run under the other's MFMAs (with 32 keys per wave on the
// 32x32x16 shape the kernel needed 128 accumulator registers, ran one wave per SIMD and executed its phases --
// score products, exponentials, accumulating products, each waiting for its own LDS reads -- strictly one after the
// other: matrix pipe busy 14 % of the cycles).  Per query tile of 64 (four blocks of 16 queries) a wave forms
// S = Q K^T and dP = dO V^T with the QUERIES in the row dimension, so each lane owns one key column and four queries
// per block; P and dS of two blocks are, as they sit in the lane, one B operand (32 queries deep) for
// dV^T += dO^T P and dK^T += Q^T dS, whose A operands come out of the same row-major LDS tiles by transposing reads.
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_mfma_kernel(
    const bf16* __restrict__ qkv, int64_t ld, const bf16* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ dqkv, int B, int S, int H, int Hkv, float scale, const float* __restrict__ rope_cs, float* __restrict__ part, int pair) {
  constexpr int NK = HD / 32;                        // 32-deep contraction steps over the head dimension
  constexpr int NFB = HD / 16;                       // 16-feature blocks of dK^T / dV^T
  constexpr int TILE = 64 * HD * 2;
  constexpr int STAGE = 2 * TILE + 512;              // Q and dO row-major (read along the rows and transposed), lse2[64], delta[64]
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int G = H / Hkv;
  const int nkt = (S + 63) / 64;
  int rank, kvh, b;
  // part != nullptr: one workgroup per (key tile, QUERY head); its dk / dv contribution goes to
  // part[head within the group][token][dk | dv columns of all kv heads] in fp32 and attn_dkv_sum_kernel adds the group.
  int hsel = 0;
  if (part) {
    if (!xcd_map((int)blockIdx.x, paired_tiles(pair, nkt), G, Hkv, B, rank, hsel, b)) return;
    kvh = hsel / G;
  } else if (!xcd_map((int)blockIdx.x, paired_tiles(pair, nkt), 1, Hkv, B, rank, kvh, b)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l15 = lane & 15, lg = lane >> 4;
  const int Dq = H * HD, Dkv = Hkv * HD;
  const float c2 = scale * 1.4426950408889634f;
  TileOffsets<HD, 4, 1> toff_q, toff_d;
  toff_q.init(ld, wave, lane);
  toff_d.init(Dq, wave, lane);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  for (int pass = 0; pass < n_passes(pair, nkt, rank); ++pass) {
  const int kt = pass == 0 ? rank : nkt - 1 - rank;  // under the causal mask the first key tiles have the longest columns
  const int k0 = kt * 64, wk0 = k0 + wave * 16, mykey = wk0 + l15;
  const int krow = min(mykey, S - 1);

  bf16x8 kf[NK], vf[NK];                              // this lane's key / value row, 8 features of every 32
  {
    const bf16* kp = qkv + ((int64_t)b * S + krow) * ld + Dq + (int64_t)kvh * HD;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(kp + kk * 32 + lg * 8);
      vf[kk] = *reinterpret_cast<const bf16x8*>(kp + Dkv + kk * 32 + lg * 8);
    }
  }
  const int qstart = CAUSAL ? k0 : 0;                // a multiple of 64
  const int nq = (S - qstart + 63) / 64;             // query tiles per head
  const int ntiles = part ? nq : nq * G;
  float lreg = 0.0f, dlreg = 0.0f;
  auto stage_tile = [&](int j, int stage) {            // Q and dO tiles straight to LDS; the two per-query scalars via registers
    const int h = part ? hsel : kvh * G + j / nq, q0 = qstart + (j % nq) * 64;
    char* base = smem + stage * STAGE;
    const bf16* qrows = qkv + (int64_t)b * S * ld + (int64_t)h * HD;
    const bf16* drows = dout + (int64_t)b * S * Dq + (int64_t)h * HD;
    // the two scalar loads go first: they are waited for when the tile is nearly done, and a wait for a load also
    // waits for every older one -- behind the tile loads they would drag those along
    if (tid < 64) {
      const int64_t li = ((int64_t)b * H + h) * S + min(q0 + tid, S - 1);
      lreg = lse[li];
      dlreg = delta[li];
    }
    if (q0 + 64 <= S) {                              // whole tile inside the sequence (uniform)
      stage_tile_fast<HD, 4, 1>(qrows + (int64_t)q0 * ld, toff_q, base, wave_u);
      stage_tile_fast<HD, 4, 1>(drows + (int64_t)q0 * Dq, toff_d, base + TILE, wave_u);
    } else {
      stage_two_tiles<HD, 1>(qrows, ld, drows, Dq, q0, S - 1, base, base + TILE, wave, lane);
    }
  };
  auto store_scalars = [&](int stage) {
    if (tid < 64) {
      char* base = smem + stage * STAGE;
      reinterpret_cast<float*>(base + 2 * TILE)[tid] = lreg * 1.4426950408889634f;
      reinterpret_cast<float*>(base + 2 * TILE + 256)[tid] = dlreg;
    }
  };

  f32x4 dk[NFB], dv[NFB];
#pragma unroll
  for (int i = 0; i < NFB; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) { dk[i][r] = 0.0f; dv[i][r] = 0.0f; }

  if (ntiles > 0) {
    stage_tile(0, 0);
    store_scalars(0);
  }
  dma_wait_all();
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const bool more = j + 1 < ntiles;
    if (more) stage_tile(j + 1, (j + 1) & 1);
    const int q0 = qstart + (j % nq) * 64;
    const char* qs = smem + (j & 1) * STAGE;
    const char* ds_ = qs + TILE;
    const float* ls = reinterpret_cast<const float*>(qs + 2 * TILE);
    const float* dls = ls + 64;
    const bool need_mask = (CAUSAL && q0 < wk0 + 15) || (q0 + 64 > S);
    bf16x8 pf[2], dsf[2];                            // P and dS of the tile: [32-query half], as the B operands below
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const int qb = 2 * jj + h2, row = qb * 16 + l15;
        f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f}, dp = {0.0f, 0.0f, 0.0f, 0.0f};
  #pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
          const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qs + rm_off<HD, 1>(row, kk * 4 + lg));
          const bf16x8 df = *reinterpret_cast<const bf16x8*>(ds_ + rm_off<HD, 1>(row, kk * 4 + lg));
          s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf, kf[kk], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_16x16x32_bf16(df, vf[kk], dp, 0, 0, 0);
        }
          // this lane: key mykey, queries q0 + 16 qb + 4 lg + r
        if (need_mask) {                             // one uniform branch; a masked score of -inf gives p = 0 below
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int q = q0 + qb * 16 + 4 * lg + r;
            if ((CAUSAL && q < mykey) || q >= S) s[r] = -INFINITY;
          }
        }
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(ls + qb * 16 + 4 * lg);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dls + qb * 16 + 4 * lg);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -l4[r]));
          pf[jj][h2 * 4 + r] = (bf16)p;
          dsf[jj][h2 * 4 + r] = (bf16)(p * (dp[r] - d4[r]));
        }
      }
    }
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const bf16x8 dtf = tr16_fragment<HD>(ds_, jj, fb, lane);
        const bf16x8 qtf = tr16_fragment<HD>(qs, jj, fb, lane);
        dv[fb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dtf, pf[jj], dv[fb], 0, 0, 0);
        dk[fb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qtf, dsf[jj], dk[fb], 0, 0, 0);
      }
    if (more) store_scalars((j + 1) & 1);
    dma_wait_all();
    __syncthreads();                                  // fence + barrier: the next tiles have landed for everybody
  }
  // this lane: key mykey, features 16 fb + 4 lg .. + 3 of dK and dV
  if (mykey < S && part) {                           // the rotation is linear: undone per contribution
    float* out = part + (((int64_t)(hsel - kvh * G) * B + b) * S + mykey) * (2 * Dkv) + (int64_t)kvh * HD;
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb) {
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = dk[fb][i] * scale;
      if (rope_cs) unrope4<HD>(v, rope_cs, mykey, fb * 16 + lg * 4);
      f32x4 ok;
#pragma unroll
      for (int i = 0; i < 4; ++i) ok[i] = v[i];
      *reinterpret_cast<f32x4*>(out + fb * 16 + lg * 4) = ok;
      *reinterpret_cast<f32x4*>(out + Dkv + fb * 16 + lg * 4) = dv[fb];
    }
  } else if (!part) {
    // dk and dv leave through LDS as whole rows: the wave's two 16 x HD blocks (dk scaled and rotated back), in bf16, go
    // into its patch of the second stage's tiles (free after the loop's last barrier; the next pass loads into the first
    // stage) with the 16-byte chunks XOR-swizzled by the key, and come back so that HD / 8 consecutive lanes hold one row.
    constexpr int KCH = HD / 8, RPO = 64 / KCH, ROWB = HD * 2;
    LDS char* const patch = (LDS char*)smem + STAGE + wave_u * (2 * 16 * ROWB);
    int e15 = l15, elg = lg, elane = lane;            // opaque: the patch addresses are not to live across the tile loop
    asm volatile("" : "+v"(e15), "+v"(elg), "+v"(elane));
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb) {
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = dk[fb][i] * scale;
      if (rope_cs) unrope4<HD>(v, rope_cs, krow, fb * 16 + lg * 4);
      bf16x4 pk, pv;
#pragma unroll
      for (int i = 0; i < 4; ++i) { pk[i] = (bf16)v[i]; pv[i] = (bf16)dv[fb][i]; }
      LDS char* const at = patch + e15 * ROWB + (((fb * 2 + (elg >> 1)) ^ (e15 & (KCH - 1))) << 4) + (elg & 1) * 8;
      *reinterpret_cast<LDS bf16x4*>(at) = pk;
      *reinterpret_cast<LDS bf16x4*>(at + 16 * ROWB) = pv;
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);               // lgkmcnt(0): the patch is complete before it is read back
    __builtin_amdgcn_wave_barrier();
    const int orow = elane / KCH, ochunk = elane % KCH;
#pragma unroll
    for (int it = 0; it < 16 / RPO; ++it) {
      const int row = it * RPO + orow, key = wk0 + row;
      LDS const char* const at = patch + row * ROWB + ((ochunk ^ (row & (KCH - 1))) << 4);
      const bf16x8 vk = *reinterpret_cast<const LDS bf16x8*>(at);
      const bf16x8 vv = *reinterpret_cast<const LDS bf16x8*>(at + 16 * ROWB);
      if (key < S) {
        bf16* out = dqkv + ((int64_t)b * S + key) * ld + Dq + (int64_t)kvh * HD + ochunk * 8;
        *reinterpret_cast<bf16x8*>(out) = vk;
        *reinterpret_cast<bf16x8*>(out + Dkv) = vv;
      }
    }
  }
  }  // pass
}

// dk | dv of the G query heads of every group, added in the order of the heads: one thread per 4 columns of a token
__global__ __launch_bounds__(256) void attn_dkv_sum_kernel(const float* __restrict__ part, bf16* __restrict__ dqkv, int64_t ld, int Dq,
                                                           int Dkv, int G, int64_t T) {
  const int c4 = (2 * Dkv) >> 2;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * c4) return;
  const int64_t t = idx / c4;
  const int col = (int)(idx % c4) * 4;
  const float* p = part + t * (2 * Dkv) + col;
  f32x4 sum = *reinterpret_cast<const f32x4*>(p);
  for (int g = 1; g < G; ++g) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(p + (int64_t)g * T * (2 * Dkv));
#pragma unroll
    for (int i = 0; i < 4; ++i) sum[i] += v[i];
  }
  bf16x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (bf16)sum[i];
  *reinterpret_cast<bf16x4*>(dqkv + t * ld + Dq + col) = o;
}

}  // namespace

bool mfma_attn_supported(int S, int H, int Hkv, int hd, int64_t ld) {
  return (hd == 32 || hd == 64 || hd == 128) && S >= 1 && H % Hkv == 0 && ld % 8 == 0;
}

hipError_t mfma_attn_fwd(const void* qkv, int64_t ld, void* o, float* lse, int B, int S, int H, int Hkv, int hd, int causal, hipStream_t st,
                         int scale_hd) {
  if (!mfma_attn_supported(S, H, Hkv, hd, ld)) return hipErrorInvalidValue;
  if (B <= 0) return hipSuccess;
  const int nqt = (S + BQ - 1) / BQ;
  const int pair = pair_tiles(causal, nqt);
  const dim3 grid(xcd_grid(paired_tiles(pair, nqt), H / Hkv, Hkv, B)), block(256);
  const float c = 1.4426950408889634f / sqrtf((float)(scale_hd > 0 ? scale_hd : hd));
#define SV_ATTN_LAUNCH(HDV, CZ)                                                                                         \
  do {                                                                                                                  \
    auto kern = attn_fwd_mfma_kernel<HDV, CZ>;                                                                          \
    constexpr int lds = 2 * (BKV * HDV * 2 + HDV * 128);                                                                \
    static bool configured = false;                                                                                     \
    if (!configured) {                                                                                                  \
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);           \
      if (e != hipSuccess) return e;                                                                                    \
      configured = true;                                                                                                \
    }                                                                                                                   \
    hipLaunchKernelGGL(kern, grid, block, lds, st, (const bf16*)qkv, ld, (bf16*)o, lse, B, S, H, Hkv, c, pair);                  \
  } while (0)
  if (hd == 128) { if (causal) SV_ATTN_LAUNCH(128, true); else SV_ATTN_LAUNCH(128, false); }
  else if (hd == 64) { if (causal) SV_ATTN_LAUNCH(64, true); else SV_ATTN_LAUNCH(64, false); }
  else { if (causal) SV_ATTN_LAUNCH(32, true); else SV_ATTN_LAUNCH(32, false); }
#undef SV_ATTN_LAUNCH
  return hipGetLastError();
}


hipError_t mfma_attn_bwd(const void* qkv, int64_t ld, const void* o, const void* dout, const float* lse, float* delta, void* dqkv, int B,
                         int S, int H, int Hkv, int hd, int causal, const float* rope_cs, hipStream_t st, int scale_hd, float* part_ws,
                         int64_t part_floats) {
  if (!mfma_attn_supported(S, H, Hkv, hd, ld)) return hipErrorInvalidValue;
  if (B <= 0) return hipSuccess;
  // A launch that leaves workgroup slots empty (two per CU) -- one long sequence, few kv heads -- gives every query head
  // of a group its own workgroup, and the group is added afterwards; fuller launches keep the group in one workgroup
  // and save the fp32 partial results their round trip through memory.
  const int G = H / Hkv, nqt = (S + BQ - 1) / BQ, nkt = (S + 63) / 64;
  const int pair_q = pair_tiles(causal, nqt), pair_k = pair_tiles(causal, nkt);
  const bool split = G > 1 && part_ws && (int64_t)paired_tiles(pair_k, nkt) * Hkv * B < kDkvSplitWorkgroups &&
                     (int64_t)G * B * S * 2 * Hkv * hd <= part_floats;
  float* part = split ? part_ws : nullptr;
  const dim3 gq(xcd_grid(paired_tiles(pair_q, nqt), G, Hkv, B)), gk(xcd_grid(paired_tiles(pair_k, nkt), split ? G : 1, Hkv, B)), block(256);
  const float scale = 1.0f / sqrtf((float)(scale_hd > 0 ? scale_hd : hd));
#define SV_ATTN_BWD_LAUNCH(HDV, CZ)                                                                                     \
  do {                                                                                                                  \
    auto kq = attn_bwd_dq_mfma_kernel<HDV, CZ>;                                                                         \
    auto kk = attn_bwd_dkv_mfma_kernel<HDV, CZ>;                                                                        \
    constexpr int lq = 2 * 2 * (64 * HDV * 2), lk = 2 * (2 * 64 * HDV * 2 + 512);                                       \
    static bool configured = false;                                                                                     \
    if (!configured) {                                                                                                  \
      hipError_t e = hipFuncSetAttribute((const void*)kq, hipFuncAttributeMaxDynamicSharedMemorySize, lq);              \
      if (e == hipSuccess) e = hipFuncSetAttribute((const void*)kk, hipFuncAttributeMaxDynamicSharedMemorySize, lk);    \
      if (e != hipSuccess) return e;                                                                                    \
      configured = true;                                                                                                \
    }                                                                                                                   \
    hipLaunchKernelGGL(kq, gq, block, lq, st, (const bf16*)qkv, ld, (const bf16*)o, (const bf16*)dout, lse, delta,      \
                       (bf16*)dqkv, B, S, H, Hkv, scale, rope_cs, pair_q);                                              \
    hipLaunchKernelGGL(kk, gk, block, lk, st, (const bf16*)qkv, ld, (const bf16*)dout, lse, delta, (bf16*)dqkv, B, S,   \
                       H, Hkv, scale, rope_cs, part, pair_k);                                                           \
  } while (0)
  if (hd == 128) { if (causal) SV_ATTN_BWD_LAUNCH(128, true); else SV_ATTN_BWD_LAUNCH(128, false); }
  else if (hd == 64) { if (causal) SV_ATTN_BWD_LAUNCH(64, true); else SV_ATTN_BWD_LAUNCH(64, false); }
  else { if (causal) SV_ATTN_BWD_LAUNCH(32, true); else SV_ATTN_BWD_LAUNCH(32, false); }
#undef SV_ATTN_BWD_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !split) return e;
  const int64_t T = (int64_t)B * S, threads = T * (2 * Hkv * hd / 4);
  hipLaunchKernelGGL(attn_dkv_sum_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, part, (bf16*)dqkv, ld, H * hd, Hkv * hd,
                     G, T);
  return hipGetLastError();
}

}  // namespace sv
