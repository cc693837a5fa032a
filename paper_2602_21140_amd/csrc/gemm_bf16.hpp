// Grouped bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
//   C[rows of tile, n] = sum_k A[row, k] * B_group[n, k]        ("NT": both operands K-contiguous)
//
// A is one tall activation matrix whose rows are split into row-tiles that each belong to one
// group (physical expert slot); B is that group's output-major weight matrix.  Three epilogues:
//   EPI_F32     store fp32                         (router logits)
//   EPI_BF16    round to bf16 and store            (down projection)
//   EPI_SWIGLU  B holds gate rows [0, n_out) and up rows [n_out, 2 n_out); store
//               bf16(silu(gate) * up)              (gate/up projection of a SwiGLU expert)
//
// Work decomposition: one workgroup computes a BM x BN tile with WAVES_M x WAVES_N wavefronts of
// 64 lanes; each wavefront owns (BM/WAVES_M) x (BN/WAVES_N) outputs as 32x32 MFMA tiles.  K is
// walked in steps of 64: the next step's global loads are issued into registers before the MFMAs
// of the current step and written to the other half of a double-buffered LDS tile afterwards, one
// barrier per step.  LDS rows are 128 bytes (64 bf16); the 16-byte chunk index is XOR-ed with
// ((row >> 1) & 7) so that both the 16-byte writes and the per-lane 16-byte fragment reads are
// conflict-free on the 64-bank LDS.  The weights go in as the MFMA's first operand so that each lane ends up with
// four consecutive output columns of one activation row, which it stores as one 8/16-byte word.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "ctx.hpp"

namespace revive {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
// Pointers that are known to address HBM: lets the compiler emit global_load/global_store
// instead of flat accesses (which also tick the LDS counter and so serialise with LDS waits).
typedef const __attribute__((address_space(1))) u32x4* gptr_u32x4;

__device__ __forceinline__ u32x4 load_global_16B(const unsigned char* p) {
  return *reinterpret_cast<gptr_u32x4>(reinterpret_cast<uintptr_t>(p));
}

enum { EPI_F32 = 0, EPI_BF16 = 1, EPI_SWIGLU = 2 };

// Tiled weight layout: a [rows, K] output-major matrix is stored as [rows/128][K/32][128][32]
// (rows zero-padded to a multiple of 128), so the 128 x 32 block a workgroup fetches per K-step is
// 8 KiB contiguous and a whole 128-row panel is one contiguous stream over K.
constexpr int kWeightTileRows = 128;
constexpr int kWeightTileK = 32;

struct GemmArgs {
  const void* A;             // [rows, K] bf16
  int64_t lda;               // elements between rows of A
  const void* const* B_tab;  // device table: group -> [n_rows_B, K] bf16, or null
  const void* B_one;         // used for every group when B_tab is null
  int64_t ldb;               // elements between rows of B
  void* C;                   // [rows, n_out] fp32 or bf16
  int64_t ldc;
  int n_out;                 // output columns (SwiGLU: I, with B holding 2*I rows)
  int K;                     // multiple of 64
  const MTile* tiles;        // device row-tile list, or null for a dense [0, M) matrix
  const int32_t* tile_count; // device count of valid entries in `tiles`
  int M;                     // dense case: number of rows
  int n_col_tiles;
  int b_sel;                 // -1: weights from B_tab / B_one; 0 or 1: from the tile record's w[b_sel]
  int b_tiled;               // B is stored in the tiled weight layout (see kWeightTileRows)
  int b_rows_pad;            // tiled: rows of B (of each half for SwiGLU) padded to whole tiles
  int a_rows;                // > 0: A is stored K-panel-major, [K/32][a_rows][32]: the 32 K-elements of a row that one
                             // K-step needs are 64 contiguous bytes and consecutive rows follow each other, so the
                             // copies of a row-tile read one contiguous run per K-step (used for the intermediate h)
  int c_rows;                // > 0 (bf16 epilogues): C is written in the same layout, [n_out/32][c_rows][32]
};

// Up to two independent problems served by one launch (e.g. the routed experts' grouped GEMM and
// the shared expert's dense GEMM): their tiles are numbered one after the other.
struct GemmArgs2 {
  GemmArgs p0, p1;
  int two;  // 0: only p0 is valid
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Round-to-nearest-even fp32 -> bf16 bits (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Two fp32 -> one word of two bf16 (round-to-nearest-even), one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// LDS swizzle.  The gfx950 LDS has 64 four-byte banks (256 B per clock) and serves a 16-byte
// per-lane access in groups of 16 lanes.  Tile rows are 128 bytes, so rows r and r+2 start on the
// same bank; XOR-ing the 16-byte chunk index with (row >> 1) & 7 makes the 16 rows a lane group
// touches (same logical chunk) fall on 16 distinct 16-byte bank groups.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// silu(z) = z / (1 + exp(-z)) with the hardware reciprocal (1 ulp) instead of an IEEE division: the
// result is rounded to bf16 right after, and the division sequence is ten instructions per output.
// exp overflows to +inf for z < -88, where the product is the correct -0.
__device__ __forceinline__ float silu_f32(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// KID (the library's kernel id) only gives each use of the kernel its own symbol name in profiles.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int KID>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(GemmArgs g) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int ITER_A = BM * 8 / NT, ITER_B = BN * 8 / NT;
  constexpr int BN_OUT = EPI == EPI_SWIGLU ? BN / 2 : BN;  // output columns per workgroup
  constexpr int STAGE = (BM + BN) * 128;                   // bytes of one LDS stage
  static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "tile shape");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "load split");
  static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU needs gate and up tiles in one wave");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- which tile is mine: spread the valid tiles evenly over the 8 XCDs (workgroup i runs on
  // XCD i % 8) so that each XCD's L2 sees a contiguous run of tiles sharing activations/weights.
  const int n_m_tiles = g.tiles ? *g.tile_count : (g.M + BM - 1) / BM;
  const int total = n_m_tiles * g.n_col_tiles;
  const int per_xcd = (total + 7) >> 3;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int logical = xcd * per_xcd + local;
  if (local >= per_xcd || logical >= total) return;
  const int m_idx = logical / g.n_col_tiles;
  const int n_idx = logical - m_idx * g.n_col_tiles;

  int group = 0, row_begin, row_end;
  if (g.tiles) {
    const MTile t = g.tiles[m_idx];
    group = t.group;
    tile_span(t.group_begin, t.group_end, t.pad >> 16, t.pad & 0xFFFF, BM, row_begin, row_end);
  } else {
    row_begin = m_idx * BM;
    row_end = min(g.M, row_begin + BM);
  }
  const unsigned char* Bbase = static_cast<const unsigned char*>(g.B_tab ? g.B_tab[group] : g.B_one);
  const unsigned char* Abase = static_cast<const unsigned char*>(g.A);
  const int n0 = n_idx * BN_OUT;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- per-thread global sources and LDS destinations of the cooperative tile loads
  const unsigned char* a_src[ITER_A];
  const unsigned char* b_src[ITER_B];
  int a_dst[ITER_A], b_dst[ITER_B];
#pragma unroll
  for (int it = 0; it < ITER_A; ++it) {
    const int idx = it * NT + tid, row = idx >> 3, chunk = idx & 7;
    const int grow = min(row_begin + row, row_end - 1);  // rows past the tile re-read its last row
    a_src[it] = Abase + (static_cast<int64_t>(grow) * g.lda + chunk * 8) * 2;
    a_dst[it] = row * 128 + ((chunk ^ swz(row)) << 4);
  }
#pragma unroll
  for (int it = 0; it < ITER_B; ++it) {
    const int idx = it * NT + tid, row = idx >> 3, chunk = idx & 7;
    int brow;
    if (EPI == EPI_SWIGLU) {
      const int half = row >= BN / 2;
      const int col = min(n0 + row - half * (BN / 2), g.n_out - 1);
      brow = col + half * g.n_out;
    } else {
      brow = min(n0 + row, g.n_out - 1);
    }
    b_src[it] = Bbase + (static_cast<int64_t>(brow) * g.ldb + chunk * 8) * 2;
    b_dst[it] = BM * 128 + row * 128 + ((chunk ^ swz(row)) << 4);
  }

  // ---- per-lane LDS fragment addresses (without the k-step part)
  int a_frag[TM], b_frag[TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) a_frag[tm] = wm * WM + tm * 32 + (lane & 31);
#pragma unroll
  for (int tn = 0; tn < TN; ++tn) {
    int r;
    if (EPI == EPI_SWIGLU) {
      const int half = tn >= TN / 2;
      r = half * (BN / 2) + wn * (WN / 2) + (tn - half * (TN / 2)) * 32 + (lane & 31);
    } else {
      r = wn * WN + tn * 32 + (lane & 31);
    }
    b_frag[tn] = BM + r;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.f;

  u32x4 a_reg[ITER_A], b_reg[ITER_B];
  auto load_global = [&](int kt) {
    const int64_t koff = static_cast<int64_t>(kt) * 128;  // 64 bf16
#pragma unroll
    for (int it = 0; it < ITER_A; ++it) a_reg[it] = load_global_16B(a_src[it] + koff);
#pragma unroll
    for (int it = 0; it < ITER_B; ++it) b_reg[it] = load_global_16B(b_src[it] + koff);
  };
  auto store_lds = [&](int stage) {
    unsigned char* base = smem + stage * STAGE;
#pragma unroll
    for (int it = 0; it < ITER_A; ++it) *reinterpret_cast<u32x4*>(base + a_dst[it]) = a_reg[it];
#pragma unroll
    for (int it = 0; it < ITER_B; ++it) *reinterpret_cast<u32x4*>(base + b_dst[it]) = b_reg[it];
  };

  // Fragment loads of one 16-wide k-step from an LDS stage.
  auto load_frags = [&](const unsigned char* base, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      const int r = a_frag[tm];
      af[tm] = *reinterpret_cast<const bf16x8*>(base + r * 128 + ((chunk ^ swz(r)) << 4));
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const int r = b_frag[tn];
      bfr[tn] = *reinterpret_cast<const bf16x8*>(base + r * 128 + ((chunk ^ swz(r)) << 4));
    }
  };
  auto mfma_step = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tn], af[tm], acc[tm][tn], 0, 0, 0);
  };

  // Software pipeline: the fragments of k-step s+1 are read from LDS while the MFMAs of step s
  // run; the next K-tile (already in registers) is written to the other LDS stage and the
  // workgroup synchronised *before* the last k-step's MFMAs, so that the first fragments of the
  // next stage are in flight while those MFMAs execute.
  const int KT = g.K >> 6;
  bf16x8 af0[TM], bf0[TN], af1[TM], bf1[TN];
  load_global(0);
  store_lds(0);
  __syncthreads();
  if (KT > 1) load_global(1);
  load_frags(smem, 0, af0, bf0);

  for (int kt = 0; kt < KT; ++kt) {
    const unsigned char* cur = smem + (kt & 1) * STAGE;
    load_frags(cur, 1, af1, bf1);
    mfma_step(af0, bf0);
    load_frags(cur, 2, af0, bf0);
    mfma_step(af1, bf1);
    load_frags(cur, 3, af1, bf1);
    mfma_step(af0, bf0);
    if (kt + 1 < KT) {
      store_lds((kt + 1) & 1);
      if (kt + 2 < KT) load_global(kt + 2);
      __syncthreads();
      load_frags(smem + ((kt + 1) & 1) * STAGE, 0, af0, bf0);
    }
    mfma_step(af1, bf1);
  }

  // ---- epilogue.  Lane holds, per 32x32 tile, for q = 0..3 the four columns
  // q*8 + (lane/32)*4 + {0..3} of activation row lane % 32.
  constexpr int TN_OUT = EPI == EPI_SWIGLU ? TN / 2 : TN;
  constexpr int WN_OUT = EPI == EPI_SWIGLU ? WN / 2 : WN;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int row = row_begin + wm * WM + tm * 32 + (lane & 31);
    if (row >= row_end) continue;
#pragma unroll
    for (int tn = 0; tn < TN_OUT; ++tn) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = n0 + wn * WN_OUT + tn * 32 + q * 8 + (lane >> 5) * 4;
        if (col >= g.n_out) continue;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (EPI == EPI_SWIGLU) v[r] = silu_f32(acc[tm][tn][q * 4 + r]) * acc[tm][tn + TN / 2][q * 4 + r];
          else v[r] = acc[tm][tn][q * 4 + r];
        }
        const int64_t off = static_cast<int64_t>(row) * g.ldc + col;
        if (col + 3 < g.n_out && (g.ldc & 3) == 0) {
          if (EPI == EPI_F32) {
            f32x4 o = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + off) = o;
          } else {
            u32x2 o = {f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16),
                       f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16)};
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(g.C) + off) = o;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (col + r >= g.n_out) break;
            if (EPI == EPI_F32) static_cast<float*>(g.C)[off + r] = v[r];
            else static_cast<uint16_t*>(g.C)[off + r] = static_cast<uint16_t>(f32_to_bf16_bits(v[r]));
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Variant with asynchronous global->LDS copies (global_load_lds_dwordx4) and a four-stage ring.
//
// Same contract and output layout as gemm_bf16_kernel.  K is walked in steps of 32; a stage holds
// a BM x 32 tile of A and a BN x 32 tile of B (64-byte rows).  The copy of K-step t+3 is issued
// while step t is being multiplied, so three steps (about 1.3 us of MFMA work at full rate) are
// in flight to cover HBM latency, and no register is spent on staging.  Per K-step there is one
// workgroup barrier, placed before the last 16-wide half-step's MFMAs so that the first fragment
// reads of the next stage overlap them.
//
// LDS layout of a stage: row r at r*64 bytes, its four 16-byte chunks stored at chunk ^ ((r>>2)&3):
// a copy instruction writes lane l's 16 bytes to (its 1 KiB window) + 16*l, i.e. 16 rows per
// wavefront instruction, and each lane fetches the chunk that belongs in its slot; the fragment
// reads (16 lanes = 16 consecutive rows, same logical chunk) then cover all 64 banks once.
// s_waitcnt immediate (gfx9 encoding) for "vmcnt(vm) lgkmcnt(0)", export counter ignored.
__host__ __device__ constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 0xF) | ((vm >> 4) << 14) | (0x7 << 4) | (0 << 8); }

__device__ __forceinline__ int swz32(int row) { return (row >> 2) & 3; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int KID, int STAGES = 4>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_dma_kernel(GemmArgs2 a2) {
  constexpr int NT = 64 * WAVES_M * WAVES_N, NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int BN_OUT = EPI == EPI_SWIGLU ? BN / 2 : BN;
  constexpr int D = STAGES - 1;  // copies run D K-steps ahead of the MFMAs
  constexpr int STAGE = (BM + BN) * 64;       // bytes
  constexpr int CP_A = BM / 16 / NW, CP_B = BN / 16 / NW;  // copy instructions per wavefront and stage
  constexpr int CP = CP_A + CP_B;
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "copy split");
  static_assert(TM <= 4, "row sub-tile dispatch below covers up to four");
  static_assert(STAGES >= 3 && STAGES <= 5, "prologue and tail are written for 2 to 4 steps of copy-ahead");
  static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU needs gate and up tiles in one wave");
  typedef __attribute__((address_space(1))) const void* gptr;
  typedef __attribute__((address_space(3))) void* lptr;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto stage_of = [](int kt) { return (STAGES & (STAGES - 1)) == 0 ? (kt & (STAGES - 1)) : kt % STAGES; };

  // Tile -> workgroup map.  Workgroup i runs on XCD i % 8; each XCD takes a contiguous eighth of
  // every problem's tiles (neighbouring tiles share activations / weights in that XCD's L2), and
  // works through the problem with the longer K first so that the cheap tiles fill the last round.
  // A dense problem (no tile list) is split by whole row-tiles instead: XCD x owns n_m / 8 of them
  // (the first n_m % 8 XCDs one more), so that the order below can walk its own block of the
  // output; its workgroup budget per XCD is that of the XCDs with one more.
  const int nm0 = a2.p0.tiles ? *a2.p0.tile_count : (a2.p0.M + BM - 1) / BM;
  const int nm1 = a2.two ? (a2.p1.tiles ? *a2.p1.tile_count : (a2.p1.M + BM - 1) / BM) : 0;
  const int t0 = nm0 * a2.p0.n_col_tiles, t1 = nm1 * a2.p1.n_col_tiles;
  const int px0 = a2.p0.tiles ? (t0 + 7) >> 3 : ((nm0 + 7) >> 3) * a2.p0.n_col_tiles;
  const int px1 = !a2.two ? 0 : a2.p1.tiles ? (t1 + 7) >> 3 : ((nm1 + 7) >> 3) * a2.p1.n_col_tiles;
  const int xcd = blockIdx.x & 7;
  int local = blockIdx.x >> 3;
  const bool p1_first = a2.two && a2.p1.K > a2.p0.K;
  bool second;  // uniform: this workgroup serves the second problem
  if (p1_first) {
    second = local < px1;
    if (!second) local -= px1;
  } else {
    second = local >= px0;
    if (second) local -= px0;
  }
  if (local >= (second ? px1 : px0)) return;
  const GemmArgs g = second ? a2.p1 : a2.p0;
  int m_idx, n_idx, logical = 0;
  if (g.tiles) {
    logical = xcd * (second ? px1 : px0) + local;
    if (logical >= (second ? t1 : t0)) return;
    m_idx = logical / g.n_col_tiles;
    n_idx = logical - m_idx * g.n_col_tiles;
  } else {
    // The XCD's G row-tiles times all column tiles, column tiles taken in pairs and inside a pair
    // the row-tile slower than the column: a row-tile's activations are needed again by the very
    // next workgroup and a column tile's weights by the one after that, down the whole block,
    // instead of the weights coming back only after a full row of column tiles.
    const int nm = second ? nm1 : nm0;
    const int G = (nm >> 3) + (xcd < (nm & 7));
    if (local >= G * g.n_col_tiles) return;
    const int blk = local / (2 * G), within = local - blk * 2 * G;
    int j;
    if (blk * 2 + 1 < g.n_col_tiles) { j = within >> 1; n_idx = blk * 2 + (within & 1); }
    else { j = within; n_idx = blk * 2; }
    m_idx = xcd * (nm >> 3) + min(xcd, nm & 7) + j;
  }

  int row_begin, row_end;
  const unsigned char* Bbase;
  if (g.tiles) {
    // One read of any record of the group tells everything.  Inside one group's block of tiles
    // the column index runs slowest: the row-tiles of a slot that use the same weight columns are
    // neighbours in launch order and meet in L2 (up to two row-tiles; see below for more).
    const MTile t = g.tiles[m_idx];
    const int in_group = t.pad >> 16;
    int j = t.pad & 0xFFFF;
    if (in_group > 1) {
      const int r = logical - (m_idx - j) * g.n_col_tiles;
      if (in_group >= 3) {
        // three or more row-tiles: column tiles are taken in pairs and inside a pair the row-tile
        // runs slower than the column, so that a row-tile's activations are needed again by the
        // very next workgroup instead of in_group workgroups later (by then L2 has dropped them)
        const int blk = r / (2 * in_group), within = r - blk * 2 * in_group;
        if (blk * 2 + 1 < g.n_col_tiles) { j = within >> 1; n_idx = blk * 2 + (within & 1); }
        else { j = within; n_idx = blk * 2; }
      } else {
        n_idx = r / in_group;
        j = r - n_idx * in_group;
      }
    }
    tile_span(t.group_begin, t.group_end, in_group, j, BM, row_begin, row_end);
    Bbase = static_cast<const unsigned char*>(g.b_sel >= 0 ? t.w[g.b_sel] : (g.B_tab ? g.B_tab[t.group] : g.B_one));
  } else {
    row_begin = m_idx * BM;
    row_end = min(g.M, row_begin + BM);
    Bbase = static_cast<const unsigned char*>(g.B_one);
  }
  const unsigned char* Abase = static_cast<const unsigned char*>(g.A);
  const int n0 = n_idx * BN_OUT;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform: keeps per-wavefront offsets in SGPRs
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- copy plan: instruction i of this wavefront fills rows [(wave*CP_x + i)*16, +16) of the A
  // (then B) part of a stage; lane l owns row l/4 of those, physical chunk l%4.
  // The source address of a copy is a wavefront-uniform 64-bit base (the tile's first row of A, the
  // weight matrix) kept in scalar registers plus a 32-bit per-lane byte offset that never changes:
  // walking K only advances the two scalar bases, no vector arithmetic.
  uint32_t cp_off[CP];
  int cp_dst[CP];  // wavefront-uniform LDS offset of the 1 KiB window inside a stage
#pragma unroll
  for (int i = 0; i < CP; ++i) {
    const bool isA = i < CP_A;
    const int blk = isA ? wave * CP_A + i : wave * CP_B + (i - CP_A);
    const int row = blk * 16 + (lane >> 2);
    const int chunk = (lane & 3) ^ swz32(row);
    if (isA) {
      const int rrow = min(row, row_end - row_begin - 1);  // rows past the tile re-read its last row
      cp_off[i] = g.a_rows > 0 ? static_cast<uint32_t>((rrow * 32 + chunk * 8) * 2)
                               : static_cast<uint32_t>((static_cast<int64_t>(rrow) * g.lda + chunk * 8) * 2);
      cp_dst[i] = blk * 1024;
    } else {
      if (g.b_tiled) {
        // padded row index of this LDS row in the tiled matrix (gate half first, then up half)
        int R;
        if (EPI == EPI_SWIGLU) {
          const int half = row >= BN / 2;
          R = min(n0 + row - half * (BN / 2), g.b_rows_pad - 1) + half * g.b_rows_pad;
        } else {
          R = min(n0 + row, g.b_rows_pad - 1);
        }
        const int64_t panel = static_cast<int64_t>(R / kWeightTileRows) * (g.K / kWeightTileK) * kWeightTileRows;
        cp_off[i] = static_cast<uint32_t>(((panel + (R % kWeightTileRows)) * kWeightTileK + chunk * 8) * 2);
      } else {
        int brow;
        if (EPI == EPI_SWIGLU) {
          const int half = row >= BN / 2;
          const int col = min(n0 + row - half * (BN / 2), g.n_out - 1);
          brow = col + half * g.n_out;
        } else {
          brow = min(n0 + row, g.n_out - 1);
        }
        cp_off[i] = static_cast<uint32_t>((static_cast<int64_t>(brow) * g.ldb + chunk * 8) * 2);
      }
      cp_dst[i] = BM * 64 + blk * 1024;
    }
  }
  // The copy is written as inline assembly on purpose: the compiler's wait-count bookkeeping treats
  // a global_load_lds it knows about as "may touch both memory and LDS" and from then on turns
  // every LDS wait into a full drain, which would undo the software pipeline.  Issued this way the
  // copies are invisible to that bookkeeping and are waited for explicitly before each barrier.
  const uint32_t smem_lds = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lptr)smem));
  auto uniform64 = [](uint64_t v) {
    // the builtin returns a signed int: widen both halves as unsigned
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v >> 32)));
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
    return (static_cast<uint64_t>(hi) << 32) | lo;
  };
  const uint64_t base_a = uniform64(reinterpret_cast<uint64_t>(Abase) + static_cast<uint64_t>(row_begin) * (g.a_rows > 0 ? 32 : g.lda) * 2);
  const uint64_t kstep_a = g.a_rows > 0 ? static_cast<uint64_t>(g.a_rows) * 64 : 64;
  const uint64_t base_b = uniform64(reinterpret_cast<uint64_t>(Bbase));
  const uint32_t kstep_b = g.b_tiled ? kWeightTileRows * kWeightTileK * 2 : 64;  // bytes between K-steps of B
  auto issue_copy = [&](int kt) {
    const uint32_t stage = smem_lds + stage_of(kt) * STAGE;
    const uint64_t src_a = base_a + static_cast<uint64_t>(kt) * kstep_a;
    const uint64_t src_b = base_b + static_cast<uint64_t>(kt) * kstep_b;
#pragma unroll
    for (int i = 0; i < CP; ++i) {
      const uint32_t dst = __builtin_amdgcn_readfirstlane(stage + cp_dst[i]);
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(cp_off[i]), "s"(i < CP_A ? src_a : src_b), "s"(dst) : "memory", "m0");
    }
  };

  // The same with the ring position PH of the destination stage known at compile time.
  auto issue_copy_at = [&](int kt, auto ph_tag) {
    constexpr int PH = decltype(ph_tag)::value;
    const uint64_t src_a = base_a + static_cast<uint64_t>(kt) * kstep_a;
    const uint64_t src_b = base_b + static_cast<uint64_t>(kt) * kstep_b;
#pragma unroll
    for (int i = 0; i < CP; ++i) {
      const uint32_t dst = __builtin_amdgcn_readfirstlane(smem_lds + cp_dst[i] + PH * STAGE);
      const uint32_t off = cp_off[i];
      const uint64_t src = i < CP_A ? src_a : src_b;
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(src), "s"(dst) : "memory", "m0");
    }
  };

  // ---- per-lane fragment addresses.  32-row sub-tiles are dealt round-robin to the wavefront
  // rows (sub-tile tm*WAVES_M + wm), so a ragged row-tile keeps every wavefront equally busy.
  // Every fragment row of a lane is (a multiple of 32) + lane % 32, so the swizzle term depends on
  // the lane only: the lane keeps one loop-invariant byte offset per operand and half-step, and
  // the individual fragments are reached with immediate offsets from it.
  const int lrow = lane & 31;
  int a_off[2], b_off[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int sw = ((ks * 2 + (lane >> 5)) ^ swz32(lrow)) << 4;
    a_off[ks] = (wm * 32 + lrow) * 64 + sw;
    b_off[ks] = (BM + (EPI == EPI_SWIGLU ? wn * (WN / 2) : wn * WN) + lrow) * 64 + sw;
  }
  // The same bases two stages further on: with the ring position known at compile time every
  // fragment of every stage is an immediate offset below 64 KiB away from one of the two.
  int a_off2[2], b_off2[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_off2[ks] = a_off[ks] + 2 * STAGE;
    b_off2[ks] = b_off[ks] + 2 * STAGE;
  }
  constexpr int A_STEP = WAVES_M * 32 * 64;  // bytes between a wavefront's successive row sub-tiles
  auto b_imm = [](int tn) {                   // byte offset of column tile tn from the lane's base
    if (EPI == EPI_SWIGLU) return ((tn >= TN / 2 ? BN / 2 : 0) + (tn % (TN / 2 > 0 ? TN / 2 : 1)) * 32) * 64;
    return tn * 32 * 64;
  };
  f32x16 acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.f;

  // A ragged row-tile leaves some 32-row sub-tiles of a wavefront without any valid row; the
  // main loop is instantiated for each count of valid sub-tiles so that those MFMAs (and their
  // fragment reads) are not issued at all.  The wavefront still takes part in copies and barriers.
  const int KT = g.K >> 5;
  const int n_sub = (row_end - row_begin + 31) >> 5;  // sub-tiles holding at least one valid row
  const int tm_valid = min(TM, max(0, (n_sub - wm + WAVES_M - 1) / WAVES_M));

  auto run = [&](auto tmv_tag) {
    constexpr int TMV = decltype(tmv_tag)::value;
    auto load_frags = [&](const unsigned char* base, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
      if (TMV == 0) return;
      const unsigned char* pa = base + a_off[ks];
      const unsigned char* pb = base + b_off[ks];
#pragma unroll
      for (int tm = 0; tm < TMV; ++tm) af[tm] = *reinterpret_cast<const bf16x8*>(pa + tm * A_STEP);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) bfr[tn] = *reinterpret_cast<const bf16x8*>(pb + b_imm(tn));
    };
    auto mfma_step = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
      for (int tm = 0; tm < TMV; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tn], af[tm], acc[tm][tn], 0, 0, 0);
    };
    // One K-step.  COPY: issue the copy of step kt+3.  VM: copies that may stay pending at the
    // barrier (those of the steps after kt+1).  LAST: no next stage to publish.
    bf16x8 af0[TM], bf0[TN], af1[TM], bf1[TN];
    auto step = [&](int kt, auto copy_tag, auto vm_tag, auto last_tag) {
      constexpr bool COPY = decltype(copy_tag)::value, LAST = decltype(last_tag)::value;
      constexpr int VM = decltype(vm_tag)::value;
      const unsigned char* cur = smem + stage_of(kt) * STAGE;
      // stage (kt+3)%4 held step kt-1, which every wavefront finished reading before the last barrier
      if (COPY) issue_copy(kt + D);
      load_frags(cur, 1, af1, bf1);
      __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the MFMAs they overlap with
      mfma_step(af0, bf0);
      __builtin_amdgcn_sched_barrier(0);
      if (!LAST) {
        // this wavefront's copies of step kt+1 have landed once only VM newer copies are pending;
        // all its fragment reads of the current stage have returned (lgkmcnt 0)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(VM));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        load_frags(smem + stage_of(kt + 1) * STAGE, 0, af0, bf0);
        __builtin_amdgcn_sched_barrier(0);
      }
      mfma_step(af1, bf1);
      __builtin_amdgcn_sched_barrier(0);
    };
    // The MFMAs of one half-step with the fragment reads of the next half-step dealt in between
    // them (one read after each of the first MFMAs; the order is pinned with scheduling groups):
    // the reads then issue in the shadow of the matrix pipe instead of in a block ahead of it.
    auto mfma_reads_at = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN], auto ph_tag, int ks, bf16x8 (&naf)[TM],
                             bf16x8 (&nbf)[TN]) {
      constexpr int PH = decltype(ph_tag)::value;
      if (TMV == 0) return;
      const unsigned char* pa = smem + (PH >= 2 ? a_off2[ks] : a_off[ks]) + (PH & 1) * STAGE;
      const unsigned char* pb = smem + (PH >= 2 ? b_off2[ks] : b_off[ks]) + (PH & 1) * STAGE;
      constexpr int NR = TMV + TN, NM = TMV * TN;  // reads, MFMAs
#pragma unroll
      for (int tm = 0; tm < TMV; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tn], af[tm], acc[tm][tn], 0, 0, 0);
          const int idx = tm * TN + tn;
          if (idx < TMV) naf[idx] = *reinterpret_cast<const bf16x8*>(pa + idx * A_STEP);
          else if (idx < NR) nbf[idx - TMV] = *reinterpret_cast<const bf16x8*>(pb + b_imm(idx - TMV));
        }
#pragma unroll
      for (int idx = NM; idx < NR; ++idx) {  // fewer MFMAs than reads: the remaining reads follow
        if (idx < TMV) naf[idx] = *reinterpret_cast<const bf16x8*>(pa + idx * A_STEP);
        else nbf[idx - TMV] = *reinterpret_cast<const bf16x8*>(pb + b_imm(idx - TMV));
      }
      constexpr int PAIRS = NR < NM ? NR : NM;
#pragma unroll
      for (int i = 0; i < PAIRS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
      }
      if (NM > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, NM - PAIRS, 0);
      if (NR > PAIRS) __builtin_amdgcn_sched_group_barrier(0x100, NR - PAIRS, 0);
    };
    // Steady-state forms of the two steps (the late group's is described below) for a four-stage
    // ring, with the ring position PH = kt % 4 known at compile time: stage addresses fold into
    // immediates and the K loop, unrolled by four, carries no vector ALU instruction at all.
    auto step_at = [&](int kt, auto ph_tag) {
      constexpr int PH = decltype(ph_tag)::value;
      issue_copy_at(kt + D, std::integral_constant<int, (PH + D) & 3>{});
      __builtin_amdgcn_sched_barrier(0);
      mfma_reads_at(af0, bf0, ph_tag, 1, af1, bf1);
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((D - 1) * CP));
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      mfma_reads_at(af1, bf1, std::integral_constant<int, (PH + 1) & 3>{}, 0, af0, bf0);
      __builtin_amdgcn_sched_barrier(0);
    };
    auto step_late_at = [&](int kt, auto ph_tag) {
      constexpr int PH = decltype(ph_tag)::value;
      mfma_reads_at(af0, bf0, ph_tag, 1, af1, bf1);
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((D - 1) * CP));
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      issue_copy_at(kt + D + 1, ph_tag);  // (PH + 4) % 4: into this step's own stage
      __builtin_amdgcn_sched_barrier(0);
      mfma_reads_at(af1, bf1, std::integral_constant<int, (PH + 1) & 3>{}, 0, af0, bf0);
      __builtin_amdgcn_sched_barrier(0);
    };
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    using P3 = std::integral_constant<int, 3>;
    // Skewed schedule.  Both wavefronts of a SIMD (w and w + NW/2) would otherwise leave the
    // barrier in lockstep and do their non-MFMA work (copy issue, address arithmetic) at the same
    // time, leaving the matrix pipe idle.  The late group issues its copy right after the barrier
    // (one step further ahead) instead of after the second half-step's MFMAs, so one group's
    // overhead always runs under the other group's MFMAs.
    auto step_late = [&](int kt, auto copy_tag, auto vm_tag, auto last_tag) {
      constexpr bool COPY = decltype(copy_tag)::value, LAST = decltype(last_tag)::value;
      constexpr int VM = decltype(vm_tag)::value;
      const unsigned char* cur = smem + stage_of(kt) * STAGE;
      load_frags(cur, 1, af1, bf1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_step(af0, bf0);
      __builtin_amdgcn_sched_barrier(0);
      if (!LAST) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(VM));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (COPY) issue_copy(kt + D + 1);  // into this step's own stage: all its reads ended before the barrier
        load_frags(smem + stage_of(kt + 1) * STAGE, 0, af0, bf0);
        __builtin_amdgcn_sched_barrier(0);
      }
      mfma_step(af1, bf1);
      __builtin_amdgcn_sched_barrier(0);
    };
    // Tail: with j copies-ahead steps left, (j - 1) * CP copies may stay pending at the barrier.
    auto tail = [&](auto& fn, int& kt) {
      if (D >= 4 && kt + 4 < KT) { fn(kt, F{}, std::integral_constant<int, 3 * CP>{}, F{}); ++kt; }
      if (D >= 3 && kt + 3 < KT) { fn(kt, F{}, std::integral_constant<int, 2 * CP>{}, F{}); ++kt; }
      if (D >= 2 && kt + 2 < KT) { fn(kt, F{}, std::integral_constant<int, CP>{}, F{}); ++kt; }
      if (kt + 1 < KT) { fn(kt, F{}, std::integral_constant<int, 0>{}, F{}); ++kt; }
      fn(kt, F{}, std::integral_constant<int, 0>{}, T{});
    };
    constexpr int VM_STEADY = (D - 1) * CP;
    if (wave < NW / 2) {
      load_frags(smem, 0, af0, bf0);
      int kt = 0;
      if constexpr (STAGES == 4)  // kt stays a multiple of four here: ring position = unrolled position
        for (; kt + D + 3 < KT; kt += 4) { step_at(kt, P0{}); step_at(kt + 1, P1{}); step_at(kt + 2, P2{}); step_at(kt + 3, P3{}); }
      for (; kt + D < KT; ++kt) step(kt, T{}, std::integral_constant<int, VM_STEADY>{}, F{});
      // here kt + D >= KT: the copies of every remaining step are already issued
      if (D >= 4 && kt + 3 < KT) { step(kt, F{}, std::integral_constant<int, 2 * CP>{}, F{}); ++kt; }
      if (D >= 3 && kt + 2 < KT) { step(kt, F{}, std::integral_constant<int, CP>{}, F{}); ++kt; }
      if (kt + 1 < KT) { step(kt, F{}, std::integral_constant<int, 0>{}, F{}); ++kt; }
      step(kt, F{}, std::integral_constant<int, 0>{}, T{});
    } else {
      if (KT > D) issue_copy(D);
      load_frags(smem, 0, af0, bf0);
      int kt = 0;
      if constexpr (STAGES == 4)
        for (; kt + D + 4 < KT; kt += 4) { step_late_at(kt, P0{}); step_late_at(kt + 1, P1{}); step_late_at(kt + 2, P2{}); step_late_at(kt + 3, P3{}); }
      for (; kt + D + 1 < KT; ++kt) step_late(kt, T{}, std::integral_constant<int, VM_STEADY>{}, F{});
      tail(step_late, kt);
    }
  };

  // prologue: copies of the first D steps, then publish step 0
  issue_copy(0);
  if (KT > 1) issue_copy(1);
  if (D >= 3 && KT > 2) issue_copy(2);
  if (D >= 4 && KT > 3) issue_copy(3);
  asm volatile("" ::: "memory");
  if (D >= 4 && KT > 3) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(3 * CP));
  else if (D >= 3 && KT > 2) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * CP));
  else if (KT > 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(CP));
  else __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  switch (tm_valid) {
    case 0: run(std::integral_constant<int, 0>{}); break;
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: run(std::integral_constant<int, (TM >= 2 ? 2 : TM)>{}); break;
    case 3: run(std::integral_constant<int, (TM >= 3 ? 3 : TM)>{}); break;
    default: run(std::integral_constant<int, TM>{}); break;
  }

  // ---- epilogue.  Per 32x32 tile a lane holds, for q = 0..3, the four columns
  // q*8 + (lane/32)*4 + {0..3} of activation row lane % 32.  Each wavefront transposes its
  // outputs through its own slice of LDS (padded rows: conflict-free 8-byte writes) and stores
  // them to global memory as full 16-byte words, a whole row segment per group of lanes.
  constexpr int TN_OUT = EPI == EPI_SWIGLU ? TN / 2 : TN;
  constexpr int WN_OUT = EPI == EPI_SWIGLU ? WN / 2 : WN;
  static_assert(EPI != EPI_F32, "this kernel stores bf16");
  constexpr int ROWB = WN_OUT * 2 + 8;          // bytes between rows of the wavefront's LDS slice
  constexpr int SLICE = TM * 32 * ROWB;
  constexpr int LPR = WN_OUT * 2 / 16;          // lanes per row when reading back
  constexpr int RPI = 64 / LPR;                 // rows per read-back instruction
  __syncthreads();                              // every wavefront is done with the copy stages
  unsigned char* slice = smem + wave * SLICE;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    if (tm >= tm_valid) break;
#pragma unroll
    for (int tn = 0; tn < TN_OUT; ++tn) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (EPI == EPI_SWIGLU) v[r] = silu_f32(acc[tm][tn][q * 4 + r]) * acc[tm][tn + TN / 2][q * 4 + r];
          else v[r] = acc[tm][tn][q * 4 + r];
        }
        u32x2 o = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<u32x2*>(slice + (tm * 32 + (lane & 31)) * ROWB + (tn * 32 + q * 8 + (lane >> 5) * 4) * 2) = o;
      }
    }
  }
  // read back: lane l takes 16 bytes (8 columns) of row l / LPR of each group of RPI rows
  const int rcol = (lane % LPR) * 8;
  const int col = n0 + wn * WN_OUT + rcol;
  if (col < g.n_out) {  // n_out is a multiple of 8: a word is entirely inside or outside
#pragma unroll
    for (int it = 0; it < TM * 32 / RPI; ++it) {
      const int lrow = it * RPI + lane / LPR;     // row inside the wavefront's slice
      const int tm = lrow >> 5;
      if (tm >= tm_valid) break;
      const int row = row_begin + (tm * WAVES_M + wm) * 32 + (lrow & 31);
      if (row < row_end) {
        const u32x4 o = *reinterpret_cast<const u32x4*>(slice + lrow * ROWB + rcol * 2);
        uint16_t* dst = static_cast<uint16_t*>(g.C);
        // a 16-byte word is 8 columns inside one 32-column panel
        if (g.c_rows > 0) dst += (static_cast<int64_t>(col / kWeightTileK) * g.c_rows + row) * kWeightTileK + col % kWeightTileK;
        else dst += static_cast<int64_t>(row) * g.ldc + col;
        *reinterpret_cast<u32x4*>(dst) = o;
      }
    }
  }
}

// Launch helpers: grids cover `max_m_tiles` row-tiles per problem (upper bounds; surplus
// workgroups exit at once).
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int KID>
int launch_gemm_bf16(revive_ctx* ctx, const GemmArgs& args, int max_m_tiles, hipStream_t stream) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr size_t lds = 2 * (BM + BN) * 128;
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, EPI, KID>;
  REVIVE_HIP(ctx, allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
  const int64_t total = static_cast<int64_t>(max_m_tiles) * args.n_col_tiles;
  if (total <= 0) return REVIVE_OK;
  const int grid = static_cast<int>((total + 7) / 8 * 8);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, stream, args);
  return check_hip(ctx, hipGetLastError(), "gemm_bf16 launch");
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int KID, int STAGES = 4>
int launch_gemm_bf16_dma(revive_ctx* ctx, const GemmArgs& p0, int max_m_tiles0, const GemmArgs* p1, int max_m_tiles1,
                         hipStream_t stream) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WN_OUT_ = (EPI == EPI_SWIGLU ? BN / 2 : BN) / WAVES_N;
  constexpr size_t lds_epi = static_cast<size_t>(WAVES_M * WAVES_N) * (BM / WAVES_M) * (WN_OUT_ * 2 + 8);
  constexpr size_t lds_ring = STAGES * (BM + BN) * 64;
  constexpr size_t lds = lds_ring > lds_epi ? lds_ring : lds_epi;
  auto kern = gemm_bf16_dma_kernel<BM, BN, WAVES_M, WAVES_N, EPI, KID, STAGES>;
  REVIVE_HIP(ctx, allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
  GemmArgs2 a{};
  a.p0 = p0;
  a.two = p1 != nullptr;
  if (p1) a.p1 = *p1;
  auto budget = [](const GemmArgs& p, int max_m_tiles) -> int64_t {  // workgroups per XCD, as the kernel splits the problem
    return p.tiles ? (static_cast<int64_t>(max_m_tiles) * p.n_col_tiles + 7) / 8 : static_cast<int64_t>((max_m_tiles + 7) / 8) * p.n_col_tiles;
  };
  const int64_t per_xcd = budget(p0, max_m_tiles0) + (p1 ? budget(*p1, max_m_tiles1) : 0);
  if (per_xcd <= 0) return REVIVE_OK;
  const int grid = static_cast<int>(per_xcd * 8);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, stream, a);
  return check_hip(ctx, hipGetLastError(), "gemm_bf16_dma launch");
}

}  // namespace revive
