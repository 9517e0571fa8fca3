// Grouped bf16 GEMM, both operands unit-stride along the contraction ("NT"):
//
//   C[g] (M x N, fp32) = A[g] (M x Kd) * B[g]^T,   A stored [M][Kd], B stored [N][Kd]
//
// Each operand is either fp32 (rounded to bf16 nearest-even while it is staged) or already
// bf16 (a rounded copy made once by its producer), chosen per operand at compile time.
// Every GEMM of the bf16 training step is brought into this one shape by keeping transposed
// bf16 copies of the operands whose natural layout is contraction-major (see hpsgd_api.hip).
//
// Tile 128 x 128 x 64 per workgroup of 4 waves (each wave 64 x 64 = 2 x 2 blocks of
// v_mfma_f32_32x32x16_bf16), LDS double-buffered with one barrier per k-tile: while the
// matrix cores work on buffer kt&1, the global loads of tile kt+1 are in flight and are
// written to the other buffer afterwards.  72 KB of LDS per workgroup keeps two workgroups
// per CU, so one's barrier wait is covered by the other's MFMAs.
// LDS rows are [i][k] with a pitch of 72 halves (144 B): the 16-byte operand reads of 16
// consecutive rows then fall on 64 distinct banks.
#include "kernels.h"

namespace hpsgd {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int NBM = 128, NBN = 128, NBK = 64, NPITCH = NBK + 8;
static constexpr int NTHREADS = 256;

// 8 consecutive contraction elements of one row, as loaded from memory.  Loads are
// branch-free and nothing touches the loaded registers until they are packed for LDS (any
// use would force a wait right after the load and undo the prefetch): the caller clamps the
// row and the column into range (rows beyond M or N only feed outputs that are never stored)
// and a unit that lies beyond Kd is zeroed when it is packed.
template <typename T>
struct Unit8;

template <>
struct Unit8<float> {
  float4 lo, hi;
  __device__ __forceinline__ void load(const float* __restrict__ p) {
    lo = *reinterpret_cast<const float4*>(p);
    hi = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ bf16x8 pack(bool valid) const {
    bf16x8 v;
    v[0] = (__bf16)lo.x; v[1] = (__bf16)lo.y; v[2] = (__bf16)lo.z; v[3] = (__bf16)lo.w;
    v[4] = (__bf16)hi.x; v[5] = (__bf16)hi.y; v[6] = (__bf16)hi.z; v[7] = (__bf16)hi.w;
    if (!valid) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.f;
    }
    return v;
  }
};

template <>
struct Unit8<__bf16> {
  bf16x8 v;
  __device__ __forceinline__ void load(const __bf16* __restrict__ p) {
    v = *reinterpret_cast<const bf16x8*>(p);
  }
  __device__ __forceinline__ bf16x8 pack(bool valid) const {
    bf16x8 r = v;
    if (!valid) {
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = (__bf16)0.f;
    }
    return r;
  }
};

struct GemmNtDesc {
  const void* A; long lda; long strideA;   // in elements of A's type
  const void* B; long ldb; long strideB;
  float* C; long ldc; long strideC;
  const float* bias; long strideBias;      // per column n, nullable
  const float* win; long strideWin;        // nullable; else C = win - lr * acc (win has C's layout, may be C)
  float lr;
  int M, N, Kd, groups;
};

// Workgroup -> (group, tile).  Returns false for the padding of the last round of slow tiles.
__device__ __forceinline__ bool nt_tile(const GemmNtDesc& d, int& g, int& tile_m, int& tile_n) {
  // Tile order.  Workgroup i runs on XCD i % 8 and every XCD has its own L2.  The dimension
  // with more tiles ("slow") is dealt out to the XCDs (tile s goes to XCD s % 8), and on an
  // XCD consecutive workgroups sweep the other ("fast") dimension for a fixed slow tile:
  // the slow operand's tile is then fetched from memory by one L2 only and is reused at once
  // by all fast tiles, while the fast operand (the smaller one) stays resident in every L2.
  {
    const int tm = (d.M + NBM - 1) / NBM, tn = (d.N + NBN - 1) / NBN;
    const bool slow_is_n = tn >= tm;
    const int ts = slow_is_n ? tn : tm, tf = slow_is_n ? tm : tn;
    const int s8 = (ts + 7) >> 3;
    const int c = blockIdx.x & 7, li = blockIdx.x >> 3;
    const int f = li % tf, sl = (li / tf) % s8;
    g = li / (tf * s8);
    const int st = c + 8 * sl;
    if (st >= ts) return false;
    tile_m = slow_is_n ? f : st;
    tile_n = slow_is_n ? st : f;
  }
  return true;
}

// Epilogue of both NT kernels: accumulators -> LDS tile -> coalesced 16-byte stores.
// The epilogue's traffic is used once (the matrix to update is read once, the result is read by a
// later kernel at the earliest): non-temporal, so that it does not push the operand panels, which
// other tiles of the XCD are still reading, out of the L2.
typedef float f4nt_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float* p) {
  const f4nt_t v = __builtin_nontemporal_load(reinterpret_cast<const f4nt_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store4(float* p, float4 v) {
  const f4nt_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<f4nt_t*>(p));
}

template <bool COMMIT>
__device__ __forceinline__ void nt_epilogue(const GemmNtDesc& d, floatx16 (&acc)[2][2], unsigned char* nt_smem,
                                            int g, int m0, int n0) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int lrow = lane & 31, lk = lane >> 5;
  // Epilogue through LDS (the operand buffers are free after the last barrier): the
  // accumulators are laid out as the 128 x 128 tile, then every wave instruction moves two
  // whole 512-byte row segments, so the stores (and the loads of W in the commit form, all
  // requested before the first is used) are fully coalesced 16-byte accesses.
  float* C = d.C + (long)g * d.strideC;
  const float* bias = d.bias ? d.bias + (long)g * d.strideBias : nullptr;
  float* sC = reinterpret_cast<float*>(nt_smem);
  constexpr int CP = NBN + 4;  // pitch in floats
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        sC[(wm * 64 + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4)) * CP + wn * 64 + j * 32 + lrow] = acc[i][j][v];
  __syncthreads();
  const int c4 = (tid & 31) << 2, rbase = tid >> 5;
  const int col = n0 + c4;
  const bool vec = ((d.ldc | d.strideC) & 3) == 0 && ((uintptr_t)d.C & 15) == 0 &&
                   (!COMMIT || (((uintptr_t)d.win & 15) == 0 && (d.strideWin & 3) == 0));
  if (vec && col + 3 < d.N) {
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!COMMIT && bias) bv = make_float4(bias[col], bias[col + 1], bias[col + 2], bias[col + 3]);
    float4 w[COMMIT ? 16 : 1];
    if (COMMIT) {
      const float* W = d.win + (long)g * d.strideWin;
#pragma unroll
      for (int p = 0; p < 16; ++p) {
        const int row = min(m0 + rbase + 8 * p, d.M - 1);  // clamped: not stored when outside
        w[COMMIT ? p : 0] = nt_load4(W + (long)row * d.ldc + col);
      }
    }
#pragma unroll
    for (int p = 0; p < 16; ++p) {
      const int rl = rbase + 8 * p, row = m0 + rl;
      if (row >= d.M) continue;
      const float4 a = *reinterpret_cast<const float4*>(&sC[rl * CP + c4]);
      float4 o;
      if (COMMIT) {
        const float4 wv = w[COMMIT ? p : 0];
        o = make_float4(wv.x - d.lr * a.x, wv.y - d.lr * a.y, wv.z - d.lr * a.z, wv.w - d.lr * a.w);
      } else {
        o = make_float4(a.x + bv.x, a.y + bv.y, a.z + bv.z, a.w + bv.w);
      }
      nt_store4(C + (long)row * d.ldc + col, o);
    }
  } else {
    const float* W = COMMIT ? d.win + (long)g * d.strideWin : nullptr;
    for (int p = 0; p < 16; ++p) {
      const int rl = rbase + 8 * p, row = m0 + rl;
      if (row >= d.M) continue;
      for (int e = 0; e < 4; ++e) {
        if (col + e >= d.N) break;
        const long off = (long)row * d.ldc + col + e;
        const float a = sC[rl * CP + c4 + e];
        C[off] = COMMIT ? W[off] - d.lr * a : a + (bias ? bias[col + e] : 0.f);
      }
    }
  }
}

// COMMIT: the epilogue is C = win - lr * acc; the tile of win is requested before the
// contraction starts, so that the epilogue does not wait for it.
template <typename TA, typename TB, bool COMMIT>
__global__ void __launch_bounds__(NTHREADS, 2)
gemm_bf16_nt_kernel(GemmNtDesc d) {
  constexpr int UPT = NBM * (NBK / 8) / NTHREADS;  // 8-element units per thread per operand (4)
  extern __shared__ __attribute__((aligned(16))) unsigned char nt_smem[];
  __bf16(*sA)[NBM * NPITCH] = reinterpret_cast<__bf16(*)[NBM * NPITCH]>(nt_smem);
  __bf16(*sB)[NBN * NPITCH] = reinterpret_cast<__bf16(*)[NBN * NPITCH]>(nt_smem + 2 * NBM * NPITCH * 2);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int lrow = lane & 31, lk = lane >> 5;
  int g, tile_m, tile_n;
  if (!nt_tile(d, g, tile_m, tile_n)) return;  // padding of the last round of slow tiles
  const int m0 = tile_m * NBM, n0 = tile_n * NBN;
  const TA* __restrict__ A = reinterpret_cast<const TA*>(d.A) + (long)g * d.strideA;
  const TB* __restrict__ B = reinterpret_cast<const TB*>(d.B) + (long)g * d.strideB;

  // two register stages: while tile kt is multiplied out of LDS, the global loads of tiles
  // kt+1 and kt+2 are in flight
  Unit8<TA> ra[2][UPT];
  Unit8<TB> rb[2][UPT];
  // per-thread row bases (clamped into the matrix) are loop invariants
  const TA* arow[UPT];
  const TB* brow[UPT];
#pragma unroll
  for (int u = 0; u < UPT; ++u) {
    const int i = (tid + u * NTHREADS) >> 3;
    arow[u] = A + (long)min(m0 + i, d.M - 1) * d.lda;
    brow[u] = B + (long)min(n0 + i, d.N - 1) * d.ldb;
  }
  const int kofs = (tid & 7) << 3;  // NTHREADS is a multiple of 8: the same for every unit of a thread
  bool rvalid[2] = {true, true};
  auto load_tiles = [&](int st, int kt) {
    const int k = kt * NBK + kofs;
    rvalid[st] = k < d.Kd;                // Kd is a multiple of 8: a unit is all in or all out
    const int kc = rvalid[st] ? k : 0;
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      ra[st][u].load(arow[u] + kc);
      rb[st][u].load(brow[u] + kc);
    }
  };
  auto store_tiles = [&](int st, int buf) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * NTHREADS;
      const int i = unit >> 3, k = (unit & 7) << 3;
      *reinterpret_cast<bf16x8*>(&sA[buf][i * NPITCH + k]) = ra[st][u].pack(rvalid[st]);
      *reinterpret_cast<bf16x8*>(&sB[buf][i * NPITCH + k]) = rb[st][u].pack(rvalid[st]);
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < NBK; kk += 16) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wm * 64 + i * 32 + lrow) * NPITCH + kk + 8 * lk]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&sB[buf][(wn * 64 + j * 32 + lrow) * NPITCH + kk + 8 * lk]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // The loop body has no branch: tiles past the end of the contraction load from column 0
  // and are packed as zeros, so the extra stores and MFMAs of the last round add nothing.
  // (With conditionals around the loads the compiler can no longer count the outstanding
  // loads and waits for all of them before every LDS store, which undoes the prefetch.)
  const int nk = (d.Kd + NBK - 1) / NBK;
  load_tiles(0, 0);
  store_tiles(0, 0);
  load_tiles(0, 1);
  load_tiles(1, 2);
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    compute(0);               // tile kt
    store_tiles(0, 1);        // tile kt+1 -> buffer 1
    load_tiles(0, kt + 3);
    __syncthreads();
    compute(1);               // tile kt+1
    store_tiles(1, 0);        // tile kt+2 -> buffer 0
    load_tiles(1, kt + 4);
    __syncthreads();
  }

  nt_epilogue<COMMIT>(d, acc, nt_smem, g, m0, n0);
}

// ---------------------------------------------------------------------------- direct-to-LDS variant
// Both operands bf16: the tiles go from memory straight into LDS (global_load_lds_dwordx4: no
// staging registers, no conversion, no LDS store instructions).  A wave instruction fills 1 KB
// of LDS, lane j at byte 16*j, i.e. 8 rows of 128 bytes; rows carry no padding, so the 16-byte
// chunks of a row are stored XOR-swizzled (chunk c of row r sits at position c ^ ((r >> 1) & 7)):
// the 16 rows a quarter-wave reads for one MFMA operand then fall on 64 distinct banks.
// Chunks beyond Kd (ragged last k-tile) are read from 16 zero bytes instead.  Two LDS stages
// (64 KB, raised to the 66 KB of the epilogue tile): two workgroups per CU.
__device__ __attribute__((aligned(16))) unsigned nt_zero16[4] = {0u, 0u, 0u, 0u};

#define HPSGD_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define HPSGD_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

template <bool COMMIT>
__global__ void __launch_bounds__(NTHREADS, 2)
gemm_bf16_dl_kernel(GemmNtDesc d) {
  extern __shared__ __attribute__((aligned(16))) unsigned char nt_smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int lrow = lane & 31, lk = lane >> 5;
  int g, tile_m, tile_n;
  if (!nt_tile(d, g, tile_m, tile_n)) return;
  const int m0 = tile_m * NBM, n0 = tile_n * NBN;
  const __bf16* __restrict__ A = reinterpret_cast<const __bf16*>(d.A) + (long)g * d.strideA;
  const __bf16* __restrict__ B = reinterpret_cast<const __bf16*>(d.B) + (long)g * d.strideB;
  // loader: wave w, instruction i covers tile rows (4w + i)*8 .. +7; lane j: row + (j >> 3),
  // LDS chunk j & 7, which holds the row's chunk (j & 7) ^ ((row >> 1) & 7).  Rows beyond M / N
  // are clamped (their products are never stored).
  const __bf16* ga[4];
  const __bf16* gb[4];
  int kofs[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (wave * 4 + i) * 8 + (lane >> 3);
    kofs[i] = ((lane & 7) ^ ((row >> 1) & 7)) * 8;
    ga[i] = A + (long)min(m0 + row, d.M - 1) * d.lda + kofs[i];
    gb[i] = B + (long)min(n0 + row, d.N - 1) * d.ldb + kofs[i];
  }
  const __bf16* zero = reinterpret_cast<const __bf16*>(nt_zero16);
  auto issue = [&](int stage, int kt) {
    unsigned char* sa = nt_smem + stage * 32768 + wave * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = kt * NBK + kofs[i] < d.Kd;  // Kd is a multiple of 8: a chunk is all in or all out
      __builtin_amdgcn_global_load_lds(HPSGD_GPTR(ok ? ga[i] + kt * NBK : zero), HPSGD_LPTR(sa + i * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(HPSGD_GPTR(ok ? gb[i] + kt * NBK : zero), HPSGD_LPTR(sa + 16384 + i * 1024),
                                       16, 0, 0);
    }
  };
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // operand fragments: row r, chunk c = 2*ks + lk at byte r*128 + ((c ^ ((r >> 1) & 7)) << 4)
  int ra[2], rb[2], swa[2], swb[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = wm * 64 + i * 32 + lrow, rn = wn * 64 + i * 32 + lrow;
    ra[i] = r * 128;
    swa[i] = (r >> 1) & 7;
    rb[i] = 16384 + rn * 128;
    swb[i] = (rn >> 1) & 7;
  }
  const int nk = (d.Kd + NBK - 1) / NBK;
  issue(0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    // The tile's loads are the only ones in flight.  A bare barrier: with __syncthreads the
    // compiler would add its own wait for every LDS-bound load, also the next tile's.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // tile kt is in LDS; everyone is done reading tile kt-1
    if (kt + 1 < nk) issue((kt + 1) & 1, kt + 1);
    const unsigned char* sb = nt_smem + (kt & 1) * 32768;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const bf16x8*>(sb + ra[i] + (((2 * ks + lk) ^ swa[i]) << 4));
        b[i] = *reinterpret_cast<const bf16x8*>(sb + rb[i] + (((2 * ks + lk) ^ swb[i]) << 4));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
  __syncthreads();  // the operand buffers become the epilogue tile
  nt_epilogue<COMMIT>(d, acc, nt_smem, g, m0, n0);
}

// ---------------------------------------------------------------------------- one workgroup per CU
// The same direct-to-LDS scheme with the whole CU given to one workgroup of WGM x WGN waves (two
// per SIMD), each wave owning (32 TM) x (32 TN) outputs, and S stages of LDS: the loads of the
// k-tiles kt+1 .. kt+S-1 are in flight while tile kt is multiplied, so that the memory latency is
// covered by S-1 tiles of matrix work instead of one (with two independent 4-wave workgroups per
// CU and two stages each, a workgroup waits for most of the latency on every k-tile).
// The fragments of contraction step ks+1 are read from LDS while the MFMAs of step ks run.
// A wave's share of a stage's loads is IPW instructions; a wave waits until all but the newest
// (S-2) IPW of its own loads have landed, and the barrier extends that to every wave's loads.
// S buffers hold tile kt and the S-1 tiles behind it.
// Tiles beyond the contraction are still "loaded" (from 16 zero bytes), so the count of loads
// in flight is the same on every trip.
template <int WGM, int WGN, int TM, int TN, int S>
struct DlxShape {
  static constexpr int NW = WGM * WGN, NT = 64 * NW;
  static constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
  static constexpr int ROWS = BM + BN;             // rows of 128 bytes per stage: A's, then B's
  static constexpr int IPW = ROWS / 8 / NW;        // loader instructions (8 rows each) per wave and stage
  static constexpr int STAGE = ROWS * 128;         // bytes
  static constexpr int CP = BN + 4;                // pitch (floats) of the epilogue tile
  static constexpr int EH = (size_t)BM * CP * 4 > 160 * 1024 ? 2 : 1;  // the epilogue goes through LDS in EH row chunks
  static constexpr int ER = BM / EH;               // rows per chunk
  static constexpr size_t LDS = (size_t)S * STAGE > (size_t)ER * CP * 4 ? (size_t)S * STAGE : (size_t)ER * CP * 4;
  static_assert(ROWS % (8 * NW) == 0, "the loader instructions must divide evenly over the waves");
  static_assert(BM % 16 == 0, "the swizzle of B's rows must not depend on BM");
  static_assert((NT * 4) % BN == 0 && ER % (NT * 4 / BN) == 0 && ER % 32 == 0, "epilogue passes");
};

// Workgroup -> (group, tile): the list of all tiles, ordered by group, then by the dimension with
// more tiles, is cut into 8 contiguous runs, one per XCD (workgroup i runs on XCD i % 8 and every
// XCD has its own L2).  An XCD then works on few groups at a time (with 8 groups of up to 32
// tiles: on one), whose operand panels are fetched into its L2 once and shared by its CUs; dealing
// the tiles of every group out to all XCDs made each L2 fetch the panels of all groups.
template <int BM, int BN>
__device__ __forceinline__ bool dlx_tile(const GemmNtDesc& d, unsigned bid, int& g, int& tile_m, int& tile_n) {
  const int tm = (d.M + BM - 1) / BM, tn = (d.N + BN - 1) / BN;
  const int per_group = tm * tn, total = per_group * d.groups;
  const int run = (total + 7) >> 3;
  const int li = bid >> 3;
  const int v = (bid & 7) * run + li;
  if (li >= run || v >= total) return false;
  g = v / per_group;
  const int r = v - g * per_group;
  if (tn >= tm) {
    tile_n = r / tm;
    tile_m = r - tile_n * tm;
  } else {
    tile_m = r / tn;
    tile_n = r - tile_m * tn;
  }
  return true;
}

// bid: the workgroup's index among those of this product (blockIdx.x, unless a launch holds two products)
template <bool COMMIT, int WGM, int WGN, int TM, int TN, int S>
__device__ __forceinline__ void dlx_body(const GemmNtDesc& d, unsigned bid) {
  using Sh = DlxShape<WGM, WGN, TM, TN, S>;
  constexpr int BM = Sh::BM, BN = Sh::BN, IPW = Sh::IPW, CP = Sh::CP, NT = Sh::NT;
  extern __shared__ __attribute__((aligned(16))) unsigned char nt_smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: LDS addresses of the loader stay scalar
  const int wm = wave % WGM, wn = wave / WGM;
  const int lrow = lane & 31, lk = lane >> 5;
  int g, tile_m, tile_n;
  if (!dlx_tile<BM, BN>(d, bid, g, tile_m, tile_n)) return;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const __bf16* __restrict__ A = reinterpret_cast<const __bf16*>(d.A) + (long)g * d.strideA;
  const __bf16* __restrict__ B = reinterpret_cast<const __bf16*>(d.B) + (long)g * d.strideB;
  // loader: instruction i of wave w covers stage rows (w IPW + i) 8 .. +7 (rows below BM are A's);
  // lane j: row + (j >> 3), LDS chunk j & 7, which holds the row's chunk (j & 7) ^ ((row >> 1) & 7)
  const __bf16* gp[IPW];
  int kofs[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int row = (wave * IPW + i) * 8 + (lane >> 3);
    kofs[i] = ((lane & 7) ^ ((row >> 1) & 7)) * 8;
    gp[i] = (row < BM ? A + (long)min(m0 + row, d.M - 1) * d.lda : B + (long)min(n0 + row - BM, d.N - 1) * d.ldb) + kofs[i];
  }
  const __bf16* zero = reinterpret_cast<const __bf16*>(nt_zero16);
  auto issue = [&](int stage, int kt) {
    unsigned char* sa = nt_smem + stage * Sh::STAGE + wave * IPW * 1024;
    if ((kt + 1) * NBK <= d.Kd) {  // (uniform) a whole tile: no per-lane checks
#pragma unroll
      for (int i = 0; i < IPW; ++i)
        __builtin_amdgcn_global_load_lds(HPSGD_GPTR(gp[i] + kt * NBK), HPSGD_LPTR(sa + i * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const bool ok = kt * NBK + kofs[i] < d.Kd;  // Kd is a multiple of 8: a chunk is all in or all out
        __builtin_amdgcn_global_load_lds(HPSGD_GPTR(ok ? gp[i] + kt * NBK : zero), HPSGD_LPTR(sa + i * 1024), 16, 0, 0);
      }
    }
  };
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // operand fragments: row r, chunk c = 2 ks + lk at byte r * 128 + ((c ^ ((r >> 1) & 7)) << 4)
  // (a wave's row blocks are 32 rows = 4096 bytes apart and share the swizzle: one address per
  // operand and step, the blocks by immediate offsets)
  unsigned oa[4], ob[4];
  {
    const int sw = (lrow >> 1) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      oa[ks] = (wm * TM * 32 + lrow) * 128 + (((2 * ks + lk) ^ sw) << 4);
      ob[ks] = (BM + wn * TN * 32 + lrow) * 128 + (((2 * ks + lk) ^ sw) << 4);
    }
  }
  const int nk = (d.Kd + NBK - 1) / NBK;
  // The fragment reads and the waits for them are written out (ds_read_b128 / s_waitcnt): the
  // compiler's own waits are for all outstanding LDS reads at once, which would make every step
  // wait for the reads issued for the next one.  LDS returns reads in order, so "all but the
  // newest TM + TN" is exactly the older step's set.
  bf16x8 fa[2][TM], fb[2][TN];
  const unsigned lds0 = (unsigned)(uintptr_t)HPSGD_LPTR(nt_smem);
  auto fragments = [&](unsigned sb, int ks, bf16x8(&fa_)[TM], bf16x8(&fb_)[TN]) {
    const unsigned aa = sb + oa[ks], ab = sb + ob[ks];
#pragma unroll
    for (int i = 0; i < TM; ++i) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fa_[i]) : "v"(aa), "n"(i * 4096));
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fb_[j]) : "v"(ab), "n"(j * 4096));
  };
  auto mfmas = [&](const bf16x8(&fa_)[TM], const bf16x8(&fb_)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i], fb_[j], acc[i][j], 0, 0, 0);
  };
  // Pipeline: the barrier that hands over tile kt+1 sits before the last quarter of tile kt's
  // MFMAs, and the first fragments of tile kt+1 are read between the two, so that the matrix
  // cores have work queued while the waves meet and while the first LDS reads are on their way.
#pragma unroll
  for (int st = 0; st < S - 1; ++st) issue(st, st);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * IPW) : "memory");
  __builtin_amdgcn_s_barrier();  // tile 0 is in LDS
  issue(S - 1, S - 1);
  fragments(lds0, 0, fa[0], fb[0]);
  int stage = 0;
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned sb = lds0 + stage * Sh::STAGE;
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      fragments(sb, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
      asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(TM + TN) : "memory");  // step ks has landed
      __builtin_amdgcn_sched_barrier(0);
      mfmas(fa[ks & 1], fb[ks & 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's reads of tile kt are complete, its loads of tile kt+1 have landed ...
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((S - 2) * IPW) : "memory");
    __builtin_amdgcn_s_barrier();  // ... and so are and have everyone's
    issue(stage, kt + S);          // into the buffer tile kt has left
    stage = stage + 1 == S ? 0 : stage + 1;
    fragments(lds0 + stage * Sh::STAGE, 0, fa[0], fb[0]);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(fa[1], fb[1]);
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the reads issued for the tile after the last
  // the zero loads of the tiles beyond the contraction must have landed before the operand
  // buffers become the epilogue tile
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // Epilogue through LDS, as in nt_epilogue: accumulators -> tile of ER rows x BN -> row segments
  float* C = d.C + (long)g * d.strideC;
  const float* bias = d.bias ? d.bias + (long)g * d.strideBias : nullptr;
  float* sC = reinterpret_cast<float*>(nt_smem);
  constexpr int ER = Sh::ER, TPR = BN / 4, RPP = NT / TPR, PASSES = ER / RPP;
  const int c4 = (tid % TPR) << 2, rbase = tid / TPR;
  const int col = n0 + c4;
  const bool vec = ((d.ldc | d.strideC) & 3) == 0 && ((uintptr_t)d.C & 15) == 0 &&
                   (!COMMIT || (((uintptr_t)d.win & 15) == 0 && (d.strideWin & 3) == 0));
#pragma unroll
  for (int h = 0; h < Sh::EH; ++h) {
    const int mh = m0 + h * ER;
    const bool fast = vec && col + 3 < d.N;
    // in-place update: the chunk's old values are requested before the accumulators go through
    // LDS, so that their latency runs under the staging and its barrier (requesting the next
    // chunk's as well, in front of this chunk's stores, needs two chunks' worth of registers and
    // gained 2 us per round more: not kept)
    float4 w[COMMIT ? PASSES : 1];
    if (COMMIT && fast) {
      const float* W = d.win + (long)g * d.strideWin;
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int row = min(mh + rbase + RPP * p, d.M - 1);  // clamped: not stored when outside
        w[COMMIT ? p : 0] = nt_load4(W + (long)row * d.ldc + col);
      }
    }
    if (h > 0) __syncthreads();  // the previous chunk has been read
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int rb = (wm * TM + i) * 32;  // the block's first row in the tile
      if (rb / ER != h) continue;         // uniform over the wave
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          sC[(rb % ER + 8 * (v / 4) + 4 * lk + (v % 4)) * CP + (wn * TN + j) * 32 + lrow] = acc[i][j][v];
    }
    __syncthreads();
    if (fast) {
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (!COMMIT && bias) bv = make_float4(bias[col], bias[col + 1], bias[col + 2], bias[col + 3]);
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int rl = rbase + RPP * p, row = mh + rl;
        if (row >= d.M) continue;
        const float4 a = *reinterpret_cast<const float4*>(&sC[rl * CP + c4]);
        float4 o;
        if (COMMIT) {
          const float4 wv = w[COMMIT ? p : 0];
          o = make_float4(wv.x - d.lr * a.x, wv.y - d.lr * a.y, wv.z - d.lr * a.z, wv.w - d.lr * a.w);
        } else {
          o = make_float4(a.x + bv.x, a.y + bv.y, a.z + bv.z, a.w + bv.w);
        }
        nt_store4(C + (long)row * d.ldc + col, o);
      }
    } else if (col < d.N) {
      const float* W = COMMIT ? d.win + (long)g * d.strideWin : nullptr;
      for (int p = 0; p < PASSES; ++p) {
        const int rl = rbase + RPP * p, row = mh + rl;
        if (row >= d.M) continue;
        for (int e = 0; e < 4; ++e) {
          if (col + e >= d.N) break;
          const long off = (long)row * d.ldc + col + e;
          const float a = sC[rl * CP + c4 + e];
          C[off] = COMMIT ? W[off] - d.lr * a : a + (bias ? bias[col + e] : 0.f);
        }
      }
    }
  }
}

template <bool COMMIT, int WGM, int WGN, int TM, int TN, int S>
__global__ void __launch_bounds__(64 * WGM * WGN)
gemm_bf16_dlx_kernel(GemmNtDesc d) {
  dlx_body<COMMIT, WGM, WGN, TM, TN, S>(d, blockIdx.x);
}

// Two independent products of the same form in one launch: the first blocks0 workgroups (a
// multiple of 8, so that a workgroup's XCD is the same as in a launch of its own) are d0's, the
// rest d1's.  For two products that would otherwise follow each other on one stream although
// neither needs the other: the second one's tiles fill the first one's last, partial round.
template <bool COMMIT, int WGM, int WGN, int TM, int TN, int S>
__global__ void __launch_bounds__(64 * WGM * WGN)
gemm_bf16_dlx_pair_kernel(GemmNtDesc d0, GemmNtDesc d1, unsigned blocks0) {
  const bool first = blockIdx.x < blocks0;  // (uniform)
  dlx_body<COMMIT, WGM, WGN, TM, TN, S>(first ? d0 : d1, first ? blockIdx.x : blockIdx.x - blocks0);
}

template <bool COMMIT, int WGM, int WGN, int TM, int TN, int S>
hipError_t launch_dlx(const GemmNtDesc& d, hipStream_t s) {
  using Sh = DlxShape<WGM, WGN, TM, TN, S>;
  static bool ready = false;
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_dlx_kernel<COMMIT, WGM, WGN, TM, TN, S>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)Sh::LDS);
    if (e != hipSuccess) return e;
    ready = true;
  }
  const int tm = (d.M + Sh::BM - 1) / Sh::BM, tn = (d.N + Sh::BN - 1) / Sh::BN;
  const int total = tm * tn * d.groups;
  const int kid = (TM == 2 ? KID_GEMM_BF16_DLX128 : TM == 3 ? KID_GEMM_BF16_DLX192 : KID_GEMM_BF16_DLX256) + (COMMIT ? 1 : 0);
  KernelTimer kt(kid, 2.0 * d.M * d.N * (double)d.Kd * d.groups, s);
  hipLaunchKernelGGL((gemm_bf16_dlx_kernel<COMMIT, WGM, WGN, TM, TN, S>), dim3(8 * ((total + 7) / 8)),
                     dim3(Sh::NT), Sh::LDS, s, d);
  return hipGetLastError();
}

static bool pair_desc(const GemmBf16Args& a, GemmNtDesc& d) {
  if (a.M <= 0 || a.N <= 0 || a.groups <= 0 || !a.win || !a.C) return false;
  if (!gemm_bf16_nt_supported(a.A, 1, a.lda, a.sA, a.Kd) || !gemm_bf16_nt_supported(a.B, 1, a.ldb, a.sB, a.Kd)) return false;
  d.A = a.A; d.lda = a.lda; d.strideA = a.sA;
  d.B = a.B; d.ldb = a.ldb; d.strideB = a.sB;
  d.C = a.C; d.ldc = a.ldc; d.strideC = a.sC;
  d.bias = nullptr; d.strideBias = 0;
  d.win = a.win; d.strideWin = a.sWin; d.lr = a.lr;
  d.M = a.M; d.N = a.N; d.Kd = a.Kd; d.groups = a.groups;
  return true;
}

bool gemm_bf16_update_pair_supported(const GemmBf16Args& p0, const GemmBf16Args& p1) {
  GemmNtDesc d;
  return pair_desc(p0, d) && pair_desc(p1, d);
}

hipError_t launch_gemm_bf16_update_pair(const GemmBf16Args& p0, const GemmBf16Args& p1, hipStream_t s) {
  GemmNtDesc d0, d1;
  if (!pair_desc(p0, d0) || !pair_desc(p1, d1)) return hipErrorInvalidValue;
  using Sh = DlxShape<2, 4, 3, 2, 2>;
  static bool ready = false;
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_dlx_pair_kernel<true, 2, 4, 3, 2, 2>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)Sh::LDS);
    if (e != hipSuccess) return e;
    ready = true;
  }
  auto blocks = [](const GemmNtDesc& d) {
    const long total = (long)((d.M + Sh::BM - 1) / Sh::BM) * ((d.N + Sh::BN - 1) / Sh::BN) * d.groups;
    return (unsigned)(8 * ((total + 7) / 8));
  };
  const unsigned b0 = blocks(d0), b1 = blocks(d1);
  KernelTimer kt(KID_GEMM_BF16_DLX192_COMMIT,
                 2.0 * d0.M * d0.N * (double)d0.Kd * d0.groups + 2.0 * d1.M * d1.N * (double)d1.Kd * d1.groups, s);
  hipLaunchKernelGGL((gemm_bf16_dlx_pair_kernel<true, 2, 4, 3, 2, 2>), dim3(b0 + b1), dim3(Sh::NT), Sh::LDS, s, d0, d1, b0);
  return hipGetLastError();
}

// form: 0 picks the kernel; for two bf16 operands 1 .. 4 force the 128 x 128, 128 x 256, 192 x 256
// or 256 x 256 tile (every form computes every element with the same sequence of MFMAs: the
// results do not depend on it).
// a_bf16 / b_bf16: the operand is stored as bf16 (else fp32).  Leading dimensions and group
// strides are in elements of the operand's own type.  Requires 16-byte aligned bases, row
// pitches and group strides that are multiples of 16 bytes, and Kd a multiple of 8
// (gemm_bf16_nt_supported); returns hipErrorInvalidValue otherwise.
bool gemm_bf16_nt_supported(const void* p, int is_bf16, long ld, long stride, int Kd) {
  const long q = is_bf16 ? 8 : 4;
  return ((uintptr_t)p & 15) == 0 && ld % q == 0 && stride % q == 0 && Kd % 8 == 0 && Kd >= 8;
}

hipError_t launch_gemm_bf16_nt(const void* A, int a_bf16, long lda, long sA, const void* B, int b_bf16,
                               long ldb, long sB, float* C, long ldc, long sC, const float* bias,
                               long sBias, const float* win, long sWin, float lr, int M, int N, int Kd,
                               int groups, hipStream_t s, int form) {
  if (M <= 0 || N <= 0 || groups <= 0) return hipSuccess;
  if (form < 0 || form > 4 || (form > 1 && !(a_bf16 && b_bf16))) return hipErrorInvalidValue;
  GemmNtDesc d;
  d.A = A; d.lda = lda; d.strideA = sA;
  d.B = B; d.ldb = ldb; d.strideB = sB;
  d.C = C; d.ldc = ldc; d.strideC = sC;
  d.bias = bias; d.strideBias = sBias;
  d.win = win; d.strideWin = sWin; d.lr = lr;
  d.M = M; d.N = N; d.Kd = Kd; d.groups = groups;
  if (!gemm_bf16_nt_supported(A, a_bf16, lda, sA, Kd) || !gemm_bf16_nt_supported(B, b_bf16, ldb, sB, Kd))
    return hipErrorInvalidValue;
  const int tm = (M + NBM - 1) / NBM, tn = (N + NBN - 1) / NBN;
  const int ts = tn >= tm ? tn : tm, tf = tn >= tm ? tm : tn;
  dim3 grid(8 * ((ts + 7) / 8) * tf * groups);  // see the tile order in the kernel
  dim3 block(NTHREADS);
  constexpr size_t smem = (size_t)2 * (NBM + NBN) * NPITCH * sizeof(__bf16);  // 72 KB: above the static limit
  const double flops = 2.0 * M * N * (double)Kd * groups;
#define HPSGD_NT1(TA, TB, CM)                                                                     \
  do {                                                                                            \
    static bool ready = false; /* per instantiation: allow the large dynamic LDS allocation */    \
    if (!ready) {                                                                                 \
      hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_nt_kernel<TA, TB, CM>,            \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);  \
      if (e != hipSuccess) return e;                                                              \
      ready = true;                                                                               \
    }                                                                                             \
    KernelTimer kt(KID_GEMM_BF16_NT, flops, s);                                                   \
    hipLaunchKernelGGL((gemm_bf16_nt_kernel<TA, TB, CM>), grid, block, smem, s, d);               \
  } while (0)
#define HPSGD_NT(TA, TB)                \
  do {                                  \
    if (win) HPSGD_NT1(TA, TB, true);   \
    else HPSGD_NT1(TA, TB, false);      \
  } while (0)
  if (a_bf16 && b_bf16) {
    constexpr size_t dl_smem = (size_t)NBM * (NBN + 4) * sizeof(float);  // the epilogue tile; operands need 64 KB
#define HPSGD_DL(CM)                                                                              \
  do {                                                                                            \
    static bool ready = false;                                                                    \
    if (!ready) {                                                                                 \
      hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_dl_kernel<CM>,                    \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)dl_smem); \
      if (e != hipSuccess) return e;                                                              \
      ready = true;                                                                               \
    }                                                                                             \
    KernelTimer kt(CM ? KID_GEMM_BF16_DL_COMMIT : KID_GEMM_BF16_DL, flops, s);                    \
    hipLaunchKernelGGL((gemm_bf16_dl_kernel<CM>), grid, block, dl_smem, s, d);                    \
  } while (0)
    // Which tile.  One 8-wave workgroup per CU with a tile 256 wide does more matrix work per
    // byte through LDS and per byte fetched, but nothing overlaps its first loads and its
    // epilogue, which cost as much as about 8 k-tiles (12 with the in-place update); two
    // independent 128 x 128 workgroups per CU cover each other's but need 1.3 times as long
    // per k-tile.  The estimate below (rounds of 256 CUs x rows of the tile x k-tiles incl. the
    // fixed part) reproduces the measured order of the forms on the shapes of the GRU language
    // model, e.g. head dX (1120 x 1024 x 10000, 8 groups): 192 rows 314 us, 256 rows 312, 128 x 128
    // 507; recurrent weight gradient (3072 x 1024 x 1120, in place): 91 / 107 / 104; first
    // layer's input projection (1120 x 3072 x 256): 46 / 42 / 36.
    if (form == 0) {
      const double nk = (Kd + NBK - 1) / NBK;
      const double fixed = win ? 12.0 : 8.0;
      auto rounds = [&](int bm, int bn, int slots) {
        const long t = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * groups;
        return (double)((t + slots - 1) / slots);
      };
      double best = rounds(128, 128, 512) * 128 * (1.3 * nk + (win ? 8.0 : 6.0));
      form = 1;
      const double c128 = rounds(128, 256, 256) * 128 * 1.12 * (nk + fixed);
      const double c192 = rounds(192, 256, 256) * 192 * (nk + fixed);
      const double c256 = rounds(256, 256, 256) * 256 * (nk + fixed);
      if (c128 < best) { best = c128; form = 2; }
      if (c192 < best) { best = c192; form = 3; }
      if (c256 < best) { best = c256; form = 4; }
    }
    if (form == 2) return win ? launch_dlx<true, 2, 4, 2, 2, 3>(d, s) : launch_dlx<false, 2, 4, 2, 2, 3>(d, s);
    if (form == 3) return win ? launch_dlx<true, 2, 4, 3, 2, 2>(d, s) : launch_dlx<false, 2, 4, 3, 2, 2>(d, s);
    if (form == 4) return win ? launch_dlx<true, 2, 4, 4, 2, 2>(d, s) : launch_dlx<false, 2, 4, 4, 2, 2>(d, s);
    if (win) HPSGD_DL(true);
    else HPSGD_DL(false);
#undef HPSGD_DL
  } else if (a_bf16) HPSGD_NT(__bf16, float);
  else if (b_bf16) HPSGD_NT(float, __bf16);
  else HPSGD_NT(float, float);
#undef HPSGD_NT
#undef HPSGD_NT1
  return hipGetLastError();
}

}  // namespace hpsgd
