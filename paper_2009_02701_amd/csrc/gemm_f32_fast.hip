// Grouped fp32 GEMM on the fp32 matrix cores, fast path for 16-byte aligned operands.
//
//   C[g] (M x N) = op(A[g]) (M x Kd) * op(B[g]) (Kd x N)      (same contract as gemm_f32.hip)
//
// Differences from the generic kernel: k-tiles of 32 with two LDS buffers and one barrier per
// k-tile, two register prefetch stages, and a main loop without branches (rows and columns
// are clamped into the matrix, which only changes values that feed outputs never stored; the
// contraction tail is zeroed by a select when a tile is written to LDS).  Operand tiles keep
// their natural layout in LDS, so no store is transposing:
//   * an operand that is unit-stride along k is stored [i][k]; an MFMA lane then reads a
//     float4 = 4 consecutive k of its row and feeds component s to MFMA number s (the order of
//     the contraction index is free as long as both operands agree): lane half lk covers
//     k = 8c + 4*lk + s;
//   * an operand that is unit-stride along i is stored [k][i] and read one float per MFMA at
//     the same k = 8c + 4*lk + s.
// v_mfma_f32_32x32x2_f32 lane layout: A lane l holds A[m = l%32][k = l/32], B lane l holds
// B[k = l/32][n = l%32], accumulator register v holds C[8*(v/4) + 4*(l/32) + v%4][l%32].
#include "kernels.h"

namespace hpsgd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

static constexpr int FBK = 32;
static constexpr int FTHREADS = 256;

// One operand tile: BI rows/columns x FBK.  CK: unit-stride along k in memory.
template <int BI, bool CK>
struct FastOperand {
  static constexpr int PITCH = CK ? FBK + 4 : BI + 4;          // floats
  static constexpr int LDS_FLOATS = CK ? BI * PITCH : FBK * PITCH;
  static constexpr int UPT = BI * FBK / 4 / FTHREADS;          // float4 units per thread
  const float* ptr[UPT];   // each unit's row (CK) or column (not CK) base, clamped into the matrix
  float4 r[2][UPT];

  __device__ __forceinline__ void init(const float* __restrict__ base, long ld, int i0, int imax, int tid) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * FTHREADS;
      if (CK) {
        ptr[u] = base + (long)min(i0 + (unit >> 3), imax - 1) * ld;
      } else {
        ptr[u] = base + min(i0 + ((unit % (BI / 4)) << 2), imax - 4);
      }
    }
  }
  // k index of unit u inside a k-tile
  __device__ __forceinline__ static int kofs(int u, int tid) {
    const int unit = tid + u * FTHREADS;
    return CK ? ((unit & 7) << 2) : unit / (BI / 4);
  }
  __device__ __forceinline__ void load(int st, int kt, int Kd, long ld, int tid) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      // a unit past the end of the contraction re-reads k = 0 (always in bounds) and is zeroed
      // when it is stored
      const int k = kt * FBK + kofs(u, tid);
      const int kc = k < Kd ? k : 0;
      r[st][u] = *reinterpret_cast<const float4*>(ptr[u] + (CK ? (long)kc : (long)kc * ld));
    }
  }
  __device__ __forceinline__ void store(int st, int kt, int Kd, float* __restrict__ lds, int tid) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * FTHREADS;
      const bool in = kt * FBK + kofs(u, tid) < Kd;  // Kd % 4 == 0 for CK: a float4 is all in or out
      const float4 v = in ? r[st][u] : make_float4(0.f, 0.f, 0.f, 0.f);
      if (CK)
        *reinterpret_cast<float4*>(&lds[(unit >> 3) * PITCH + ((unit & 7) << 2)]) = v;
      else
        *reinterpret_cast<float4*>(&lds[(unit / (BI / 4)) * PITCH + ((unit % (BI / 4)) << 2)]) = v;
    }
  }
  // the 4 values k = 8c + 4*lk + {0..3} of row/column `i` of the tile
  __device__ __forceinline__ static float4 frag(const float* __restrict__ lds, int i, int c, int lk) {
    if (CK) return *reinterpret_cast<const float4*>(&lds[i * PITCH + 8 * c + 4 * lk]);
    const float* p = &lds[(8 * c + 4 * lk) * PITCH + i];
    return make_float4(p[0], p[PITCH], p[2 * PITCH], p[3 * PITCH]);
  }
};

template <int BM, int BN, bool TA, bool TB>
__global__ void __launch_bounds__(FTHREADS)
gemm_f32_fast_kernel(GemmDesc d) {
  using OpA = FastOperand<BM, !TA>;   // A is unit-stride along k when stored [M][Kd]
  using OpB = FastOperand<BN, TB>;    // B is unit-stride along k when stored [N][Kd]
  constexpr int TM = BM / 64, TN = BN / 64;  // 2 x 2 waves, each (BM/2) x (BN/2) in 32 x 32 blocks
  extern __shared__ __attribute__((aligned(16))) float fast_lds[];
  float* sA[2] = {fast_lds, fast_lds + OpA::LDS_FLOATS};
  float* sB[2] = {fast_lds + 2 * OpA::LDS_FLOATS, fast_lds + 2 * OpA::LDS_FLOATS + OpB::LDS_FLOATS};

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int lrow = lane & 31, lk = lane >> 5;
  // Tile order.  Workgroup i runs on XCD i % 8 and every XCD has its own L2: the tiles, in
  // (group, row tile, column tile) order, are cut into 8 contiguous runs, one per XCD, so that
  // an XCD fetches the A rows of its run once and only the B operands of the groups it touches.
  const int tn = (d.N + BN - 1) / BN, tm = (d.M + BM - 1) / BM;
  const int splits = d.splits > 1 ? d.splits : 1;
  const long ntiles = (long)tn * tm * d.groups * splits, per = (ntiles + 7) / 8;
  const long tile = (long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((long)(blockIdx.x >> 3) >= per || tile >= ntiles) return;  // padding of the last run
  const int gp = (int)(tile / ((long)tn * tm));   // group * splits + part of the contraction
  const int g = gp / splits, part = gp - g * splits;
  const int m0 = (int)((tile / tn) % tm) * BM, n0 = (int)(tile % tn) * BN;

  OpA a;
  OpB b;
  // a part of a split contraction starts part * Kd further along k
  const long ka = (long)part * d.Kd * (TA ? d.lda : 1), kb = (long)part * d.Kd * (TB ? 1 : d.ldb);
  a.init(d.A + (long)g * d.strideA + ka, d.lda, m0, d.M, tid);
  b.init(d.B + (long)g * d.strideB + kb, d.ldb, n0, d.N, tid);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  auto compute = [&](int buf) {
#pragma unroll
    for (int c = 0; c < FBK / 8; ++c) {
      float4 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = OpA::frag(sA[buf], wm * (BM / 2) + i * 32 + lrow, c, lk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = OpB::frag(sB[buf], wn * (BN / 2) + j * 32 + lrow, c, lk);
      // contraction steps outermost: consecutive MFMAs update different accumulator tiles
      // (a dependent MFMA waits for the previous one to leave the pipeline)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].x, fb[j].x, acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].y, fb[j].y, acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].z, fb[j].z, acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].w, fb[j].w, acc[i][j], 0, 0, 0);
    }
  };

  const int nk = (d.Kd + FBK - 1) / FBK;
  a.load(0, 0, d.Kd, d.lda, tid);
  b.load(0, 0, d.Kd, d.ldb, tid);
  a.store(0, 0, d.Kd, sA[0], tid);
  b.store(0, 0, d.Kd, sB[0], tid);
  a.load(0, 1, d.Kd, d.lda, tid);
  b.load(0, 1, d.Kd, d.ldb, tid);
  a.load(1, 2, d.Kd, d.lda, tid);
  b.load(1, 2, d.Kd, d.ldb, tid);
  // The epilogue's extra matrix operand in C's layout (the old C, the ReLU mask or the weights
  // to update) is requested here, behind the first operand tiles: it arrives during the
  // contraction instead of holding up the epilogue (a weight gradient over one batch is a few
  // k-tiles of matrix work and as many bytes of weights to update as of operands).
  float* C = d.C + (long)(splits > 1 ? gp : g) * d.strideC;
  const float* aux = d.aux ? d.aux + (long)g * d.strideAux : nullptr;
  constexpr int CP = BN + 4;                       // pitch in floats
  constexpr int RPP = FTHREADS / (BN / 4);         // rows per pass
  constexpr int PASSES = BM / RPP;
  const int c4 = (tid % (BN / 4)) << 2, rbase = tid / (BN / 4);
  const int col = n0 + c4;
  const int epi = d.epilogue;
  const float* X = epi == EPI_ACCUM ? C : (epi == EPI_RELU_MASK || epi == EPI_COMMIT) ? aux : nullptr;
  const long xs = epi == EPI_ACCUM ? d.strideC : d.strideAux;
  const bool vec = ((d.ldc | d.strideC) & 3) == 0 && ((uintptr_t)d.C & 15) == 0 &&
                   (!X || (((uintptr_t)(epi == EPI_ACCUM ? d.C : d.aux) & 15) == 0 && (xs & 3) == 0));
  float4 x[PASSES];
  if (X && vec && col + 3 < d.N) {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int row = min(m0 + rbase + RPP * p, d.M - 1);  // clamped: not stored when outside
      x[p] = *reinterpret_cast<const float4*>(X + (long)row * d.ldc + col);
    }
  }
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    compute(0);                                   // tile kt
    a.store(0, kt + 1, d.Kd, sA[1], tid);         // tile kt+1 -> buffer 1
    b.store(0, kt + 1, d.Kd, sB[1], tid);
    a.load(0, kt + 3, d.Kd, d.lda, tid);
    b.load(0, kt + 3, d.Kd, d.ldb, tid);
    __syncthreads();
    compute(1);                                   // tile kt+1 (all zeros past the end)
    a.store(1, kt + 2, d.Kd, sA[0], tid);         // tile kt+2 -> buffer 0
    b.store(1, kt + 2, d.Kd, sB[0], tid);
    a.load(1, kt + 4, d.Kd, d.lda, tid);
    b.load(1, kt + 4, d.Kd, d.ldb, tid);
    __syncthreads();
  }

  // Epilogue through LDS (the operand buffers are free after the last barrier): the
  // accumulators are laid out as the BM x BN tile, then every thread moves 16-byte pieces of
  // whole rows, so the stores and the loads of the extra operand (the old C, the ReLU mask or
  // the weights to update; all requested before the first is used) are fully coalesced.
  float* sC = fast_lds;
  static_assert((size_t)BM * CP <= 2 * (OpA::LDS_FLOATS + OpB::LDS_FLOATS), "epilogue tile fits the operand buffers");
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        sC[(wm * (BM / 2) + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4)) * CP + wn * (BN / 2) + j * 32 + lrow] =
            acc[i][j][v];
  __syncthreads();
  if (vec && col + 3 < d.N) {
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (epi == EPI_BIAS || epi == EPI_BIAS_RELU) bv = make_float4(aux[col], aux[col + 1], aux[col + 2], aux[col + 3]);
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int rl = rbase + RPP * p, row = m0 + rl;
      if (row >= d.M) continue;
      const float4 a = *reinterpret_cast<const float4*>(&sC[rl * CP + c4]);
      float4 o = a;
      switch (epi) {
        case EPI_BIAS: o = make_float4(a.x + bv.x, a.y + bv.y, a.z + bv.z, a.w + bv.w); break;
        case EPI_BIAS_RELU:
          o = make_float4(fmaxf(a.x + bv.x, 0.f), fmaxf(a.y + bv.y, 0.f), fmaxf(a.z + bv.z, 0.f),
                          fmaxf(a.w + bv.w, 0.f));
          break;
        case EPI_ACCUM: o = make_float4(a.x + x[p].x, a.y + x[p].y, a.z + x[p].z, a.w + x[p].w); break;
        case EPI_RELU_MASK:
          o = make_float4(x[p].x > 0.f ? a.x : 0.f, x[p].y > 0.f ? a.y : 0.f, x[p].z > 0.f ? a.z : 0.f,
                          x[p].w > 0.f ? a.w : 0.f);
          break;
        case EPI_COMMIT:
          o = make_float4(x[p].x - d.alpha * a.x, x[p].y - d.alpha * a.y, x[p].z - d.alpha * a.z,
                          x[p].w - d.alpha * a.w);
          break;
        default: break;
      }
      *reinterpret_cast<float4*>(C + (long)row * d.ldc + col) = o;
    }
  } else {
    for (int p = 0; p < PASSES; ++p) {
      const int rl = rbase + RPP * p, row = m0 + rl;
      if (row >= d.M) continue;
      for (int e = 0; e < 4; ++e) {
        if (col + e >= d.N) break;
        const long off = (long)row * d.ldc + col + e;
        float val = sC[rl * CP + c4 + e];
        switch (epi) {
          case EPI_BIAS: val += aux[col + e]; break;
          case EPI_BIAS_RELU: val = fmaxf(val + aux[col + e], 0.f); break;
          case EPI_ACCUM: val += C[off]; break;
          case EPI_RELU_MASK: val = aux[off] > 0.f ? val : 0.f; break;
          case EPI_COMMIT: val = aux[off] - d.alpha * val; break;
          default: break;
        }
        C[off] = val;
      }
    }
  }
}

template <int BM, int BN, bool TA, bool TB>
static hipError_t launch_fast_cfg(const GemmDesc& d, hipStream_t s) {
  using OpA = FastOperand<BM, !TA>;
  using OpB = FastOperand<BN, TB>;
  constexpr size_t smem = (size_t)2 * (OpA::LDS_FLOATS + OpB::LDS_FLOATS) * sizeof(float);
  static bool ready = false;  // per instantiation: allow dynamic LDS above 64 KB
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_f32_fast_kernel<BM, BN, TA, TB>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    ready = true;
  }
  const long ntiles = (long)((d.N + BN - 1) / BN) * ((d.M + BM - 1) / BM) * d.groups * (d.splits > 1 ? d.splits : 1);
  dim3 grid((unsigned)(8 * ((ntiles + 7) / 8)));
  KernelTimer kt(KID_GEMM_F32_FAST, 2.0 * d.M * d.N * (double)d.Kd * d.groups * (d.splits > 1 ? d.splits : 1), s);
  hipLaunchKernelGGL((gemm_f32_fast_kernel<BM, BN, TA, TB>), grid, dim3(FTHREADS), smem, s, d);
  return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_fast_layout(const GemmDesc& d, hipStream_t s) {
  if (!d.transA && d.transB) return launch_fast_cfg<BM, BN, false, true>(d, s);
  if (!d.transA && !d.transB) return launch_fast_cfg<BM, BN, false, false>(d, s);
  if (d.transA && !d.transB) return launch_fast_cfg<BM, BN, true, false>(d, s);
  return launch_fast_cfg<BM, BN, true, true>(d, s);
}

// Returns hipErrorNotSupported (nothing launched) when an operand does not allow 16-byte loads
// or a dimension is below one vector; the caller then takes the generic kernel.
hipError_t launch_gemm_f32_fast(const GemmDesc& d, hipStream_t s) {
  auto aligned = [](const float* p, long ld, long stride) {
    return ((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (stride & 3) == 0;
  };
  if (d.splits > 1 && (d.epilogue != EPI_STORE || (d.Kd & 3) != 0)) return hipErrorInvalidValue;
  if (!aligned(d.A, d.lda, d.strideA) || !aligned(d.B, d.ldb, d.strideB)) return hipErrorNotSupported;
  // unit-stride-along-k operands load float4 along k; the others along m / n
  if (!d.transA ? (d.Kd & 3) != 0 : ((d.M & 3) != 0 || d.M < 4)) return hipErrorNotSupported;
  if (d.transB ? (d.Kd & 3) != 0 : ((d.N & 3) != 0 || d.N < 4)) return hipErrorNotSupported;
  if (d.Kd < 4) return hipErrorNotSupported;
  auto tiles = [&](int bm, int bn) {
    return (long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.groups;
  };
  // 128 x 128 tiles from two full rounds of workgroups on: below that the smaller tiles' better
  // balance over the CUs outweighs their extra LDS traffic (the fp32 matrix rate is low enough).
  // A contraction of a few k-tiles (a weight gradient over one batch) is mostly first loads and
  // epilogue: four small workgroups per SIMD cover those better than two large ones (matrix
  // pipes busy 52 % of the time with the large tile at Kd = 128)
  if (d.M > 64 && d.N > 64 && tiles(128, 128) >= 512 && d.Kd > 256) return launch_fast_layout<128, 128>(d, s);
  return launch_fast_layout<64, 64>(d, s);
}

}  // namespace hpsgd
