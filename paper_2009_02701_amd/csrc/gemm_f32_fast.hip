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

// COMMIT: the epilogue is C = W - alpha * acc (EPI_COMMIT); the tile of W is requested before
// the contraction starts, so that the epilogue does not wait for it.
template <int BM, int BN, bool TA, bool TB, bool COMMIT>
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
  const int g = blockIdx.z;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  OpA a;
  OpB b;
  a.init(d.A + (long)g * d.strideA, d.lda, m0, d.M, tid);
  b.init(d.B + (long)g * d.strideB, d.ldb, n0, d.N, tid);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  floatx16 wv[COMMIT ? TM : 1][COMMIT ? TN : 1];
  if (COMMIT) {
    const float* W = d.aux + (long)g * d.strideAux;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * (BN / 2) + j * 32 + lrow;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * (BM / 2) + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
          wv[COMMIT ? i : 0][COMMIT ? j : 0][v] =
              W[(long)min(row, d.M - 1) * d.ldc + min(col, d.N - 1)];  // clamped: never stored when outside
        }
    }
  }

  auto compute = [&](int buf) {
#pragma unroll
    for (int c = 0; c < FBK / 8; ++c) {
      float4 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = OpA::frag(sA[buf], wm * (BM / 2) + i * 32 + lrow, c, lk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = OpB::frag(sB[buf], wn * (BN / 2) + j * 32 + lrow, c, lk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].x, fb[j].x, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].y, fb[j].y, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].z, fb[j].z, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].w, fb[j].w, acc[i][j], 0, 0, 0);
        }
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

  float* C = d.C + (long)g * d.strideC;
  const float* aux = d.aux ? d.aux + (long)g * d.strideAux : nullptr;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * (BN / 2) + j * 32 + lrow;
    if (col >= d.N) continue;
    float bias = 0.f;
    if (d.epilogue == EPI_BIAS || d.epilogue == EPI_BIAS_RELU) bias = aux[col];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * (BM / 2) + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
        if (row >= d.M) continue;
        const long off = (long)row * d.ldc + col;
        float val = acc[i][j][v];
        if (COMMIT) {
          val = wv[COMMIT ? i : 0][COMMIT ? j : 0][v] - d.alpha * val;
        } else {
          switch (d.epilogue) {
            case EPI_BIAS: val += bias; break;
            case EPI_BIAS_RELU: val = fmaxf(val + bias, 0.f); break;
            case EPI_ACCUM: val += C[off]; break;
            case EPI_RELU_MASK: val = aux[off] > 0.f ? val : 0.f; break;
            default: break;
          }
        }
        C[off] = val;
      }
    }
  }
}

template <int BM, int BN, bool TA, bool TB, bool COMMIT>
static hipError_t launch_fast_cfg(const GemmDesc& d, hipStream_t s) {
  using OpA = FastOperand<BM, !TA>;
  using OpB = FastOperand<BN, TB>;
  constexpr size_t smem = (size_t)2 * (OpA::LDS_FLOATS + OpB::LDS_FLOATS) * sizeof(float);
  static bool ready = false;  // per instantiation: allow dynamic LDS above 64 KB
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_f32_fast_kernel<BM, BN, TA, TB, COMMIT>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    ready = true;
  }
  dim3 grid((d.N + BN - 1) / BN, (d.M + BM - 1) / BM, d.groups);
  hipLaunchKernelGGL((gemm_f32_fast_kernel<BM, BN, TA, TB, COMMIT>), grid, dim3(FTHREADS), smem, s, d);
  return hipGetLastError();
}

template <int BM, int BN, bool COMMIT>
static hipError_t launch_fast_layout2(const GemmDesc& d, hipStream_t s) {
  if (!d.transA && d.transB) return launch_fast_cfg<BM, BN, false, true, COMMIT>(d, s);
  if (!d.transA && !d.transB) return launch_fast_cfg<BM, BN, false, false, COMMIT>(d, s);
  if (d.transA && !d.transB) return launch_fast_cfg<BM, BN, true, false, COMMIT>(d, s);
  return launch_fast_cfg<BM, BN, true, true, COMMIT>(d, s);
}

template <int BM, int BN>
static hipError_t launch_fast_layout(const GemmDesc& d, hipStream_t s) {
  return d.epilogue == EPI_COMMIT ? launch_fast_layout2<BM, BN, true>(d, s)
                                  : launch_fast_layout2<BM, BN, false>(d, s);
}

// Returns hipErrorNotSupported (nothing launched) when an operand does not allow 16-byte loads
// or a dimension is below one vector; the caller then takes the generic kernel.
hipError_t launch_gemm_f32_fast(const GemmDesc& d, hipStream_t s) {
  auto aligned = [](const float* p, long ld, long stride) {
    return ((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (stride & 3) == 0;
  };
  if (!aligned(d.A, d.lda, d.strideA) || !aligned(d.B, d.ldb, d.strideB)) return hipErrorNotSupported;
  // unit-stride-along-k operands load float4 along k; the others along m / n
  if (!d.transA ? (d.Kd & 3) != 0 : ((d.M & 3) != 0 || d.M < 4)) return hipErrorNotSupported;
  if (d.transB ? (d.Kd & 3) != 0 : ((d.N & 3) != 0 || d.N < 4)) return hipErrorNotSupported;
  if (d.Kd < 4) return hipErrorNotSupported;
  auto tiles = [&](int bm, int bn) {
    return (long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.groups;
  };
  if (d.M > 64 && d.N > 64 && tiles(128, 128) >= 192) return launch_fast_layout<128, 128>(d, s);
  return launch_fast_layout<64, 64>(d, s);
}

}  // namespace hpsgd
