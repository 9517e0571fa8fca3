// Grouped GEMM with bf16 operands and fp32 accumulation on the CDNA4 matrix cores
// (v_mfma_f32_32x32x16_bf16).  Operands live in HBM as fp32 (master parameters, fp32
// activations and gradients); they are rounded to bf16 (nearest-even) on their way into LDS,
// so no bf16 copy of anything is kept in memory.
//
// LDS tiles are [i][k] with k contiguous (BK = 32 plus 8 halves of padding: an 80-byte row
// pitch makes the 16-byte operand reads of 16 consecutive rows hit distinct banks).
// MFMA 32x32x16 lane layout: A operand lane l holds A[m = l%32][k = 8*(l/32) .. +7], B operand
// lane l holds B[k = 8*(l/32) .. +7][n = l%32]; accumulator register v of lane l holds
// C[8*(v/4) + 4*(l/32) + v%4][l%32].
#include "kernels.h"

namespace hpsgd {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

static constexpr int BKB = 32;
static constexpr int PITCH = BKB + 8;  // in bf16 elements

__device__ __forceinline__ float4 ldg4(const float* __restrict__ p, int c, int cmax, bool vec) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (vec && c + 3 < cmax) {
    v = *reinterpret_cast<const float4*>(p);
  } else {
    if (c + 0 < cmax) v.x = p[0];
    if (c + 1 < cmax) v.y = p[1];
    if (c + 2 < cmax) v.z = p[2];
    if (c + 3 < cmax) v.w = p[3];
  }
  return v;
}

// Stages one operand tile (BI rows x BKB) through registers into LDS as bf16.
template <int BI, int NT, bool CONTIG_K>
struct TileLoaderBf16 {
  // CONTIG_K: unit = 8 consecutive k of one row; else unit = 4 consecutive rows at one k
  static constexpr int UNITS = CONTIG_K ? BI * (BKB / 8) : BKB * (BI / 4);
  static constexpr int U = (UNITS + NT - 1) / NT;
  float4 r[U][CONTIG_K ? 2 : 1];

  __device__ __forceinline__ void load(const float* __restrict__ base, long ld, int i0, int k0,
                                       int imax, int kmax, bool vec, int tid) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = tid + u * NT;
      if (UNITS % NT != 0 && unit >= UNITS) break;
      if (CONTIG_K) {
        const int i = i0 + unit / (BKB / 8);
        const int k = k0 + (unit % (BKB / 8)) * 8;
        if (i < imax) {
          const float* p = base + (long)i * ld + k;
          r[u][0] = ldg4(p, k, kmax, vec);
          r[u][1] = ldg4(p + 4, k + 4, kmax, vec);
        } else {
          r[u][0] = make_float4(0.f, 0.f, 0.f, 0.f);
          r[u][1] = r[u][0];
        }
      } else {
        const int k = k0 + unit / (BI / 4);
        const int i = i0 + (unit % (BI / 4)) * 4;
        if (k < kmax)
          r[u][0] = ldg4(base + (long)k * ld + i, i, imax, vec);
        else
          r[u][0] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  }

  __device__ __forceinline__ void store(__bf16* __restrict__ lds, int tid) const {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = tid + u * NT;
      if (UNITS % NT != 0 && unit >= UNITS) break;
      if (CONTIG_K) {
        const int i = unit / (BKB / 8);
        const int k = (unit % (BKB / 8)) * 8;
        bf16x8 v;
        v[0] = (__bf16)r[u][0].x; v[1] = (__bf16)r[u][0].y; v[2] = (__bf16)r[u][0].z; v[3] = (__bf16)r[u][0].w;
        v[4] = (__bf16)r[u][1].x; v[5] = (__bf16)r[u][1].y; v[6] = (__bf16)r[u][1].z; v[7] = (__bf16)r[u][1].w;
        *reinterpret_cast<bf16x8*>(&lds[i * PITCH + k]) = v;
      } else {
        const int k = unit / (BI / 4);
        const int i = (unit % (BI / 4)) * 4;
        lds[(i + 0) * PITCH + k] = (__bf16)r[u][0].x;
        lds[(i + 1) * PITCH + k] = (__bf16)r[u][0].y;
        lds[(i + 2) * PITCH + k] = (__bf16)r[u][0].z;
        lds[(i + 3) * PITCH + k] = (__bf16)r[u][0].w;
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_bf16_kernel(GemmDesc d, int vecA, int vecB) {
  constexpr int WAVES_M = BM / WM;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  __shared__ __attribute__((aligned(16))) __bf16 sA[BM * PITCH];
  __shared__ __attribute__((aligned(16))) __bf16 sB[BN * PITCH];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WAVES_M;
  const int wn = wave / WAVES_M;
  const int g = blockIdx.z;
  const int m0 = blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;

  const float* __restrict__ A = d.A + (long)g * d.strideA;
  const float* __restrict__ B = d.B + (long)g * d.strideB;
  float* C = d.C + (long)g * d.strideC;

  TileLoaderBf16<BM, NT, !TA> la;
  TileLoaderBf16<BN, NT, TB> lb;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (d.Kd + BKB - 1) / BKB;
  la.load(A, d.lda, m0, 0, d.M, d.Kd, vecA, tid);
  lb.load(B, d.ldb, n0, 0, d.N, d.Kd, vecB, tid);

  const int lrow = lane & 31;
  const int lk = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    la.store(sA, tid);
    lb.store(sB, tid);
    __syncthreads();
    if (kt + 1 < nk) {
      la.load(A, d.lda, m0, (kt + 1) * BKB, d.M, d.Kd, vecA, tid);
      lb.load(B, d.ldb, n0, (kt + 1) * BKB, d.N, d.Kd, vecB, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BKB; kk += 16) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm * WM + i * 32 + lrow) * PITCH + kk + 8 * lk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&sB[(wn * WN + j * 32 + lrow) * PITCH + kk + 8 * lk]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  const float* aux = d.aux ? d.aux + (long)g * d.strideAux : nullptr;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * WN + j * 32 + lrow;
    if (col >= d.N) continue;
    float bias = 0.f;
    if (d.epilogue == EPI_BIAS || d.epilogue == EPI_BIAS_RELU) bias = aux[col];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * WM + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
        if (row >= d.M) continue;
        const long off = (long)row * d.ldc + col;
        float val = acc[i][j][v];
        switch (d.epilogue) {
          case EPI_BIAS: val += bias; break;
          case EPI_BIAS_RELU: val = fmaxf(val + bias, 0.f); break;
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

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg_bf16(const GemmDesc& d, int vecA, int vecB, hipStream_t s) {
  dim3 grid((d.N + BN - 1) / BN, (d.M + BM - 1) / BM, d.groups);
  dim3 block((BM / WM) * (BN / WN) * 64);
  KernelTimer kt(KID_GEMM_F32, 2.0 * d.M * d.N * (double)d.Kd * d.groups, s);
  if (!d.transA && d.transB)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, false, true>), grid, block, 0, s, d, vecA, vecB);
  else if (!d.transA && !d.transB)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, false, false>), grid, block, 0, s, d, vecA, vecB);
  else if (d.transA && !d.transB)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, true, false>), grid, block, 0, s, d, vecA, vecB);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, true, true>), grid, block, 0, s, d, vecA, vecB);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const GemmDesc& d, hipStream_t s) {
  auto vec_ok = [](const float* p, long ld, long stride) {
    return (((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (stride & 3) == 0) ? 1 : 0;
  };
  const int vecA = vec_ok(d.A, d.lda, d.strideA);
  const int vecB = vec_ok(d.B, d.ldb, d.strideB);
  auto tiles = [&](int bm, int bn) {
    return (long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.groups;
  };
  if (d.M > 64 && d.N > 64 && tiles(128, 128) >= 192) return launch_cfg_bf16<128, 128, 64, 64>(d, vecA, vecB, s);
  if (d.M > 32 && d.N > 32 && tiles(64, 64) >= 192) return launch_cfg_bf16<64, 64, 32, 32>(d, vecA, vecB, s);
  if (d.M > 32 && tiles(64, 32) >= 128) return launch_cfg_bf16<64, 32, 32, 32>(d, vecA, vecB, s);
  return launch_cfg_bf16<32, 32, 32, 32>(d, vecA, vecB, s);
}

}  // namespace hpsgd
