// Grouped fp32 GEMM on the CDNA4 fp32 matrix cores (v_mfma_f32_32x32x2_f32).
//
//   C[g] (M x N) = op(A[g]) (M x Kd) * op(B[g]) (Kd x N),  g = blockIdx.z  (one group per worker)
//
// Each workgroup owns a BM x BN tile of C and walks Kd in steps of BK = 16.  Both operand
// tiles are staged in LDS as [k][m] / [k][n] rows (the unit-stride index is the one the
// MFMA lanes vary over), so a wave's operand fetch for one MFMA is a conflict-free run of 32
// consecutive floats.  Global loads for tile kt+1 are issued before the MFMAs of tile kt and
// only written to LDS after them, so HBM/L2 latency hides behind the matrix work.
//
// MFMA 32x32x2 lane layout (64-lane wave): A operand lane l holds A[m = l%32][k = l/32],
// B operand lane l holds B[k = l/32][n = l%32]; accumulator register v of lane l holds
// C[8*(v/4) + 4*(l/32) + v%4][l%32].
#include "kernels.h"

namespace hpsgd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

static constexpr int BK = 16;
static constexpr int LDS_PAD = 4;

// One 4-float unit of an operand tile.  `contig_k`: the source is unit-stride along k
// (element (i,k) at base[i*ld + k]), else unit-stride along i (element (i,k) at base[k*ld + i]).
template <bool CONTIG_K>
__device__ __forceinline__ float4 load_unit(const float* __restrict__ base, long ld, int i, int k,
                                            int imax, int kmax, bool vec) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (CONTIG_K) {
    if (i < imax) {
      const float* p = base + (long)i * ld + k;
      if (vec && k + 3 < kmax) {
        v = *reinterpret_cast<const float4*>(p);
      } else {
        if (k + 0 < kmax) v.x = p[0];
        if (k + 1 < kmax) v.y = p[1];
        if (k + 2 < kmax) v.z = p[2];
        if (k + 3 < kmax) v.w = p[3];
      }
    }
  } else {
    if (k < kmax) {
      const float* p = base + (long)k * ld + i;
      if (vec && i + 3 < imax) {
        v = *reinterpret_cast<const float4*>(p);
      } else {
        if (i + 0 < imax) v.x = p[0];
        if (i + 1 < imax) v.y = p[1];
        if (i + 2 < imax) v.z = p[2];
        if (i + 3 < imax) v.w = p[3];
      }
    }
  }
  return v;
}

// Tile staging for one operand: BI rows (m or n) x BK, NT threads, U units per thread.
template <int BI, int NT, bool CONTIG_K>
struct TileLoader {
  static constexpr int UNITS = BI * BK / 4;
  static constexpr int U = (UNITS + NT - 1) / NT;
  float4 r[U];

  __device__ __forceinline__ void load(const float* __restrict__ base, long ld, int i0, int k0,
                                       int imax, int kmax, bool vec, int tid) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = tid + u * NT;
      if (UNITS % NT != 0 && unit >= UNITS) break;
      int i, k;
      if (CONTIG_K) {
        i = unit / (BK / 4);
        k = (unit % (BK / 4)) * 4;
      } else {
        k = unit / (BI / 4);
        i = (unit % (BI / 4)) * 4;
      }
      r[u] = load_unit<CONTIG_K>(base, ld, i0 + i, k0 + k, imax, kmax, vec);
    }
  }

  // LDS tile is [BK][BI + LDS_PAD]
  __device__ __forceinline__ void store(float* __restrict__ lds, int tid) const {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = tid + u * NT;
      if (UNITS % NT != 0 && unit >= UNITS) break;
      if (CONTIG_K) {
        const int i = unit / (BK / 4);
        const int k = (unit % (BK / 4)) * 4;
        lds[(k + 0) * (BI + LDS_PAD) + i] = r[u].x;
        lds[(k + 1) * (BI + LDS_PAD) + i] = r[u].y;
        lds[(k + 2) * (BI + LDS_PAD) + i] = r[u].z;
        lds[(k + 3) * (BI + LDS_PAD) + i] = r[u].w;
      } else {
        const int k = unit / (BI / 4);
        const int i = (unit % (BI / 4)) * 4;
        *reinterpret_cast<float4*>(&lds[k * (BI + LDS_PAD) + i]) = r[u];
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_f32_kernel(GemmDesc d, int vecA, int vecB) {
  constexpr int WAVES_M = BM / WM;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  __shared__ __attribute__((aligned(16))) float sA[BK * (BM + LDS_PAD)];
  __shared__ __attribute__((aligned(16))) float sB[BK * (BN + LDS_PAD)];

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

  // A is unit-stride along k when it is stored [M][Kd] (TA == false);
  // B is unit-stride along k when it is stored [N][Kd] (TB == true).
  TileLoader<BM, NT, !TA> la;
  TileLoader<BN, NT, TB> lb;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (d.Kd + BK - 1) / BK;
  la.load(A, d.lda, m0, 0, d.M, d.Kd, vecA, tid);
  lb.load(B, d.ldb, n0, 0, d.N, d.Kd, vecB, tid);

  const int lrow = lane & 31;
  const int lk = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    la.store(sA, tid);
    lb.store(sB, tid);
    __syncthreads();
    if (kt + 1 < nk) {
      la.load(A, d.lda, m0, (kt + 1) * BK, d.M, d.Kd, vecA, tid);
      lb.load(B, d.ldb, n0, (kt + 1) * BK, d.N, d.Kd, vecB, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = sA[(kk + lk) * (BM + LDS_PAD) + wm * WM + i * 32 + lrow];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = sB[(kk + lk) * (BN + LDS_PAD) + wn * WN + j * 32 + lrow];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue
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
static hipError_t launch_cfg(const GemmDesc& d, int vecA, int vecB, hipStream_t s) {
  dim3 grid((d.N + BN - 1) / BN, (d.M + BM - 1) / BM, d.groups);
  dim3 block((BM / WM) * (BN / WN) * 64);
  KernelTimer kt(KID_GEMM_F32, 2.0 * d.M * d.N * (double)d.Kd * d.groups, s);
  if (!d.transA && d.transB)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, false, true>), grid, block, 0, s, d, vecA, vecB);
  else if (!d.transA && !d.transB)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, false, false>), grid, block, 0, s, d, vecA, vecB);
  else if (d.transA && !d.transB)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, true, false>), grid, block, 0, s, d, vecA, vecB);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, true, true>), grid, block, 0, s, d, vecA, vecB);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const GemmDesc& d, hipStream_t s);      // gemm_bf16.hip
hipError_t launch_gemm_f32_fast(const GemmDesc& d, hipStream_t s);  // gemm_f32_fast.hip

hipError_t launch_gemm(const GemmDesc& d, hipStream_t s) {
  if (d.M <= 0 || d.N <= 0 || d.groups <= 0) return hipSuccess;
  if (d.splits > 1) {  // only the pipelined fp32 kernel cuts the contraction
    if (d.bf16 || d.background) return hipErrorInvalidValue;
    const hipError_t e = launch_gemm_f32_fast(d, s);
    return e == hipErrorNotSupported ? hipErrorInvalidValue : e;
  }
  if (d.bf16) return launch_gemm_bf16(d, s);
  if (!d.background) {
    // aligned operands: the pipelined kernel.  Not for background work: its LDS footprint (up to
    // 72 KB per workgroup) would keep the recurrent step kernels off the CUs it occupies.
    const hipError_t e = launch_gemm_f32_fast(d, s);
    if (e != hipErrorNotSupported) return e;
  }
  auto vec_ok = [](const float* p, long ld, long stride) {
    return (((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (stride & 3) == 0) ? 1 : 0;
  };
  const int vecA = vec_ok(d.A, d.lda, d.strideA);
  const int vecB = vec_ok(d.B, d.ldb, d.strideB);
  // Pick the largest tile that still yields at least ~1 workgroup per CU.
  auto tiles = [&](int bm, int bn) {
    return (long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.groups;
  };
  if (d.M > 64 && d.N > 64 && tiles(128, 128) >= 192) return launch_cfg<128, 128, 64, 64>(d, vecA, vecB, s);
  if (d.M > 32 && d.N > 32 && tiles(64, 64) >= 192) return launch_cfg<64, 64, 32, 32>(d, vecA, vecB, s);
  if (d.M > 32 && tiles(64, 32) >= 128) return launch_cfg<64, 32, 32, 32>(d, vecA, vecB, s);
  return launch_cfg<32, 32, 32, 32>(d, vecA, vecB, s);
}

}  // namespace hpsgd
