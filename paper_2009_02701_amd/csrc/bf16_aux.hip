// Helpers of the bf16 training path that are not contractions: rounded / transposed operand
// copies, the softmax-CE that emits bf16 logit gradients, and row sums of a bf16 matrix.
// Every time-batched GEMM of that path takes contraction-contiguous bf16 operands; these
// kernels produce the ones that no other kernel's epilogue writes.
#include "kernels.h"

namespace hpsgd {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// (the copy kernels read their input once and write what later launches read: non-temporal)
typedef float f4nt_a __attribute__((ext_vector_type(4)));
typedef unsigned u4nt_a __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4 load4_as_bf16(const float* p) {
  const f4nt_a v = __builtin_nontemporal_load(reinterpret_cast<const f4nt_a*>(p));
  bf16x4 r;
  r[0] = (__bf16)v.x; r[1] = (__bf16)v.y; r[2] = (__bf16)v.z; r[3] = (__bf16)v.w;
  return r;
}
__device__ __forceinline__ bf16x4 load4_as_bf16(const __bf16* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(p));
}

// in: R x C (fp32 or bf16, row pitch ld_in).  out_p (nullable): the bf16 rounding, row pitch
// ld_p.  out_t (nullable): its transpose, out_t[c][r], row pitch ld_t.  One 64 x 64 tile per
// workgroup, read once: 16-byte (fp32) or 8-byte (bf16) loads, 8-byte plain stores, and the
// transposed tile goes through LDS and leaves as 16-byte pieces of 8 consecutive input rows.
// Needs C % 4 == 0, R % 8 == 0 and the alignments cvt2_supported checks.
template <typename TIN>
__device__ __forceinline__ void cvt2_tile(const TIN* __restrict__ src, long ld_in, __bf16* __restrict__ dst_p, long ld_p,
                                          __bf16* __restrict__ dst_t, long ld_t, int R, int C, int c0, int r0,
                                          __bf16 (&tile)[64][72]) {
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  // All four loads are issued before anything waits for one (clamped addresses instead of
  // branches: behind a branch each load would be waited for, and stored, before the next is issued).
  const int c = c0 + 4 * tx;
  const bool c_ok = c < C;
  const int cl = c_ok ? c : C - 4;
  bf16x4 v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = load4_as_bf16(src + (long)min(r0 + ty + 16 * i, R - 1) * ld_in + cl);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rl = ty + 16 * i, r = r0 + rl;
    if (r < R && c_ok) {
      if (dst_p) __builtin_nontemporal_store(v[i], reinterpret_cast<bf16x4*>(dst_p + (long)r * ld_p + c));
    } else {
      v[i][0] = v[i][1] = v[i][2] = v[i][3] = (__bf16)0.f;
    }
    if (dst_t) {
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[4 * tx + e][rl] = v[i][e];
    }
  }
  if (!dst_t) return;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int idx = threadIdx.x + 256 * q, col = idx >> 3, part = idx & 7;
    const int c = c0 + col, r = r0 + 8 * part;
    if (c < C && r < R)
      __builtin_nontemporal_store(*reinterpret_cast<const u4nt_a*>(&tile[col][8 * part]),
                                  reinterpret_cast<u4nt_a*>(dst_t + (long)c * ld_t + r));
  }
}

template <typename TIN>
__global__ void __launch_bounds__(256)
cvt2_kernel(const TIN* __restrict__ in, long ld_in, long s_in, __bf16* __restrict__ out_p, long ld_p,
            long s_p, __bf16* __restrict__ out_t, long ld_t, long s_t, int R, int C) {
  __shared__ __attribute__((aligned(16))) __bf16 tile[64][72];  // [column][row]
  const int g = blockIdx.z;
  cvt2_tile<TIN>(in + g * s_in, ld_in, out_p ? out_p + g * s_p : nullptr, ld_p, out_t ? out_t + g * s_t : nullptr, ld_t,
                 R, C, blockIdx.x * 64, blockIdx.y * 64, tile);
}

// Several fp32 matrices in one launch (the weight matrices of a model: each is a few hundred
// tiles, and a launch of its own costs more than its copies).  blockIdx.x runs over the tiles of
// all jobs, job j owning [tile0[j], tile0[j+1]).
__global__ void __launch_bounds__(256) cvt2_pack_kernel(Cvt2Pack p) {
  __shared__ __attribute__((aligned(16))) __bf16 tile[64][72];
  int j = 0;
  while (j + 1 < p.n && (int)blockIdx.x >= p.tile0[j + 1]) ++j;  // (uniform)
  const Cvt2Job& q = p.job[j];
  const int t = blockIdx.x - p.tile0[j], g = blockIdx.z;
  __bf16* op = reinterpret_cast<__bf16*>(q.out_p);
  __bf16* ot = reinterpret_cast<__bf16*>(q.out_t);
  cvt2_tile<float>(q.in + g * q.s_in, q.ld_in, op ? op + g * q.s_p : nullptr, q.ld_p, ot ? ot + g * q.s_t : nullptr,
                   q.ld_t, q.R, q.C, (t % q.tiles_x) * 64, (t / q.tiles_x) * 64, tile);
}

bool cvt2_supported(const void* in, int in_bf16, long ld_in, long s_in, const void* out_p, long ld_p,
                    long s_p, const void* out_t, long ld_t, long s_t, int R, int C) {
  const uintptr_t in_mask = in_bf16 ? 7 : 15;
  if (((uintptr_t)in & in_mask) != 0 || ld_in % 4 != 0 || s_in % 4 != 0 || C % 4 != 0 || R % 8 != 0) return false;
  if (out_p && (((uintptr_t)out_p & 7) != 0 || ld_p % 4 != 0 || s_p % 4 != 0)) return false;
  if (out_t && (((uintptr_t)out_t & 15) != 0 || ld_t % 8 != 0 || s_t % 8 != 0)) return false;
  return R > 0 && C > 0;
}

hipError_t launch_cvt2(const void* in, int in_bf16, long ld_in, long s_in, void* out_p, long ld_p, long s_p,
                       void* out_t, long ld_t, long s_t, int R, int C, int groups, hipStream_t s) {
  if (!cvt2_supported(in, in_bf16, ld_in, s_in, out_p, ld_p, s_p, out_t, ld_t, s_t, R, C))
    return hipErrorInvalidValue;
  dim3 grid((C + 63) / 64, (R + 63) / 64, groups);
  // bytes: one read of the input, one write of each copy
  KernelTimer kt(KID_CVT2, (double)R * C * groups * ((in_bf16 ? 2 : 4) + (out_p ? 2 : 0) + (out_t ? 2 : 0)), s);
  if (in_bf16)
    hipLaunchKernelGGL(cvt2_kernel<__bf16>, grid, dim3(256), 0, s, (const __bf16*)in, ld_in, s_in,
                       (__bf16*)out_p, ld_p, s_p, (__bf16*)out_t, ld_t, s_t, R, C);
  else
    hipLaunchKernelGGL(cvt2_kernel<float>, grid, dim3(256), 0, s, (const float*)in, ld_in, s_in,
                       (__bf16*)out_p, ld_p, s_p, (__bf16*)out_t, ld_t, s_t, R, C);
  return hipGetLastError();
}

bool cvt2_pack_push(Cvt2Pack& p, const float* in, long ld_in, long s_in, void* out_p, long ld_p, long s_p,
                    void* out_t, long ld_t, long s_t, int R, int C) {
  if (p.n >= Cvt2Pack::MAX || !cvt2_supported(in, 0, ld_in, s_in, out_p, ld_p, s_p, out_t, ld_t, s_t, R, C)) return false;
  Cvt2Job& q = p.job[p.n];
  q.in = in; q.ld_in = ld_in; q.s_in = s_in;
  q.out_p = out_p; q.ld_p = ld_p; q.s_p = s_p;
  q.out_t = out_t; q.ld_t = ld_t; q.s_t = s_t;
  q.R = R; q.C = C;
  q.tiles_x = (C + 63) / 64;
  const long tiles = (long)q.tiles_x * ((R + 63) / 64);
  if (tiles + p.tile0[p.n] > (1L << 30)) return false;
  p.tile0[p.n + 1] = p.tile0[p.n] + (int)tiles;
  p.bytes += (double)R * C * (4 + (out_p ? 2 : 0) + (out_t ? 2 : 0));
  ++p.n;
  return true;
}

hipError_t launch_cvt2_pack(const Cvt2Pack& p, int groups, hipStream_t s) {
  if (p.n == 0 || groups <= 0) return hipSuccess;
  KernelTimer kt(KID_CVT2_PACK, p.bytes * groups, s);
  hipLaunchKernelGGL(cvt2_pack_kernel, dim3(p.tile0[p.n], 1, groups), dim3(256), 0, s, p);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- softmax-CE, bf16 gradient
// One workgroup per row; the row (C <= 1024 * V4 logits) is read once into registers.
// Writes dlogits = (softmax - onehot)/N rounded to bf16 (row pitch ld_d), the row's loss
// -log softmax[y] and the row's (max, 1/sum) pair; the logits stay as they are.
template <int V4>
__global__ void __launch_bounds__(256)
softmax_ce_bf16_kernel(const float* __restrict__ logits, long s_logits, const int32_t* __restrict__ y,
                       long s_y, __bf16* __restrict__ dlog, long ld_d, long s_d,
                       float* __restrict__ rowloss, long s_rowloss, float2* __restrict__ rowstat,
                       long s_rowstat, int N, int C) {
  __shared__ float red[4];
  __shared__ float bcast;
  const int g = blockIdx.y, row = blockIdx.x;
  const float* lr = logits + g * s_logits + (long)row * C;
  const int label = y[g * s_y + row];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float4 v[V4];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int c = 4 * (tid + 256 * i);
    if (c < C) {
      v[i] = *reinterpret_cast<const float4*>(lr + c);
      m = fmaxf(fmaxf(m, fmaxf(v[i].x, v[i].y)), fmaxf(v[i].z, v[i].w));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if (lane == 0) red[wave] = m;
  __syncthreads();
  if (tid == 0) bcast = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  m = bcast;
  __syncthreads();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int c = 4 * (tid + 256 * i);
    if (c < C) {
      v[i].x = expf(v[i].x - m); v[i].y = expf(v[i].y - m);
      v[i].z = expf(v[i].z - m); v[i].w = expf(v[i].w - m);
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) bcast = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  sum = bcast;
  const float inv_sum = 1.0f / sum, inv_n = 1.0f / (float)N;
  if (tid == 0) {
    rowloss[g * s_rowloss + row] = -((lr[label] - m) - logf(sum));
    rowstat[g * s_rowstat + row] = make_float2(m, inv_sum);
  }
  __bf16* dr = dlog + g * s_d + (long)row * ld_d;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int c = 4 * (tid + 256 * i);
    if (c < C) {
      bf16x4 o;
      o[0] = (__bf16)((v[i].x * inv_sum - (c + 0 == label ? 1.0f : 0.0f)) * inv_n);
      o[1] = (__bf16)((v[i].y * inv_sum - (c + 1 == label ? 1.0f : 0.0f)) * inv_n);
      o[2] = (__bf16)((v[i].z * inv_sum - (c + 2 == label ? 1.0f : 0.0f)) * inv_n);
      o[3] = (__bf16)((v[i].w * inv_sum - (c + 3 == label ? 1.0f : 0.0f)) * inv_n);
      *reinterpret_cast<bf16x4*>(dr + c) = o;
    }
  }
}

// The same for SMR consecutive rows per workgroup, which also sums the unrounded gradient of its
// rows per column (a thread owns the same columns in every row): colpart[g][block][c], the
// partial sums of the head's bias gradient, added up by a second small kernel.  The next row's
// loads are issued before the current row is reduced.
constexpr int SMR = 8;  // the fewest rows per workgroup

template <int V4, int NT>
__global__ void __launch_bounds__(NT)
softmax_ce_bf16_rows_kernel(const float* __restrict__ logits, long s_logits, const int32_t* __restrict__ y,
                            long s_y, __bf16* __restrict__ dlog, long ld_d, long s_d,
                            float* __restrict__ rowloss, long s_rowloss, float2* __restrict__ rowstat,
                            long s_rowstat, float* __restrict__ colpart, long s_colpart, int N, int C, int rpb) {
  // partial results of the NW waves, one set per reduction and row parity: a set is written
  // again two rows later, with two barriers in between, so one barrier per reduction is enough
  constexpr int NW = NT / 64;
  static_assert(NW == 4 || NW == 8, "four or eight waves");
  __shared__ float red_m[2][NW], red_s[2][NW];
  const int g = blockIdx.y, row0 = blockIdx.x * rpb;
  const int nr = min(rpb, N - row0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float inv_n = 1.0f / (float)N;
  float4 acc[V4], nx[V4];
#pragma unroll
  for (int i = 0; i < V4; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  auto load_row = [&](int row) {
    const float* lr = logits + g * s_logits + (long)row * C;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int c = 4 * (tid + NT * i);
      typedef float f4nt __attribute__((ext_vector_type(4)));
      const f4nt t4 = __builtin_nontemporal_load(reinterpret_cast<const f4nt*>(lr + (c < C ? c : 0)));
      nx[i] = make_float4(t4.x, t4.y, t4.z, t4.w);
    }
  };
  load_row(row0);
  for (int r = 0; r < nr; ++r) {
    const int row = row0 + r;
    const int label = y[g * s_y + row];
    float4 v[V4];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      v[i] = nx[i];
      if (4 * (tid + NT * i) < C) m = fmaxf(fmaxf(m, fmaxf(v[i].x, v[i].y)), fmaxf(v[i].z, v[i].w));
    }
    if (r + 1 < nr) load_row(row + 1);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) red_m[r & 1][wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red_m[r & 1][0], red_m[r & 1][1]), fmaxf(red_m[r & 1][2], red_m[r & 1][3]));
    if (NW == 8)
      m = fmaxf(m, fmaxf(fmaxf(red_m[r & 1][NW - 4], red_m[r & 1][NW - 3]), fmaxf(red_m[r & 1][NW - 2], red_m[r & 1][NW - 1])));
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < V4; ++i)
      if (4 * (tid + NT * i) < C) {
        v[i].x = expf(v[i].x - m); v[i].y = expf(v[i].y - m);
        v[i].z = expf(v[i].z - m); v[i].w = expf(v[i].w - m);
        sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red_s[r & 1][wave] = sum;
    __syncthreads();
    sum = (red_s[r & 1][0] + red_s[r & 1][1]) + (red_s[r & 1][2] + red_s[r & 1][3]);
    if (NW == 8)
      sum += (red_s[r & 1][NW - 4] + red_s[r & 1][NW - 3]) + (red_s[r & 1][NW - 2] + red_s[r & 1][NW - 1]);
    const float inv_sum = 1.0f / sum;
    if (tid == 0) {
      rowloss[g * s_rowloss + row] = -((logits[g * s_logits + (long)row * C + label] - m) - logf(sum));
      rowstat[g * s_rowstat + row] = make_float2(m, inv_sum);
    }
    __bf16* dr = dlog + g * s_d + (long)row * ld_d;
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int c = 4 * (tid + NT * i);
      if (c < C) {
        const float4 d4 = make_float4((v[i].x * inv_sum - (c + 0 == label ? 1.0f : 0.0f)) * inv_n,
                                      (v[i].y * inv_sum - (c + 1 == label ? 1.0f : 0.0f)) * inv_n,
                                      (v[i].z * inv_sum - (c + 2 == label ? 1.0f : 0.0f)) * inv_n,
                                      (v[i].w * inv_sum - (c + 3 == label ? 1.0f : 0.0f)) * inv_n);
        acc[i].x += d4.x; acc[i].y += d4.y; acc[i].z += d4.z; acc[i].w += d4.w;
        bf16x4 o;
        o[0] = (__bf16)d4.x; o[1] = (__bf16)d4.y; o[2] = (__bf16)d4.z; o[3] = (__bf16)d4.w;
        __builtin_nontemporal_store(o, reinterpret_cast<bf16x4*>(dr + c));
      }
    }
  }
  float* cp = colpart + g * s_colpart + (long)blockIdx.x * C;
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int c = 4 * (tid + NT * i);
    if (c < C) *reinterpret_cast<float4*>(cp + c) = acc[i];
  }
}

// Rows per workgroup.  The kernel holds three workgroups of four waves per CU (168 registers; two of
// eight waves for long rows), and a launch
// whose workgroups outnumber those places leaves the chip half empty at its end: 1120 x 8 rows in
// blocks of 8 are 1120 workgroups for 768 places, i.e. 16 rows' time where blocks of 12 take 12.
// So: as many rows per workgroup as fill every place once, at least SMR, at most 64.
// sizing_groups: the number of workers the launch is sized for (0: the upper bound on the number
// of blocks, for allocations).
static bool softmax_rows_wide(int C) { return C > 4096; }  // eight waves, five vectors per thread

int softmax_ce_bf16_rows_per_block(int N, int sizing_groups, int C) {
  if (sizing_groups <= 0) return SMR;
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      return SMR;
  }
  const int places = (softmax_rows_wide(C) ? 2 : 3) * cus;
  const long rows = (long)N * sizing_groups;
  long rpb = (rows + places - 1) / places;
  if (rpb < SMR) rpb = SMR;
  if (rpb > 64) rpb = 64;
  return (int)rpb;
}
int softmax_ce_bf16_row_blocks(int N, int sizing_groups, int C) {
  const int rpb = softmax_ce_bf16_rows_per_block(N, sizing_groups, C);
  return (N + rpb - 1) / rpb;
}

bool softmax_ce_bf16_supported(const float* logits, long s_logits, const void* dlog, long ld_d, long s_d,
                               int C) {
  return C % 4 == 0 && C >= 4 && C <= 1024 * 10 && ((uintptr_t)logits & 15) == 0 && s_logits % 4 == 0 &&
         ((uintptr_t)dlog & 7) == 0 && ld_d % 4 == 0 && s_d % 4 == 0;
}

// colpart (nullable): [groups][softmax_ce_bf16_row_blocks(N)][C] floats (group stride s_colpart, a
// multiple of 4, 16-byte aligned), receives the per-block column sums of the unrounded gradient.
hipError_t launch_softmax_ce_bf16(const float* logits, long s_logits, const int32_t* y, long s_y, void* dlog,
                                  long ld_d, long s_d, float* rowloss, long s_rowloss, float* rowstat,
                                  long s_rowstat, int N, int C, int groups, hipStream_t s, float* colpart,
                                  long s_colpart, int sizing_groups) {
  if (!softmax_ce_bf16_supported(logits, s_logits, dlog, ld_d, s_d, C)) return hipErrorInvalidValue;
  // bytes: the logits read once (fp32), the logit gradient written in bf16
  KernelTimer kt(KID_SOFTMAX_CE_BF16, 6.0 * N * C * groups, s);
  if (colpart) {
    if (((uintptr_t)colpart & 15) != 0 || s_colpart % 4 != 0) return hipErrorInvalidValue;
    const int rpb = softmax_ce_bf16_rows_per_block(N, sizing_groups, C);
    dim3 grid((N + rpb - 1) / rpb, groups);
#define HPSGD_SMR(V4, NT)                                                                                      \
  hipLaunchKernelGGL((softmax_ce_bf16_rows_kernel<V4, NT>), grid, dim3(NT), 0, s, logits, s_logits, y, s_y,  \
                     (__bf16*)dlog, ld_d, s_d, rowloss, s_rowloss, reinterpret_cast<float2*>(rowstat),       \
                     s_rowstat / 2, colpart, s_colpart, N, C, rpb)
    if (C <= 1024) HPSGD_SMR(1, 256);
    else if (!softmax_rows_wide(C)) HPSGD_SMR(4, 256);
    else HPSGD_SMR(5, 512);
#undef HPSGD_SMR
    return hipGetLastError();
  }
  dim3 grid(N, groups);
#define HPSGD_SM(V4)                                                                                    \
  hipLaunchKernelGGL(softmax_ce_bf16_kernel<V4>, grid, dim3(256), 0, s, logits, s_logits, y, s_y,       \
                     (__bf16*)dlog, ld_d, s_d, rowloss, s_rowloss, reinterpret_cast<float2*>(rowstat),        \
                     s_rowstat / 2, N, C)
  if (C <= 1024) HPSGD_SM(1);
  else if (C <= 4096) HPSGD_SM(4);
  else HPSGD_SM(10);
#undef HPSGD_SM
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- bias gradient of the head
// out[c] = (1/N) sum_r (softmax[r][c] - [y_r == c]), recomputed in fp32 from the logits and
// the rows' (max, 1/sum) pairs: the bias gradient is not a GEMM operand and is not rounded.
// A workgroup of 1024 threads covers 64 columns with 16 row slices, combined in a fixed order.
__global__ void __launch_bounds__(1024)
colsum_softmax_kernel(const float* __restrict__ logits, long s_logits, const float2* __restrict__ rowstat,
                      long s_rowstat, const int32_t* __restrict__ y, long s_y, float* __restrict__ out,
                      long s_out, int N, int C) {
  __shared__ float red[16][64];
  const int g = blockIdx.y, lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float a = 0.f;
  if (c < C) {
    const float* p = logits + g * s_logits + c;
    for (int r = slice; r < N; r += 16) {
      const float2 st = rowstat[g * s_rowstat + r];
      a += expf(p[(long)r * C] - st.x) * st.y - (y[g * s_y + r] == c ? 1.0f : 0.0f);
    }
  }
  red[slice][lane] = a;
  __syncthreads();
  if (slice == 0 && c < C) {
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) v += red[i][lane];
    out[g * s_out + c] = v / (float)N;
  }
}

// The same with four columns per lane (16-byte loads; C % 4 == 0, 16-byte aligned rows) and four
// rows in flight per trip: a workgroup covers 256 columns with 16 row slices.
__global__ void __launch_bounds__(1024)
colsum_softmax4_kernel(const float* __restrict__ logits, long s_logits, const float2* __restrict__ rowstat,
                       long s_rowstat, const int32_t* __restrict__ y, long s_y, float* __restrict__ out,
                       long s_out, int N, int C) {
  __shared__ float4 red[16][64];
  const int g = blockIdx.y, lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int c = blockIdx.x * 256 + 4 * lane;
  const bool cv = c < C;
  const float* p = logits + g * s_logits + (cv ? c : 0);
  const float2* st = rowstat + g * s_rowstat;
  const int32_t* yg = y + g * s_y;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  // rows slice, slice + 16, ..: four per trip, all their loads issued before the first is used
  for (int r0 = slice; r0 < N; r0 += 64) {
    float4 v[4];
    float2 s4[4];
    int lab[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = min(r0 + 16 * u, N - 1);
      v[u] = *reinterpret_cast<const float4*>(p + (long)r * C);
      s4[u] = st[r];
      lab[u] = yg[r];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (r0 + 16 * u < N) {
        a.x += expf(v[u].x - s4[u].x) * s4[u].y - (lab[u] == c ? 1.0f : 0.0f);
        a.y += expf(v[u].y - s4[u].x) * s4[u].y - (lab[u] == c + 1 ? 1.0f : 0.0f);
        a.z += expf(v[u].z - s4[u].x) * s4[u].y - (lab[u] == c + 2 ? 1.0f : 0.0f);
        a.w += expf(v[u].w - s4[u].x) * s4[u].y - (lab[u] == c + 3 ? 1.0f : 0.0f);
      }
  }
  red[slice][lane] = a;
  __syncthreads();
  if (slice == 0 && cv) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float4 t = red[i][lane];
      v.x += t.x;
      v.y += t.y;
      v.z += t.z;
      v.w += t.w;
    }
    const float inv = 1.0f / (float)N;
    *reinterpret_cast<float4*>(out + g * s_out + c) = make_float4(v.x * inv, v.y * inv, v.z * inv, v.w * inv);
  }
}

hipError_t launch_colsum_softmax(const float* logits, long s_logits, const float* rowstat, long s_rowstat,
                                 const int32_t* y, long s_y, float* out, long s_out, int N, int C, int groups,
                                 hipStream_t s) {
  if (C % 4 == 0 && ((uintptr_t)logits & 15) == 0 && (s_logits & 3) == 0 && ((uintptr_t)out & 15) == 0 &&
      (s_out & 3) == 0) {
    hipLaunchKernelGGL(colsum_softmax4_kernel, dim3((C + 255) / 256, groups), dim3(1024), 0, s, logits, s_logits,
                       reinterpret_cast<const float2*>(rowstat), s_rowstat / 2, y, s_y, out, s_out, N, C);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(colsum_softmax_kernel, dim3((C + 63) / 64, groups), dim3(1024), 0, s, logits, s_logits,
                     reinterpret_cast<const float2*>(rowstat), s_rowstat / 2, y, s_y, out, s_out, N, C);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- row sums of a bf16 matrix
// out[r] = sum_c in[r][c] (fp32 accumulation): one wave per row, lanes stride over 8-element
// pieces, fixed combination order.  C % 8 == 0, rows 16-byte aligned.
__global__ void __launch_bounds__(256)
rowsum_bf16_kernel(const __bf16* __restrict__ in, long ld, long s_in, float* __restrict__ out, long s_out,
                   int R, int C) {
  const int g = blockIdx.y, lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= R) return;
  const __bf16* p = in + g * s_in + (long)r * ld;
  float a = 0.f;
  for (int c = 8 * lane; c < C; c += 512) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(p + c);
    a += (((float)v[0] + (float)v[1]) + ((float)v[2] + (float)v[3])) +
         (((float)v[4] + (float)v[5]) + ((float)v[6] + (float)v[7]));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  if (lane == 0) out[g * s_out + r] = a;
}

hipError_t launch_rowsum_bf16(const void* in, long ld, long s_in, float* out, long s_out, int R, int C,
                              int groups, hipStream_t s) {
  if (C % 8 != 0 || ld % 8 != 0 || s_in % 8 != 0 || ((uintptr_t)in & 15) != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rowsum_bf16_kernel, dim3((R + 3) / 4, groups), dim3(256), 0, s, (const __bf16*)in, ld,
                     s_in, out, s_out, R, C);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- matrix-core rate probe
// 16 independent 32x32 accumulator tiles per wave (256 accumulator registers: one wave per
// SIMD), operands fixed in registers: nothing but MFMA issue.  256 workgroups of 4 waves: one
// wave on every SIMD of the chip.  Records the shader-clock and the 100 MHz wall-clock ticks of workgroup 0.
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8p __attribute__((ext_vector_type(8)));

template <bool BF16>
__global__ void __launch_bounds__(256)
mfma_probe_kernel(const unsigned char* __restrict__ operands, int iters, double* __restrict__ result,
                  float* __restrict__ sink) {
  const int tid = threadIdx.x;
  uint4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *reinterpret_cast<const uint4*>(operands + ((tid * 4 + i) * 16) % 8192);
    rb[i] = *reinterpret_cast<const uint4*>(operands + 8192 + ((tid * 4 + i) * 16) % 8192);
  }
  floatx16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (BF16)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8p, ra[i & 3]),
                                                         __builtin_bit_cast(bf16x8p, rb[(i >> 2) & 3]), acc[i], 0, 0, 0);
      else
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, ra[i & 3].x),
                                                      __builtin_bit_cast(float, rb[(i >> 2) & 3].x), acc[i], 0, 0, 0);
    }
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) sum += acc[i][v];
  sink[blockIdx.x * 256 + tid] = sum;
  if (blockIdx.x == 0 && tid == 0) {
    result[0] = (double)(c1 - c0);
    result[1] = (double)(w1 - w0);
    result[2] = 16.0 * iters;
    result[3] = BF16 ? 32768.0 : 4096.0;
  }
}

hipError_t launch_mfma_probe(bool bf16, const void* operands, int iterations, double* result, float* sink,
                             hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(256), dim3(256), 0, s, (const unsigned char*)operands,
                       iterations, result, sink);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(256), dim3(256), 0, s, (const unsigned char*)operands,
                       iterations, result, sink);
  return hipGetLastError();
}

}  // namespace hpsgd
