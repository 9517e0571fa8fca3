// HBM-streaming kernels over flat fp32 parameter buffers: replica merge (Eq. 1), replica
// sync (Alg. 2 "make replica"), SGD commit (Alg. 2 "update replica"), zero fill and the
// time-major batch gather.  All work on 16-byte vectors: every lane keeps K+2 independent
// loads in flight and every wave reads and writes 1 KiB contiguous per stream.  Merge and
// sync are launched with one vector per lane (a grid as long as the buffer): on this chip
// that measured 10-20% faster than a resident grid-stride grid, and the merge's operands,
// each touched exactly once, are read and written with non-temporal hints.
#include "kernels.h"

namespace hpsgd {

static constexpr int kThreads = 256;
static constexpr int kMaxBlocks = 256 * 8;  // 256 CUs, up to 8 resident blocks each

// one 256-lane workgroup per 256 vectors (the kernels still stride, should the cap bind)
static inline int onepass_blocks(size_t n_items) {
  size_t b = (n_items + kThreads - 1) / kThreads;
  if (b > (size_t)1 << 30) b = (size_t)1 << 30;
  if (b < 1) b = 1;
  return (int)b;
}

typedef float f4v __attribute__((ext_vector_type(4)));

static inline int stream_blocks(size_t n_items) {
  size_t b = (n_items + kThreads - 1) / kThreads;
  if (b > (size_t)kMaxBlocks) b = kMaxBlocks;
  if (b < 1) b = 1;
  return (int)b;
}

// ---------------------------------------------------------------------------- merge
// global[j] += (1/K) * sum_k (replica_k[j] - snapshot[j]); the sum over k runs in order.
template <int KT>
__global__ void __launch_bounds__(kThreads)
merge_kernel(float* global, PtrPack rep, const float* snapshot, int Krt, float inv_k,
             size_t n4, size_t P) {
  const int K = KT > 0 ? KT : Krt;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    const f4v s = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(snapshot) + i);
    const f4v g = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(global) + i);
    f4v acc = (f4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const f4v r = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(rep.p[k]) + i);
      acc += r - s;
    }
    __builtin_nontemporal_store(g + acc * inv_k, reinterpret_cast<f4v*>(global) + i);
  }
  // ragged tail (P not a multiple of 4): the first block's first lanes
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) {
      const float s = snapshot[j];
      float acc = 0.f;
      for (int k = 0; k < K; ++k) acc += rep.p[k][j] - s;
      global[j] = global[j] + acc * inv_k;
    }
  }
}

hipError_t launch_merge(float* global, const PtrPack& replicas, const float* snapshot, int K,
                        size_t P, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t n4 = P / 4;
  const int blocks = onepass_blocks(n4);
  const float inv_k = 1.0f / (float)K;
#define HPSGD_MERGE_CASE(KT)                                                                  \
  hipLaunchKernelGGL(merge_kernel<KT>, dim3(blocks), dim3(kThreads), 0, s, global, replicas, \
                     snapshot, K, inv_k, n4, P)
  switch (K) {
    case 1: HPSGD_MERGE_CASE(1); break;
    case 2: HPSGD_MERGE_CASE(2); break;
    case 4: HPSGD_MERGE_CASE(4); break;
    case 8: HPSGD_MERGE_CASE(8); break;
    case 16: HPSGD_MERGE_CASE(16); break;
    default: HPSGD_MERGE_CASE(0); break;
  }
#undef HPSGD_MERGE_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- sync
template <int KT>
__global__ void __launch_bounds__(kThreads)
sync_kernel(const float* __restrict__ global, PtrPack rep, int Krt, float* snapshot, size_t n4,
            size_t P) {
  const int K = KT > 0 ? KT : Krt;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    const float4 g = reinterpret_cast<const float4*>(global)[i];
#pragma unroll
    for (int k = 0; k < K; ++k) reinterpret_cast<float4*>(rep.p[k])[i] = g;
    if (snapshot) reinterpret_cast<float4*>(snapshot)[i] = g;
  }
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) {
      const float g = global[j];
      for (int k = 0; k < K; ++k) rep.p[k][j] = g;
      if (snapshot) snapshot[j] = g;
    }
  }
}

hipError_t launch_sync_all(const float* global, const PtrPack& replicas, int K, float* snapshot,
                           size_t P, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t n4 = P / 4;
  const int blocks = onepass_blocks(n4);
#define HPSGD_SYNC_CASE(KT)                                                                  \
  hipLaunchKernelGGL(sync_kernel<KT>, dim3(blocks), dim3(kThreads), 0, s, global, replicas, K, \
                     snapshot, n4, P)
  switch (K) {
    case 1: HPSGD_SYNC_CASE(1); break;
    case 2: HPSGD_SYNC_CASE(2); break;
    case 4: HPSGD_SYNC_CASE(4); break;
    case 8: HPSGD_SYNC_CASE(8); break;
    case 16: HPSGD_SYNC_CASE(16); break;
    default: HPSGD_SYNC_CASE(0); break;
  }
#undef HPSGD_SYNC_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- merge + sync in one pass
// global[j] += (1/K) * sum_k (replica_k[j] - snapshot[j]), then replica_k[j] = snapshot[j] = global[j]:
// what merge_kernel followed by sync_kernel leaves, with every buffer read once and written once
// (4 (2K + 4) bytes per parameter instead of 4 (2K + 5)).  A lane reads its elements of all K + 2
// buffers before it writes any of them, so the update in place is safe.
// CLONE = false: the replicas are only read (the snapshot alone is taken: 4 (K + 4) bytes per
// parameter, against 4 (K + 3) + 8 for the merge followed by a copy of its result).
template <int KT, bool CLONE>
__global__ void __launch_bounds__(kThreads)
merge_sync_kernel(float* global, PtrPack rep, float* snapshot, int Krt, float inv_k, size_t n4, size_t P) {
  const int K = KT > 0 ? KT : Krt;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    const f4v s = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(snapshot) + i);
    const f4v g = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(global) + i);
    f4v acc = (f4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const f4v r = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(rep.p[k]) + i);
      acc += r - s;
    }
    const f4v o = g + acc * inv_k;
    __builtin_nontemporal_store(o, reinterpret_cast<f4v*>(global) + i);
    if (CLONE) {
#pragma unroll
      for (int k = 0; k < K; ++k) __builtin_nontemporal_store(o, reinterpret_cast<f4v*>(rep.p[k]) + i);
    }
    __builtin_nontemporal_store(o, reinterpret_cast<f4v*>(snapshot) + i);
  }
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) {
      const float s = snapshot[j];
      float acc = 0.f;
      for (int k = 0; k < K; ++k) acc += rep.p[k][j] - s;
      const float o = global[j] + acc * inv_k;
      global[j] = o;
      if (CLONE)
        for (int k = 0; k < K; ++k) rep.p[k][j] = o;
      snapshot[j] = o;
    }
  }
}

hipError_t launch_merge_sync(float* global, const PtrPack& replicas, float* snapshot, int K, size_t P,
                             hipStream_t s, bool clone) {
  if (P == 0) return hipSuccess;
  const size_t n4 = P / 4;
  const int blocks = onepass_blocks(n4);
  const float inv_k = 1.0f / (float)K;
#define HPSGD_MS_CASE(KT)                                                                                  \
  do {                                                                                                     \
    if (clone)                                                                                             \
      hipLaunchKernelGGL((merge_sync_kernel<KT, true>), dim3(blocks), dim3(kThreads), 0, s, global, replicas, \
                         snapshot, K, inv_k, n4, P);                                                       \
    else                                                                                                   \
      hipLaunchKernelGGL((merge_sync_kernel<KT, false>), dim3(blocks), dim3(kThreads), 0, s, global, replicas, \
                         snapshot, K, inv_k, n4, P);                                                       \
  } while (0)
  switch (K) {
    case 1: HPSGD_MS_CASE(1); break;
    case 2: HPSGD_MS_CASE(2); break;
    case 4: HPSGD_MS_CASE(4); break;
    case 8: HPSGD_MS_CASE(8); break;
    case 16: HPSGD_MS_CASE(16); break;
    default: HPSGD_MS_CASE(0); break;
  }
#undef HPSGD_MS_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- commit
// out[k][j] = in[k][j] - lr * grad[k][j]  (in_stride 0: every worker starts from the one model `in`)
__global__ void __launch_bounds__(kThreads)
commit_kernel(const float* in, size_t in_stride, float* out, size_t stride, const float* __restrict__ grad,
              size_t grad_stride, float lr, size_t n4, size_t P) {
  const int k = blockIdx.y;
  const float* ink = in + (size_t)k * in_stride;
  float* outk = out + (size_t)k * stride;
  const float* gk = grad + (size_t)k * grad_stride;
  const size_t step = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += step) {
    const float4 w = reinterpret_cast<const float4*>(ink)[i];
    const float4 g = reinterpret_cast<const float4*>(gk)[i];
    float4 o;
    o.x = w.x - lr * g.x;
    o.y = w.y - lr * g.y;
    o.z = w.z - lr * g.z;
    o.w = w.w - lr * g.w;
    reinterpret_cast<float4*>(outk)[i] = o;
  }
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) outk[j] = ink[j] - lr * gk[j];
  }
}

// the same, one element per thread: for ranges that do not start on a 16-byte boundary
__global__ void __launch_bounds__(kThreads)
commit_scalar_kernel(const float* in, size_t in_stride, float* out, size_t stride, const float* __restrict__ grad,
                     size_t grad_stride, float lr, size_t P) {
  const size_t k = blockIdx.y;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < P; i += (size_t)gridDim.x * kThreads)
    out[k * stride + i] = in[k * in_stride + i] - lr * grad[k * grad_stride + i];
}

hipError_t launch_commit(const float* in, size_t in_stride, float* out, size_t stride, const float* grad,
                         size_t grad_stride, float lr, int K, size_t P, hipStream_t s) {
  if (P == 0) return hipSuccess;
  KernelTimer kt(KID_COMMIT, 12.0 * (double)P * K, s);
  if ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)grad) & 15) != 0 || ((in_stride | stride | grad_stride) & 3) != 0) {
    size_t blocks = (P + kThreads - 1) / kThreads;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(commit_scalar_kernel, dim3((unsigned)blocks, K), dim3(kThreads), 0, s, in, in_stride, out, stride,
                       grad, grad_stride, lr, P);
    return hipGetLastError();
  }
  const size_t n4 = P / 4;
  const int blocks = onepass_blocks(n4);
  hipLaunchKernelGGL(commit_kernel, dim3(blocks, K), dim3(kThreads), 0, s, in, in_stride, out, stride, grad,
                     grad_stride, lr, n4, P);
  return hipGetLastError();
}

// sum + p[n4] + p[2 n4] + .. + p[(n_parts-1) n4], added in that order; the loads of 16 parts are in
// flight together (with one load per trip a sum over 140 parts waits out 140 memory latencies)
__device__ __forceinline__ float4 add_parts_in_order(const float4* p, size_t n4, int n_parts, float4 sum) {
  int q = 1;
  for (; q + 16 <= n_parts; q += 16) {
    float4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(size_t)(q + u) * n4];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      sum.x += v[u].x;
      sum.y += v[u].y;
      sum.z += v[u].z;
      sum.w += v[u].w;
    }
  }
  for (; q < n_parts; ++q) {
    const float4 v = p[(size_t)q * n4];
    sum.x += v.x;
    sum.y += v.y;
    sum.z += v.z;
    sum.w += v.w;
  }
  return sum;
}

// Partial sums of a weight gradient (one per batch-row tile of the recurrence kernel), added in
// tile order, then either committed (out = in - lr * sum) or stored (out = sum).  n % 4 == 0.
__global__ void __launch_bounds__(kThreads)
reduce_parts_kernel(const float* __restrict__ parts, int n_parts, size_t n4, const float* in, size_t s_in,
                    float* out, size_t s_out, float lr, int commit) {
  const size_t k = blockIdx.y;
  const float4* pk = reinterpret_cast<const float4*>(parts) + k * n_parts * n4;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const float4 sum0 = pk[i];
    float4 sum = add_parts_in_order(pk + i, n4, n_parts, sum0);
    if (commit) {
      const float4 w = reinterpret_cast<const float4*>(in + k * s_in)[i];
      sum = make_float4(w.x - lr * sum.x, w.y - lr * sum.y, w.z - lr * sum.z, w.w - lr * sum.w);
    }
    reinterpret_cast<float4*>(out + k * s_out)[i] = sum;
  }
}

// Several such sums in one launch (each of these kernels is a few microseconds of work behind
// a launch): segment i owns the grid columns blk0[i] .. blk0[i+1]-1.
__global__ void __launch_bounds__(kThreads) reduce_parts_multi_kernel(ReducePack pk) {
  int sgi = 0;
#pragma unroll
  for (int i = 1; i < ReducePack::MAXSEG; ++i)
    if (i < pk.n && blockIdx.x >= pk.blk0[i]) sgi = i;
  const ReduceSeg& sg = pk.seg[sgi];
  const size_t k = blockIdx.y, n4 = sg.n4;
  const unsigned nblk = pk.blk0[sgi + 1] - pk.blk0[sgi];
  const float4* pkp = reinterpret_cast<const float4*>(sg.parts) + k * sg.n_parts * n4;
  for (size_t i = (size_t)(blockIdx.x - pk.blk0[sgi]) * kThreads + threadIdx.x; i < n4; i += (size_t)nblk * kThreads) {
    const float4 sum0 = pkp[i];
    float4 sum = add_parts_in_order(pkp + i, n4, sg.n_parts, sum0);
    if (sg.commit) {
      const float4 w = reinterpret_cast<const float4*>(sg.in + k * sg.s_in)[i];
      sum = make_float4(w.x - pk.lr * sum.x, w.y - pk.lr * sum.y, w.z - pk.lr * sum.z, w.w - pk.lr * sum.w);
    }
    reinterpret_cast<float4*>(sg.out + k * sg.s_out)[i] = sum;
  }
}

bool reduce_pack_push(ReducePack& pk, const float* parts, int n_parts, size_t n, const float* in, size_t s_in,
                      float* out, size_t s_out, int commit) {
  if (pk.n >= ReducePack::MAXSEG || n == 0 || n_parts < 1 || (n & 3) != 0 || ((uintptr_t)parts & 15) != 0 ||
      ((uintptr_t)out & 15) != 0 || (s_out & 3) != 0 || (commit && (!in || ((uintptr_t)in & 15) != 0 || (s_in & 3) != 0)))
    return false;
  ReduceSeg& sg = pk.seg[pk.n];
  sg.parts = parts; sg.n_parts = n_parts; sg.n4 = n / 4; sg.in = in; sg.s_in = s_in; sg.out = out; sg.s_out = s_out;
  sg.commit = commit;
  pk.blk0[pk.n + 1] = pk.blk0[pk.n] + (unsigned)onepass_blocks(n / 4);
  ++pk.n;
  return true;
}

hipError_t launch_reduce_pack(const ReducePack& pk, int groups, hipStream_t s) {
  if (pk.n == 0 || groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(reduce_parts_multi_kernel, dim3(pk.blk0[pk.n], groups), dim3(kThreads), 0, s, pk);
  return hipGetLastError();
}

hipError_t launch_reduce_parts(const float* parts, int n_parts, size_t n, const float* in, size_t s_in,
                               float* out, size_t s_out, float lr, int commit, int groups, hipStream_t s) {
  if (n == 0 || groups <= 0) return hipSuccess;
  if (n_parts < 1 || (n & 3) != 0 || ((uintptr_t)parts & 15) != 0 || ((uintptr_t)out & 15) != 0 || (s_out & 3) != 0 ||
      (commit && (!in || ((uintptr_t)in & 15) != 0 || (s_in & 3) != 0)))
    return hipErrorInvalidValue;
  const size_t n4 = n / 4;
  const int blocks = onepass_blocks(n4);
  hipLaunchKernelGGL(reduce_parts_kernel, dim3(blocks, groups), dim3(kThreads), 0, s, parts, n_parts, n4, in, s_in,
                     out, s_out, lr, commit);
  return hipGetLastError();
}

// out[k][j] = in[k][j] - lr * grad[k][j];  acc[k][j] += grad[k][j]  (Alg. 2: update the replica and
// accumulate the gradient in one pass, 20 B/param)
__global__ void __launch_bounds__(kThreads)
commit_acc_kernel(const float* in, size_t in_stride, float* out, size_t stride, const float* __restrict__ grad,
                  size_t grad_stride, float* __restrict__ acc, size_t acc_stride, float lr, size_t P) {
  const size_t k = blockIdx.y;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < P; i += (size_t)gridDim.x * kThreads) {
    const float g = grad[k * grad_stride + i];
    out[k * stride + i] = in[k * in_stride + i] - lr * g;
    acc[k * acc_stride + i] += g;
  }
}

// The same on 16-byte vectors, one per lane (all four buffers 16-byte aligned, strides multiples
// of 4): three loads in flight per lane, every wave reads and writes 1 KiB contiguous per stream.
__global__ void __launch_bounds__(kThreads)
commit_acc4_kernel(const float* in, size_t in_stride, float* out, size_t stride, const float* __restrict__ grad,
                   size_t grad_stride, float* __restrict__ acc, size_t acc_stride, float lr, size_t n4, size_t P) {
  const size_t k = blockIdx.y;
  const f4v* in4 = reinterpret_cast<const f4v*>(in + k * in_stride);
  f4v* out4 = reinterpret_cast<f4v*>(out + k * stride);
  const f4v* g4 = reinterpret_cast<const f4v*>(grad + k * grad_stride);
  f4v* a4 = reinterpret_cast<f4v*>(acc + k * acc_stride);
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    const f4v g = __builtin_nontemporal_load(g4 + i);
    const f4v w = __builtin_nontemporal_load(in4 + i);
    const f4v a = __builtin_nontemporal_load(a4 + i);
    __builtin_nontemporal_store(w - g * lr, out4 + i);
    __builtin_nontemporal_store(a + g, a4 + i);
  }
  if (blockIdx.x == 0) {  // ragged tail
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) {
      const float g = grad[k * grad_stride + j];
      out[k * stride + j] = in[k * in_stride + j] - lr * g;
      acc[k * acc_stride + j] += g;
    }
  }
}

hipError_t launch_commit_acc(const float* in, size_t in_stride, float* out, size_t stride, const float* grad,
                             size_t grad_stride, float* acc, size_t acc_stride, float lr, int K, size_t P, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const bool vec = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)grad | (uintptr_t)acc) & 15) == 0) &&
                   ((in_stride | stride | grad_stride | acc_stride) & 3) == 0 && P >= 4;
  KernelTimer kt(KID_COMMIT_ACC, 20.0 * (double)P * K, s);
  if (vec) {
    const size_t n4 = P / 4;
    hipLaunchKernelGGL(commit_acc4_kernel, dim3(onepass_blocks(n4), K), dim3(kThreads), 0, s, in, in_stride, out, stride, grad,
                       grad_stride, acc, acc_stride, lr, n4, P);
    return hipGetLastError();
  }
  size_t blocks = (P + kThreads - 1) / kThreads;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(commit_acc_kernel, dim3((unsigned)blocks, K), dim3(kThreads), 0, s, in, in_stride, out, stride, grad,
                     grad_stride, acc, acc_stride, lr, P);
  return hipGetLastError();
}

// global[j] -= lr * (1/K) * sum_k acc_k[j], the sum in worker order (Eq. 1 as printed)
template <int KT>
__global__ void __launch_bounds__(kThreads)
merge_grad_kernel(float* global, PtrPack acc, int Krt, float scale, size_t n4, size_t P) {
  const int K = KT > 0 ? KT : Krt;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    f4v t = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(acc.p[0]) + i);
#pragma unroll
    for (int k = 1; k < K; ++k) t += __builtin_nontemporal_load(reinterpret_cast<const f4v*>(acc.p[k]) + i);
    const f4v g = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(global) + i);
    __builtin_nontemporal_store(g - t * scale, reinterpret_cast<f4v*>(global) + i);
  }
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < P) {
      float t = acc.p[0][j];
      for (int k = 1; k < K; ++k) t += acc.p[k][j];
      global[j] = global[j] - t * scale;
    }
  }
}

hipError_t launch_merge_grad(float* global, const PtrPack& accs, float lr, int K, size_t P, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t n4 = P / 4;
  const int blocks = onepass_blocks(n4);
  const float scale = lr / (float)K;
#define HPSGD_MG_CASE(KT) \
  hipLaunchKernelGGL(merge_grad_kernel<KT>, dim3(blocks), dim3(kThreads), 0, s, global, accs, K, scale, n4, P)
  switch (K) {
    case 1: HPSGD_MG_CASE(1); break;
    case 2: HPSGD_MG_CASE(2); break;
    case 4: HPSGD_MG_CASE(4); break;
    case 8: HPSGD_MG_CASE(8); break;
    case 16: HPSGD_MG_CASE(16); break;
    default: HPSGD_MG_CASE(0); break;
  }
#undef HPSGD_MG_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- fill
// p[g*stride + i] = 0 for i < n, g < groups; grid row `groups`, if launched, clears a second
// range extra[0 .. n_extra) instead
__global__ void __launch_bounds__(kThreads)
fill_zero_kernel(float* p, size_t n4, size_t n, size_t stride, int groups, float* extra, size_t n_extra) {
  float* pg = p + (size_t)blockIdx.y * stride;
  if ((int)blockIdx.y == groups) {
    pg = extra;
    n = n_extra;
    n4 = n_extra / 4;
  }
  const size_t step = (size_t)gridDim.x * kThreads;
  const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += step)
    reinterpret_cast<float4*>(pg)[i] = z;
  if (blockIdx.x == 0) {
    const size_t j = n4 * 4 + threadIdx.x;
    if (j < n) pg[j] = 0.f;
  }
}

// extra (nullable, 16-byte aligned): a second range of n_extra floats cleared by the same launch
hipError_t launch_fill_zero(float* p, size_t n, size_t stride, int groups, hipStream_t s, float* extra,
                            size_t n_extra) {
  if (n == 0 || groups == 0) {
    if (!extra || n_extra == 0) return hipSuccess;
    return launch_fill_zero(extra, n_extra, n_extra, 1, s, nullptr, 0);
  }
  if (extra && ((uintptr_t)extra & 15) != 0) return hipErrorInvalidValue;
  const size_t n4 = n / 4;
  const size_t big4 = (extra && n_extra / 4 > n4) ? n_extra / 4 : n4;
  int blocks = stream_blocks(big4);
  const int rows = groups + ((extra && n_extra) ? 1 : 0);
  if (blocks * rows > kMaxBlocks) blocks = (kMaxBlocks + rows - 1) / rows;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks, rows), dim3(kThreads), 0, s, p, n4, n, stride, groups, extra,
                     n_extra);
  return hipGetLastError();
}

// Several such clears in one launch (the h_0 slots and flag words a step clears before its first
// layer: each a few microseconds behind a launch); segment i owns grid columns blk0[i] .. blk0[i+1]-1.
// Segment: p[g*stride + r*ld + c] = 0 for r < rows, c < cols, g < its groups.
__global__ void __launch_bounds__(kThreads) fill_zero_multi_kernel(FillPack pk) {
  int sgi = 0;
#pragma unroll
  for (int i = 1; i < FillPack::MAXSEG; ++i)
    if (i < pk.n && blockIdx.x >= pk.blk0[i]) sgi = i;
  const FillSeg& sg = pk.seg[sgi];
  if ((int)blockIdx.y >= sg.groups) return;
  float* pg = sg.p + (size_t)blockIdx.y * sg.stride;
  const long n = (long)sg.rows * sg.cols;
  const unsigned nblk = pk.blk0[sgi + 1] - pk.blk0[sgi];
  for (long i = (long)(blockIdx.x - pk.blk0[sgi]) * kThreads + threadIdx.x; i < n; i += (long)nblk * kThreads)
    pg[(i / sg.cols) * sg.ld + i % sg.cols] = 0.f;
}

bool fill_pack_push(FillPack& pk, float* p, long ld, int rows, long cols, size_t stride, int groups) {
  if (pk.n >= FillPack::MAXSEG || !p || rows <= 0 || cols <= 0 || groups <= 0) return false;
  FillSeg& sg = pk.seg[pk.n];
  sg.p = p; sg.ld = ld; sg.rows = rows; sg.cols = cols; sg.stride = stride; sg.groups = groups;
  const long n = (long)rows * cols;
  long blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 64) blocks = 64;
  pk.blk0[pk.n + 1] = pk.blk0[pk.n] + (unsigned)blocks;
  if (groups > pk.max_groups) pk.max_groups = groups;
  ++pk.n;
  return true;
}

hipError_t launch_fill_pack(const FillPack& pk, hipStream_t s) {
  if (pk.n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_multi_kernel, dim3(pk.blk0[pk.n], pk.max_groups), dim3(kThreads), 0, s, pk);
  return hipGetLastError();
}

// p[g*stride + r*ld + c] = 0 for r < rows, c < cols: a column block of a row-major matrix
__global__ void __launch_bounds__(kThreads)
fill_zero_2d_kernel(float* p, long ld, int rows, int cols, size_t stride) {
  float* pg = p + (size_t)blockIdx.y * stride;
  const long n = (long)rows * cols;
  for (long i = (long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long)gridDim.x * kThreads)
    pg[(i / cols) * ld + i % cols] = 0.f;
}

hipError_t launch_fill_zero_2d(float* p, long ld, int rows, int cols, size_t stride, int groups,
                               hipStream_t s) {
  if (rows <= 0 || cols <= 0 || groups <= 0) return hipSuccess;
  const long n = (long)rows * cols;
  int blocks = (int)((n + kThreads - 1) / kThreads);
  if (blocks > 256) blocks = 256;
  hipLaunchKernelGGL(fill_zero_2d_kernel, dim3(blocks, groups), dim3(kThreads), 0, s, p, ld, rows, cols, stride);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- delay
// Ends when the 100 MHz wall clock has advanced by `ticks`: the wait is bounded by construction.
__global__ void __launch_bounds__(64) delay_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(32);
}

hipError_t launch_delay(unsigned us, hipStream_t s) {
  if (us == 0) return hipSuccess;
  hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, s, (long long)us * 100);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- gather
// out[(c*n_idx + b)*chunk ...] = shard[idx[b]*row + c*chunk ...], in 4-byte words.
__global__ void __launch_bounds__(kThreads)
gather_kernel(const uint32_t* __restrict__ shard, const int32_t* __restrict__ idx, int n_idx,
              size_t row_w, int n_chunks, size_t chunk_w, uint32_t* __restrict__ out) {
  const size_t b = blockIdx.x;           // sample
  const size_t c = blockIdx.y;           // chunk (time step)
  const uint32_t* src = shard + (size_t)idx[b] * row_w + c * chunk_w;
  uint32_t* dst = out + (c * (size_t)n_idx + b) * chunk_w;
  for (size_t w = threadIdx.x; w < chunk_w; w += kThreads) dst[w] = src[w];
}

// The same for K workers in one launch: worker k = blockIdx.z reads shard[k], idx[k], writes out[k].
struct GatherPack {
  const uint32_t* shard[HPSGD_KMAX];
  const int32_t* idx[HPSGD_KMAX];
  uint32_t* out[HPSGD_KMAX];
};

__global__ void __launch_bounds__(kThreads)
gather_all_kernel(GatherPack pk, int n_idx, size_t row_w, size_t chunk_w) {
  const size_t b = blockIdx.x, c = blockIdx.y;
  const int k = blockIdx.z;
  const uint32_t* src = pk.shard[k] + (size_t)pk.idx[k][b] * row_w + c * chunk_w;
  uint32_t* dst = pk.out[k] + (c * (size_t)n_idx + b) * chunk_w;
  for (size_t w = threadIdx.x; w < chunk_w; w += kThreads) dst[w] = src[w];
}

// Chunks of a few words (token ids, labels): one thread per output word instead of one
// workgroup per chunk.  Output word o = (c*n_idx + b)*chunk_w + w.
__global__ void __launch_bounds__(kThreads)
gather_all_small_kernel(GatherPack pk, int n_idx, size_t row_w, int n_chunks, size_t chunk_w) {
  const int k = blockIdx.y;
  const size_t total = (size_t)n_chunks * n_idx * chunk_w;
  const size_t o = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= total) return;
  const size_t w = o % chunk_w, cb = o / chunk_w;
  const size_t b = cb % n_idx, c = cb / n_idx;
  pk.out[k][o] = pk.shard[k][(size_t)pk.idx[k][b] * row_w + c * chunk_w + w];
}

hipError_t launch_gather_all(const void* const* shards, const int32_t* const* idx, int K, int n_idx,
                             size_t row_bytes, int n_chunks, size_t chunk_bytes, void* const* outs,
                             hipStream_t s) {
  if (K == 0 || n_idx == 0 || n_chunks == 0 || chunk_bytes == 0) return hipSuccess;
  GatherPack pk;
  for (int k = 0; k < K; ++k) {
    pk.shard[k] = (const uint32_t*)shards[k];
    pk.idx[k] = idx[k];
    pk.out[k] = (uint32_t*)outs[k];
  }
  if (chunk_bytes / 4 < 32) {
    const size_t total = (size_t)n_chunks * n_idx * (chunk_bytes / 4);
    hipLaunchKernelGGL(gather_all_small_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads), K),
                       dim3(kThreads), 0, s, pk, n_idx, row_bytes / 4, n_chunks, chunk_bytes / 4);
  } else {
    hipLaunchKernelGGL(gather_all_kernel, dim3(n_idx, n_chunks, K), dim3(kThreads), 0, s, pk, n_idx,
                       row_bytes / 4, chunk_bytes / 4);
  }
  return hipGetLastError();
}

hipError_t launch_gather(const void* shard, const int32_t* idx, int n_idx, size_t row_bytes,
                         int n_chunks, size_t chunk_bytes, void* out, hipStream_t s) {
  if (n_idx == 0 || n_chunks == 0 || chunk_bytes == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_kernel, dim3(n_idx, n_chunks), dim3(kThreads), 0, s,
                     (const uint32_t*)shard, idx, n_idx, row_bytes / 4, n_chunks, chunk_bytes / 4,
                     (uint32_t*)out);
  return hipGetLastError();
}

}  // namespace hpsgd
