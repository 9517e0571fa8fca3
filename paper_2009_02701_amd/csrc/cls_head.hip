// The head of a classifier with few classes in two small launches per local step (fp32):
//   logits = feats W^T + b;  loss = mean cross-entropy;  dlogits = (softmax - onehot) / N;
//   dfeat = dlogits W;  dW = dlogits^T feats;  db = column sums of dlogits;
//   then either the SGD update (W_out = W_in - lr dW, b_out = b_in - lr db) or the gradients.
// With N <= 128 rows and C <= 32 classes each of the three products is a fraction of a
// megaflop per worker: as three GEMM launches, two reductions, a softmax and a loss launch
// they cost seven launch gaps and little else.  Here the forward part is cut over the rows
// (8 rows per workgroup, 32 threads per row share a dot product) and the backward part over
// the feature columns (64 per workgroup), so that a worker's head is spread over 16 CUs (a
// single workgroup per worker with everything in LDS was measured at ~95 us: bound by one
// CU's LDS rate).  Every sum runs in a fixed order.
#include <cmath>

#include "kernels.h"

namespace hpsgd {

namespace {

constexpr int HMAXC = 32;     // classes
constexpr int HMAXN = 128;    // rows
constexpr int HROWS = 8;      // rows per workgroup, forward
constexpr int HCOLS = 64;     // feature columns per workgroup, backward

// Trips 0 .. n-1 of a copy loop, U at a time: the U loads go out before the first value is used
// (a load whose value is stored at once waits out the memory latency on every trip).
template <int U, typename Load, typename Store>
__device__ __forceinline__ void batched_copy(int n, Load load, Store store) {
  for (int base = 0; base < n; base += U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load(min(base + u, n - 1));
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + u < n) store(base + u, v[u]);
  }
}

// grid (ceil(N / 8), groups), 256 threads: thread t works for row t / 32 of the slice on the
// contraction indices t % 32, + 32, ...
template <int CPAD>  // classes rounded up to 8, 16 or 32: the rows of W beyond C are zero in LDS, so that
                     // the inner loops carry no guards (a guard per class keeps the LDS reads from being batched)
__global__ void __launch_bounds__(256)
cls_head_fwd_kernel(const float* __restrict__ feats, long s_feats, const float* __restrict__ W,
                    const float* __restrict__ b, long s_in, const int32_t* __restrict__ y, long s_y,
                    float* __restrict__ dlog, long s_dlog, float* __restrict__ rowloss, long s_rowloss, int N, int C,
                    int H) {
  extern __shared__ __attribute__((aligned(16))) float head_lds[];
  float* sW = head_lds;  // [CPAD][H]
  const int g = blockIdx.y, tid = threadIdx.x;
  const int part = tid & 31, row = blockIdx.x * HROWS + (tid >> 5);
  const int rowc = min(row, N - 1);
  const float* Wg = W + g * s_in;
  const int nW = C * H;
  const float* fr = feats + g * s_feats + (long)rowc * H;
  const int nk = (H - part + 31) / 32;  // this thread's share of the row: k = part + 32 i < H
  // the first 8 values of the row are requested before W is copied, so that they arrive with it
  float f[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) f[u] = fr[part + 32 * min(u, nk - 1)];
  batched_copy<24>((nW + 255) / 256, [&](int i) { return Wg[min(tid + 256 * i, nW - 1)]; },
                   [&](int i, float v) {
                     if (tid + 256 * i < nW) sW[tid + 256 * i] = v;
                   });
  for (int i = nW + tid; i < CPAD * H; i += 256) sW[i] = 0.f;
  float acc[CPAD];
#pragma unroll
  for (int c = 0; c < CPAD; ++c) acc[c] = 0.f;
  __syncthreads();
  for (int base = 0; base < nk; base += 8) {
    if (base > 0) {
#pragma unroll
      for (int u = 0; u < 8; ++u) f[u] = fr[part + 32 * min(base + u, nk - 1)];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (base + u < nk) {
        const int k = part + 32 * (base + u);
#pragma unroll
        for (int c = 0; c < CPAD; ++c) acc[c] += f[u] * sW[c * H + k];
      }
  }
  // the 32 partial sums of a row: butterfly inside its half of the wave
#pragma unroll
  for (int c = 0; c < CPAD; ++c) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) acc[c] += __shfl_xor(acc[c], o);
  }
  if (part == 0 && row < N) {
    const float* bg = b + g * s_in;
    const int label = y[g * s_y + row];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < CPAD; ++c)
      if (c < C) {
        acc[c] += bg[c];
        m = fmaxf(m, acc[c]);
      }
    float sum = 0.f, zl = 0.f;
#pragma unroll
    for (int c = 0; c < CPAD; ++c)
      if (c < C) {
        if (c == label) zl = acc[c];
        acc[c] = expf(acc[c] - m);
        sum += acc[c];
      }
    rowloss[g * s_rowloss + row] = -((zl - m) - logf(sum));
    const float inv_sum = 1.0f / sum, inv_n = 1.0f / (float)N;
    float* dr = dlog + g * s_dlog + (long)row * C;
#pragma unroll
    for (int c = 0; c < CPAD; ++c)
      if (c < C) dr[c] = (acc[c] * inv_sum - (c == label ? 1.0f : 0.0f)) * inv_n;
  }
}

// grid (ceil(H / 64), groups), 256 threads: thread t owns column t % 64 of the slice
__global__ void __launch_bounds__(256)
cls_head_bwd_kernel(const float* __restrict__ feats, long s_feats, const float* W_in, const float* b_in, long s_in,
                    const float* __restrict__ dlog, long s_dlog, const float* __restrict__ rowloss, long s_rowloss,
                    float* __restrict__ dfeat, long s_dfeat, float* W_out, float* b_out, long s_out, float lr,
                    int commit, float* __restrict__ loss, int N, int C, int H, int relu_mask) {
  __shared__ float sD[HMAXN * HMAXC];          // dlogits [N][C]
  __shared__ float sF[HMAXN][HCOLS + 1];       // the slice of the features
  __shared__ float sW[HMAXC][HCOLS + 1];       // the slice of W
  const int g = blockIdx.y, tid = threadIdx.x;
  const int jl = tid & 63, q = tid >> 6, j = blockIdx.x * HCOLS + jl;
  const bool jv = j < H;
  const int jc = jv ? j : 0;
  const int nD = N * C;
  // the slice of W (at most 8 values per thread) and the first 1024 logit gradients are requested
  // first and stored last: they arrive while the features are copied
  const int nWq = (C - q + 3) / 4;
  float wv[HMAXC / 4], dv[4];
#pragma unroll
  for (int u = 0; u < HMAXC / 4; ++u) wv[u] = W_in[g * s_in + (long)min(q + 4 * u, C - 1) * H + jc];
#pragma unroll
  for (int u = 0; u < 4; ++u) dv[u] = dlog[g * s_dlog + min(tid + 256 * u, nD - 1)];
  batched_copy<16>((N - q + 3) / 4, [&](int i) { return feats[g * s_feats + (long)(q + 4 * i) * H + jc]; },
                   [&](int i, float v) { sF[q + 4 * i][jl] = v; });
#pragma unroll
  for (int u = 0; u < HMAXC / 4; ++u)
    if (u < nWq) sW[q + 4 * u][jl] = wv[u];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (tid + 256 * u < nD) sD[tid + 256 * u] = dv[u];
  if (nD > 1024)
    batched_copy<4>((nD - 1024 + 255) / 256, [&](int i) { return dlog[g * s_dlog + min(1024 + tid + 256 * i, nD - 1)]; },
                    [&](int i, float v) {
                      if (1024 + tid + 256 * i < nD) sD[1024 + tid + 256 * i] = v;
                    });
  __syncthreads();
  for (int r = q; r < N; r += 4) {
    float a = 0.f;
    for (int c = 0; c < C; ++c) a += sD[r * C + c] * sW[c][jl];
    // the features are the output of a ReLU layer: the gradient passes where the feature is positive
    if (relu_mask && !(sF[r][jl] > 0.f)) a = 0.f;
    if (jv) dfeat[g * s_dfeat + (long)r * H + j] = a;
  }
  for (int c = q; c < C; c += 4) {
    float a0 = 0.f, a1 = 0.f;
    int r = 0;
    for (; r + 1 < N; r += 2) {
      a0 += sD[r * C + c] * sF[r][jl];
      a1 += sD[(r + 1) * C + c] * sF[r + 1][jl];
    }
    if (r < N) a0 += sD[r * C + c] * sF[r][jl];
    const float dw = a0 + a1;
    if (jv) W_out[g * s_out + (long)c * H + j] = commit ? sW[c][jl] - lr * dw : dw;
  }
  if (blockIdx.x == 0) {
    if (tid < C) {
      float a = 0.f;
      for (int r = 0; r < N; ++r) a += sD[r * C + tid];
      b_out[g * s_out + tid] = commit ? b_in[g * s_in + tid] - lr * a : a;
    }
    if (tid == 64 && loss) {
      float v = 0.f;
      for (int r = 0; r < N; ++r) v += rowloss[g * s_rowloss + r];
      loss[g] = v / (float)N;
    }
  }
}

}  // namespace

bool cls_head_supported(int N, int C, int H) {
  const int cpad = C <= 8 ? 8 : C <= 16 ? 16 : 32;
  return N >= 1 && N <= HMAXN && C >= 2 && C <= HMAXC && H >= 1 && (size_t)cpad * H * sizeof(float) <= 128 * 1024;
}

// feats: [groups][N][H] (stride s_feats); W_in / b_in: the head's parameters in the input replicas
// (stride s_in); dlog ([N][C] per group, stride s_dlog) and rowloss ([N] per group) are scratch
// that the first launch hands to the second; dfeat: [N][H] per group (stride s_dfeat);
// commit != 0: W_out / b_out (stride s_out, may be W_in / b_in) receive the updated parameters,
// else the gradients; loss: per group mean cross-entropy, or nullptr.  relu_mask != 0: the features
// are the output of a ReLU layer and dfeat is the gradient in front of that ReLU (zero where the
// feature is not positive).
hipError_t launch_cls_head(const float* feats, long s_feats, const float* W_in, const float* b_in, long s_in,
                           const int32_t* y, long s_y, float* dlog, long s_dlog, float* rowloss, long s_rowloss,
                           float* dfeat, long s_dfeat, float* W_out, float* b_out, long s_out, float lr, int commit,
                           float* loss, int N, int C, int H, int groups, hipStream_t s, int relu_mask) {
  if (!cls_head_supported(N, C, H)) return hipErrorInvalidValue;
  const int cpad = C <= 8 ? 8 : C <= 16 ? 16 : 32;
  const size_t lds = (size_t)cpad * H * sizeof(float);
#define HPSGD_HEAD_FWD(CP)                                                                                         \
  do {                                                                                                             \
    static size_t allowed = 0;                                                                                     \
    if (lds > allowed && lds > 64 * 1024) {                                                                        \
      hipError_t e_ = hipFuncSetAttribute((const void*)cls_head_fwd_kernel<CP>,                                    \
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                  \
      if (e_ != hipSuccess) return e_;                                                                             \
      allowed = lds;                                                                                               \
    }                                                                                                              \
    hipLaunchKernelGGL(cls_head_fwd_kernel<CP>, dim3((N + HROWS - 1) / HROWS, groups), dim3(256), lds, s, feats,   \
                       s_feats, W_in, b_in, s_in, y, s_y, dlog, s_dlog, rowloss, s_rowloss, N, C, H);               \
  } while (0)
  if (cpad == 8) HPSGD_HEAD_FWD(8);
  else if (cpad == 16) HPSGD_HEAD_FWD(16);
  else HPSGD_HEAD_FWD(32);
#undef HPSGD_HEAD_FWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cls_head_bwd_kernel, dim3((H + HCOLS - 1) / HCOLS, groups), dim3(256), 0, s, feats, s_feats,
                     W_in, b_in, s_in, dlog, s_dlog, rowloss, s_rowloss, dfeat, s_dfeat, W_out, b_out, s_out, lr,
                     commit, loss, N, C, H, relu_mask);
  return hipGetLastError();
}

}  // namespace hpsgd
