// Wavefront-level kernels of the local training step: GRU cell forward and backward
// (gate nonlinearities, cell update, BPTT gate gradients), softmax cross-entropy, bias
// column sums, embedding lookup and its gradient.  The cell follows the convention
//   r = sigmoid(gx_r + gh_r), z = sigmoid(gx_z + gh_z), q = gh_n,
//   n = tanh(gx_n + r*q),     h = (1 - z)*n + z*h_prev
// with gx = W_ih x + b_ih and gh = W_hh h_prev + b_hh, gates stacked r, z, n.
#include "kernels.h"

namespace hpsgd {

static constexpr int kThreads = 256;

__device__ __forceinline__ float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

// ---------------------------------------------------------------------------- cell forward
__global__ void __launch_bounds__(kThreads)
gru_cell_fwd_kernel(const float* __restrict__ gx, long s_gx, const float* __restrict__ gh, long s_gh,
                    const float* __restrict__ h_prev, float* __restrict__ h, long s_h,
                    float* __restrict__ saved, long s_saved, int B, int H) {
  const int g = blockIdx.y;
  const int e = blockIdx.x * kThreads + threadIdx.x;  // element (b, j)
  if (e >= B * H) return;
  const int b = e / H, j = e - b * H;
  const float* gxr = gx + g * s_gx + (long)b * 3 * H;
  const float* ghr = gh + g * s_gh + (long)b * 3 * H;
  const float hp = h_prev[g * s_h + e];
  const float r = sigmoidf_(gxr[j] + ghr[j]);
  const float z = sigmoidf_(gxr[H + j] + ghr[H + j]);
  const float q = ghr[2 * H + j];
  const float n = tanhf(gxr[2 * H + j] + r * q);
  h[g * s_h + e] = (1.0f - z) * n + z * hp;
  float* sv = saved + g * s_saved + (long)b * 4 * H;
  sv[j] = r;
  sv[H + j] = z;
  sv[2 * H + j] = n;
  sv[3 * H + j] = q;
}

hipError_t launch_gru_cell_fwd(const float* gx, long s_gx, const float* gh, long s_gh,
                               const float* h_prev, float* h, long s_h, float* saved, long s_saved,
                               int B, int H, int groups, hipStream_t s) {
  dim3 grid((B * H + kThreads - 1) / kThreads, groups);
  hipLaunchKernelGGL(gru_cell_fwd_kernel, grid, dim3(kThreads), 0, s, gx, s_gx, gh, s_gh, h_prev, h,
                     s_h, saved, s_saved, B, H);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- cell backward
// dh = D + above;  dn = dh(1-z); dz = dh(h_prev - n); da_n = dn(1-n^2); dq = da_n r;
// da_r = da_n q r(1-r); da_z = dz z(1-z);  dgx = [da_r, da_z, da_n], dgh = [da_r, da_z, dq];
// D <- dh z  (the direct path to h_prev; the recurrent GEMM then adds dgh W_hh)
__global__ void __launch_bounds__(kThreads)
gru_cell_bwd_kernel(float* __restrict__ D, long s_D, const float* __restrict__ above, long s_above,
                    const float* __restrict__ saved, long s_saved, const float* __restrict__ h_prev,
                    long s_h, float* __restrict__ dgx, float* __restrict__ dgh, long s_dg, int B,
                    int H) {
  const int g = blockIdx.y;
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= B * H) return;
  const int b = e / H, j = e - b * H;
  float dh = D[g * s_D + e];
  if (above) dh += above[g * s_above + e];
  const float* sv = saved + g * s_saved + (long)b * 4 * H;
  const float r = sv[j], z = sv[H + j], n = sv[2 * H + j], q = sv[3 * H + j];
  const float hp = h_prev[g * s_h + e];
  const float dn = dh * (1.0f - z);
  const float dz = dh * (hp - n);
  const float da_n = dn * (1.0f - n * n);
  const float dq = da_n * r;
  const float da_r = da_n * q * r * (1.0f - r);
  const float da_z = dz * z * (1.0f - z);
  float* ox = dgx + g * s_dg + (long)b * 3 * H;
  float* oh = dgh + g * s_dg + (long)b * 3 * H;
  ox[j] = da_r;
  ox[H + j] = da_z;
  ox[2 * H + j] = da_n;
  oh[j] = da_r;
  oh[H + j] = da_z;
  oh[2 * H + j] = dq;
  D[g * s_D + e] = dh * z;
}

hipError_t launch_gru_cell_bwd(float* D, long s_D, const float* above, long s_above,
                               const float* saved, long s_saved, const float* h_prev, long s_h,
                               float* dgx, float* dgh, long s_dg, int B, int H, int groups,
                               hipStream_t s) {
  dim3 grid((B * H + kThreads - 1) / kThreads, groups);
  hipLaunchKernelGGL(gru_cell_bwd_kernel, grid, dim3(kThreads), 0, s, D, s_D, above, s_above, saved,
                     s_saved, h_prev, s_h, dgx, dgh, s_dg, B, H);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- softmax CE
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One workgroup per row.  Writes dlogits = (softmax - onehot)/N over the logits (in place
// when dlogits == logits) and the row's loss -log softmax[y].
__global__ void __launch_bounds__(kThreads)
softmax_ce_kernel(const float* logits, long s_logits, const int32_t* __restrict__ y, long s_y,
                  float* dlogits, float* __restrict__ rowloss, long s_rowloss, int N, int C) {
  __shared__ float red[kThreads / 64];
  __shared__ float bcast;
  const int g = blockIdx.y, row = blockIdx.x;
  const float* lr = logits + g * s_logits + (long)row * C;
  float* dr = dlogits + g * s_logits + (long)row * C;
  const int label = y[g * s_y + row];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  float m = -INFINITY;
  for (int c = tid; c < C; c += kThreads) m = fmaxf(m, lr[c]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  if (tid == 0) {
    float v = red[0];
    for (int w = 1; w < kThreads / 64; ++w) v = fmaxf(v, red[w]);
    bcast = v;
  }
  __syncthreads();
  m = bcast;
  __syncthreads();

  float sum = 0.f;
  for (int c = tid; c < C; c += kThreads) sum += expf(lr[c] - m);
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float v = red[0];
    for (int w = 1; w < kThreads / 64; ++w) v += red[w];
    bcast = v;
  }
  __syncthreads();
  sum = bcast;

  const float inv_sum = 1.0f / sum;
  const float inv_n = 1.0f / (float)N;
  if (tid == 0) rowloss[g * s_rowloss + row] = -((lr[label] - m) - logf(sum));
  __syncthreads();  // the label logit is read before it is overwritten
  for (int c = tid; c < C; c += kThreads) {
    const float p = expf(lr[c] - m) * inv_sum;
    dr[c] = (p - (c == label ? 1.0f : 0.0f)) * inv_n;
  }
}

hipError_t launch_softmax_ce(const float* logits, long s_logits, const int32_t* y, long s_y,
                             float* dlogits, float* rowloss, long s_rowloss, int N, int C,
                             int groups, hipStream_t s) {
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(N, groups), dim3(kThreads), 0, s, logits, s_logits, y,
                     s_y, dlogits, rowloss, s_rowloss, N, C);
  return hipGetLastError();
}

// loss[g] = mean of the row losses; one workgroup per group, fixed summation order.
__global__ void __launch_bounds__(kThreads)
loss_mean_kernel(const float* __restrict__ rowloss, long s_rowloss, float* __restrict__ loss, int N) {
  __shared__ float red[kThreads];
  const int g = blockIdx.x, tid = threadIdx.x;
  float v = 0.f;
  for (int i = tid; i < N; i += kThreads) v += rowloss[g * s_rowloss + i];
  red[tid] = v;
  __syncthreads();
  for (int o = kThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) loss[g] = red[0] / (float)N;
}

hipError_t launch_loss_mean(const float* rowloss, long s_rowloss, float* loss, int N, int groups,
                            hipStream_t s) {
  hipLaunchKernelGGL(loss_mean_kernel, dim3(groups), dim3(kThreads), 0, s, rowloss, s_rowloss, loss, N);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- column sums
// out[n] = sum_r in[r][n].  A workgroup of 1024 threads covers 64 columns with 16 row slices
// (slice s takes rows s, s+16, ...); the slices are combined through LDS in a fixed order.
static constexpr int kColsumSlices = 16;

__global__ void __launch_bounds__(64 * kColsumSlices)
colsum_kernel(const float* __restrict__ in, long ld, long s_in, float* __restrict__ out, long s_out,
              int R, int N) {
  __shared__ float red[kColsumSlices][64];
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.x * 64 + lane;
  const int slice = threadIdx.x >> 6;
  float a0 = 0.f, a1 = 0.f;
  if (c < N) {
    const float* p = in + g * s_in + c;
    int r = slice;
    for (; r + kColsumSlices < R; r += 2 * kColsumSlices) {
      a0 += p[(long)r * ld];
      a1 += p[(long)(r + kColsumSlices) * ld];
    }
    if (r < R) a0 += p[(long)r * ld];
  }
  red[slice][lane] = a0 + a1;
  __syncthreads();
  if (slice == 0 && c < N) {
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < kColsumSlices; ++i) v += red[i][lane];
    out[g * s_out + c] = v;
  }
}

// Column sums of several matrices in one launch (the bias gradients of all MLP layers: each is a
// few microseconds of work behind a launch); segment i owns grid columns blk0[i] .. blk0[i+1]-1.
// With b_in the sum is applied at once: out = b_in - lr * sum; without, out = scale * sum (a mean
// of per-row losses is a column sum of an R x 1 matrix scaled by 1 / R).
__global__ void __launch_bounds__(64 * kColsumSlices) colsum_multi_kernel(ColsumPack pk) {
  __shared__ float red[kColsumSlices][64];
  int sgi = 0;
#pragma unroll
  for (int i = 1; i < ColsumPack::MAXSEG; ++i)
    if (i < pk.n && blockIdx.x >= pk.blk0[i]) sgi = i;
  const ColsumSeg& sg = pk.seg[sgi];
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int c = (blockIdx.x - pk.blk0[sgi]) * 64 + lane;
  const int slice = threadIdx.x >> 6;
  float a0 = 0.f, a1 = 0.f;
  if (c < sg.N) {
    const float* p = sg.in + g * sg.s_in + c;
    int r = slice;
    for (; r + kColsumSlices < sg.R; r += 2 * kColsumSlices) {
      a0 += p[(long)r * sg.ld];
      a1 += p[(long)(r + kColsumSlices) * sg.ld];
    }
    if (r < sg.R) a0 += p[(long)r * sg.ld];
  }
  red[slice][lane] = a0 + a1;
  __syncthreads();
  if (slice == 0 && c < sg.N) {
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < kColsumSlices; ++i) v += red[i][lane];
    sg.out[g * sg.s_out + c] = sg.b_in ? sg.b_in[g * sg.s_bin + c] - pk.lr * v : v * sg.scale;
  }
}

bool colsum_pack_push(ColsumPack& pk, const float* in, long ld, long s_in, float* out, long s_out, const float* b_in,
                      long s_bin, int R, int N, float scale) {
  if (pk.n >= ColsumPack::MAXSEG || N <= 0 || R <= 0) return false;
  ColsumSeg& sg = pk.seg[pk.n];
  sg.in = in; sg.ld = ld; sg.s_in = s_in; sg.out = out; sg.s_out = s_out; sg.b_in = b_in; sg.s_bin = s_bin;
  sg.R = R; sg.N = N; sg.scale = scale;
  pk.blk0[pk.n + 1] = pk.blk0[pk.n] + (unsigned)((N + 63) / 64);
  ++pk.n;
  return true;
}

hipError_t launch_colsum_pack(const ColsumPack& pk, int groups, hipStream_t s) {
  if (pk.n == 0 || groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(colsum_multi_kernel, dim3(pk.blk0[pk.n], groups), dim3(64 * kColsumSlices), 0, s, pk);
  return hipGetLastError();
}

hipError_t launch_colsum(const float* in, long ld, long s_in, float* out, long s_out, int R, int N,
                         int groups, hipStream_t s) {
  hipLaunchKernelGGL(colsum_kernel, dim3((N + 63) / 64, groups), dim3(64 * kColsumSlices), 0, s, in,
                     ld, s_in, out, s_out, R, N);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- embedding
__global__ void __launch_bounds__(64)
embed_fwd_kernel(const float* __restrict__ E, long s_E, const int32_t* __restrict__ tok, long s_tok,
                 float* __restrict__ out, long s_out, int Ew) {
  const int g = blockIdx.y, i = blockIdx.x;
  const float* src = E + g * s_E + (long)tok[g * s_tok + i] * Ew;
  float* dst = out + g * s_out + (long)i * Ew;
  for (int c = threadIdx.x; c < Ew; c += 64) dst[c] = src[c];
}

hipError_t launch_embed_fwd(const float* E, long s_E, const int32_t* tok, long s_tok, float* out,
                            long s_out, int N, int Ew, int groups, hipStream_t s) {
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(N, groups), dim3(64), 0, s, E, s_E, tok, s_tok, out,
                     s_out, Ew);
  return hipGetLastError();
}

// One workgroup per position i.  It acts only if i is the first occurrence of its token v;
// it then adds, in increasing position, the rows of every position that holds v (thread c
// owns column c).  No atomics: duplicate ids, frequent under a Zipf draw, cost the owner a
// short serial loop instead of contention, and the order of the sum is fixed.
// E_in != nullptr: the owner writes the updated row E_in[v] - lr * sum to dE[v] instead of the sum
// (dE is then the embedding of the output replica; only the rows of tokens that occur are
// touched, so for an update in place nothing else has to be read or written).
__global__ void __launch_bounds__(kThreads)
embed_bwd_kernel(const float* __restrict__ dx, long s_dx, const int32_t* __restrict__ tok,
                 long s_tok, float* dE, long s_dE, int N, int Ew, const float* E_in, long s_E, float lr) {
  __shared__ int list[kThreads];  // positions of this chunk that hold v, ascending
  __shared__ int wcnt[kThreads / 64];
  const int g = blockIdx.y, i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* tk = tok + g * s_tok;
  const int v = tk[i];
  int seen = 0;
  for (int j = tid; j < i; j += kThreads) seen |= (tk[j] == v);
  if (__syncthreads_or(seen)) return;
  const float* src = dx + g * s_dx;
  float* dst = dE + g * s_dE + (long)v * Ew;
  for (int c0 = 0; c0 < Ew; c0 += kThreads) {
    const int c = c0 + tid;
    const bool cok = c < Ew;
    float acc = 0.f;
    for (int j0 = i; j0 < N; j0 += kThreads) {
      // compact the matching positions of this chunk (order preserved)
      const int j = j0 + tid;
      const bool m = j < N && tk[j] == v;
      const unsigned long long mask = __ballot(m);
      if (lane == 0) wcnt[wave] = __popcll(mask);
      __syncthreads();
      int base = 0, n = 0;
#pragma unroll
      for (int w = 0; w < kThreads / 64; ++w) {
        if (w < wave) base += wcnt[w];
        n += wcnt[w];
      }
      if (m) list[base + __popcll(mask & ((1ull << lane) - 1ull))] = j;
      __syncthreads();
      // rows are fetched eight at a time (independent loads) and added in position order
      if (cok) {
        int k = 0;
        for (; k + 8 <= n; k += 8) {
          float r[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) r[u] = src[(long)list[k + u] * Ew + c];
#pragma unroll
          for (int u = 0; u < 8; ++u) acc += r[u];
        }
        for (; k < n; ++k) acc += src[(long)list[k] * Ew + c];
      }
      __syncthreads();
    }
    if (cok) dst[c] = E_in ? E_in[g * s_E + (long)v * Ew + c] - lr * acc : acc;
  }
}

hipError_t launch_embed_bwd(const float* dx, long s_dx, const int32_t* tok, long s_tok, float* dE,
                            long s_dE, int N, int Ew, int groups, hipStream_t s, const float* E_in, long s_E,
                            float lr) {
  hipLaunchKernelGGL(embed_bwd_kernel, dim3(N, groups), dim3(kThreads), 0, s, dx, s_dx, tok, s_tok, dE,
                     s_dE, N, Ew, E_in, s_E, lr);
  return hipGetLastError();
}

}  // namespace hpsgd
