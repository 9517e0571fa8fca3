// Fused recurrent kernels: one launch per time step does the recurrent GEMM on the matrix
// cores AND the elementwise cell math in its epilogue, so neither gh_t nor dh_t ever goes
// through HBM and the per-step launch count drops from two to one.
//
// Forward, step t:   gh = h_{t-1} W_hh^T (+ b_hh);  r, z, n, h_t from gx_t, gh, h_{t-1}.
// Backward, step t:  dh_t = dgh_{t+1} W_hh + dh_{t+1} * z_{t+1} (+ gradient from above);
//                    gate gradients of step t from dh_t and the saved r, z, n, q.
//
// Tiling (64-lane waves, v_mfma_f32_16x16x4_f32): a workgroup of 4 waves owns 32 batch rows
// x 16 hidden units (all three gates of those units in the forward kernel, so the epilogue
// has r, z and n of a unit in one thread).  The contraction is split over the 4 waves in
// 16-wide chunks (chunk c belongs to wave c % 4); partial sums are combined through LDS.
// MFMA 16x16x4 lane layout: A lane l holds A[m = l%16][k = l/16], B lane l holds
// B[k = l/16][n = l%16], accumulator register v holds C[4*(l/16) + v][l%16].  Because the
// order of the contraction index is free as long as both operands agree, a lane fetches one
// float4 (4 consecutive k of its row) per operand and feeds component s to MFMA number s:
// lane group g then covers k = 16c + 4g + s, so operand fragments are 16-byte reads.
#include "kernels.h"

namespace hpsgd {

typedef float floatx4 __attribute__((ext_vector_type(4)));

static constexpr int FR = 32;   // batch rows per workgroup
static constexpr int FJ = 16;   // hidden units per workgroup

__device__ __forceinline__ float sigm(float a) { return 1.0f / (1.0f + expf(-a)); }

__device__ __forceinline__ float4 ld4_or_zero(const float* p, bool ok) {
  return ok ? *reinterpret_cast<const float4*>(p) : make_float4(0.f, 0.f, 0.f, 0.f);
}

__device__ __forceinline__ floatx4 mfma4(const float4& a, const float4& b, floatx4 acc) {
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc, 0, 0, 0);
  return acc;
}

// Workgroups are dispatched to the 8 XCDs round-robin (workgroup i runs on XCD i % 8) and
// each XCD has its own L2, which starts cold at every launch.  The linear id is therefore
// mapped to (worker g, unit tile x, row tile y) so that one XCD touches as few distinct
// weight slices and activation rows as possible: whole workers per XCD when there are at
// least 8 of them, else a contiguous range of a worker's unit tiles (with all its row tiles).
__device__ __forceinline__ void step_tile(int NJ, int RT, int groups, int& g, int& x, int& y) {
  const int i = blockIdx.x;
  if (groups % 8 == 0) {
    const int c = i & 7, li = i >> 3, per = NJ * RT;
    g = c + 8 * (li / per);
    const int r = li % per;
    x = r % NJ;
    y = r / NJ;
  } else if (8 % groups == 0 && NJ % (8 / groups) == 0) {
    const int s = 8 / groups, c = i & 7, li = i >> 3, xs = NJ / s;
    g = c / s;
    x = (c % s) * xs + li % xs;
    y = li / xs;
  } else {
    x = i % NJ;
    y = (i / NJ) % RT;
    g = i / (NJ * RT);
  }
}

// ---------------------------------------------------------------------------- fp32 step kernels
// Operands take the path global -> registers -> LDS -> MFMA layout: the workgroup fetches
// 64- or 128-wide slabs of its weight rows and activation rows with fully contiguous loads (one
// wave instruction = whole 256- or 512-byte row segments; LDS row pitch = slab width + 4 words,
// so that 16 rows x 16-byte reads hit all 64 banks).  Loading straight into the MFMA layout
// would need 16 row pieces of 64 bytes per instruction, which a fresh launch with a cold L2
// serves about 1.7x slower.
// acc[rb][q] += sum_k A[rb*16 + ..][k] * W_q[..][k].  Wbase points at the workgroup's first
// weight row, gate block q starts w_qstride floats further, rows are KD floats apart;
// Abase at its first activation row (rows >= rows_valid read as zero).
// BF16: the rows hold bf16 pairs; all sizes (w_qstride, KD) are then counted in 4-byte words
// (two bf16 each), the data movement is the same byte for byte, and one 16-byte fragment
// feeds a single v_mfma_f32_16x16x32_bf16 (lane l: k = 32c + 8*(l/16) .. +7).
//
// The contraction as a rolling pipeline: 64-word slabs, the loads of slab s+3 are issued
// while slab s is multiplied, so the wave never sits behind a long burst of load instructions
// (a CU accepts only ~64 bytes of vector loads per clock: issuing a workgroup's whole operand
// set up front keeps its waves busy issuing for microseconds before the first MFMA).
// Registers hold 4 slabs in flight; LDS holds 2 (one barrier per slab).  lds: 2*RT*68 words.
// RB: 16-row blocks of activations per workgroup.  NW: waves per workgroup, 4 or 8.  The
// contraction index of a slab is always split four ways (wave & 3 takes the 16-word chunks
// wave & 3, + 4, ..); with 8 waves the two halves of the workgroup take one row block each, so
// every SIMD holds two waves and one's LDS and barrier latency hides behind the other's MFMAs
// without loading anything twice.  W: slab width in words (64 or 128; lds: 2*RT*(W+4) words).
template <int NQ, bool BF16, int RB = 2, int NW = 4, int W = 64>
__device__ __forceinline__ void rolling_contraction(const float* __restrict__ Wbase, long w_qstride,
                                                    const float* __restrict__ Abase, int KD,
                                                    int rows_valid, float* __restrict__ lds,
                                                    floatx4 (&acc)[RB * 4 / NW][NQ]) {
  constexpr int NT = 64 * NW, RBW = RB * 4 / NW, NC = W / 64;
  constexpr int RT = 16 * NQ + 16 * RB, UR = W / 4, UPT = RT * UR / NT, P = W + 4;
  constexpr int PD = 3, RS = PD + 1;  // prefetch distance in slabs, register sets
  static_assert(RT * UR % NT == 0 && RB * 4 % NW == 0 && (W == 64 || W == 128), "slab shape");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, rsel = wave >> 2;
  const int lr = lane & 15, lg = lane >> 4;
  const int nslab = (KD + W - 1) / W;
  const float* rowp[UPT];
  bool rowok[UPT];
#pragma unroll
  for (int i = 0; i < UPT; ++i) {
    const int row = (tid + i * NT) / UR;
    if (row < 16 * NQ) {
      rowp[i] = Wbase + (row >> 4) * w_qstride + (long)(row & 15) * KD;
      rowok[i] = true;
    } else {
      const int ar = row - 16 * NQ;
      rowok[i] = ar < rows_valid;
      rowp[i] = Abase + (long)(rowok[i] ? ar : 0) * KD;
    }
  }
  const int colofs = (tid % UR) << 2;
  float4 regs[RS][UPT];
  bool cok[RS];
  // branch-free (a conditional around a load makes the compiler wait for every outstanding
  // load before the first use): a unit beyond KD (a whole slab past the end, or the ragged
  // tail of the last one) is zeroed at the LDS store; its load still happens, from one
  // address for all lanes (a single cache line: next to nothing of the CU's load bandwidth)
  auto issue = [&](int set, int slab) {
    const int col = slab * W + colofs;
    cok[set] = col < KD;  // KD is a multiple of 16: a float4 is all in or all out
#pragma unroll
    for (int i = 0; i < UPT; ++i)
      regs[set][i] = *reinterpret_cast<const float4*>(cok[set] ? rowp[i] + col : Wbase);
  };
  auto sstore = [&](int set, int buf) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int u = tid + i * NT;
      const bool ok = cok[set] && rowok[i];
      const float4 v = regs[set][i];  // (selected per component: a select between two float4
                                      // objects would keep the whole register array in memory)
      *reinterpret_cast<float4*>(&lds[(buf * RT + u / UR) * P + ((u % UR) << 2)]) =
          make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
    }
  };
#pragma unroll
  for (int u = 0; u < PD; ++u) issue(u, u);
  for (int s0 = 0; s0 < nslab; s0 += RS) {
#pragma unroll
    for (int u = 0; u < RS; ++u) {  // slab s0 + u: register set u, LDS buffer u & 1
      const int b = u & 1;
      // the fences keep the compiler from sinking the loads below the MFMAs or hoisting the
      // zeroing selects of the next store (which wait for their loads) above them
      __builtin_amdgcn_sched_barrier(0);
      sstore(u, b);  // waits for this slab only: the later ones stay in flight
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      issue((u + PD) % RS, s0 + u + PD);  // into the set stored one slab ago
#pragma unroll
      for (int ci = 0; ci < NC; ++ci) {
        const int kcol = 16 * (kw + 4 * ci) + 4 * lg;
        float4 a[RBW], w[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q)
          w[q] = *reinterpret_cast<const float4*>(&lds[(b * RT + q * 16 + lr) * P + kcol]);
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb)
          a[rb] = *reinterpret_cast<const float4*>(
              &lds[(b * RT + 16 * NQ + (rsel * RBW + rb) * 16 + lr) * P + kcol]);
        if (BF16) {
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
              typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
              acc[rb][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[rb]),
                                                                   __builtin_bit_cast(bf16x8_t, w[q]),
                                                                   acc[rb][q], 0, 0, 0);
            }
        } else {
          // the four contraction steps outermost: consecutive MFMAs update different
          // accumulators; every accumulator still receives its steps in order
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
              for (int q = 0; q < NQ; ++q) {
                const float av = e == 0 ? a[rb].x : e == 1 ? a[rb].y : e == 2 ? a[rb].z : a[rb].w;
                const float wv = e == 0 ? w[q].x : e == 1 ? w[q].y : e == 2 ? w[q].z : w[q].w;
                acc[rb][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, wv, acc[rb][q], 0, 0, 0);
              }
        }
      }
    }
  }
  __syncthreads();  // the LDS buffers may be reused by the caller
}

// Forward step: h_out = cell(gx_t, h_prev W_hh^T + b_hh, h_prev); saves r|z|n|q of the step.
template <int RB, int NW, int W>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, 2)))
gru_fwd_step_kernel(const float* __restrict__ W_hh, const float* __restrict__ b_hh, long s_rep,
                           const float* __restrict__ gx_t, long s_gx, const float* __restrict__ h_prev,
                           float* __restrict__ h_out, long s_hs, float* __restrict__ sv_t, long s_sv,
                           int B, int H, int groups) {
  extern __shared__ __attribute__((aligned(16))) float staged_lds[];
  float* red = staged_lds;  // [4][3 * RB][4][64], over the slab buffers once the contraction is done
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, rsel = wave >> 2;
  constexpr int RBW = RB * 4 / NW;  // row blocks per wave
  // the recurrence is the critical path: its waves issue ahead of any throughput kernel
  // (weight-gradient GEMMs, merge) that shares the SIMD
  __builtin_amdgcn_s_setprio(3);
  const int lr = lane & 15, lg = lane >> 4;
  int g, tx, ty;
  constexpr int FRB = 16 * RB;  // batch rows per workgroup
  step_tile(H / FJ, (B + FRB - 1) / FRB, groups, g, tx, ty);
  const int j0 = tx * FJ, r0 = ty * FRB;
  const float* hp = h_prev + g * s_hs;
  // the epilogue's own inputs first: they arrive during the matrix work
  const float* bh = b_hh + g * s_rep;
  const int j = j0 + lr;
  float gxv[RBW][3], hpv[RBW], bias[3];
#pragma unroll
  for (int q = 0; q < 3; ++q) bias[q] = bh[q * H + j];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    // unconditional loads from a row clamped into the batch (a select on a loaded value
    // would make the wave wait for it here, ahead of the slab loads); rows >= B are not stored
    const int row = min(r0 + (rsel * RBW + rb) * 16 + 4 * lg + kw, B - 1);
    const float* gxr = gx_t + g * s_gx + (long)row * 3 * H;
#pragma unroll
    for (int q = 0; q < 3; ++q) gxv[rb][q] = gxr[q * H + j];
    hpv[rb] = hp[(long)row * H + j];
  }
  floatx4 acc[RBW][3];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int q = 0; q < 3; ++q) acc[rb][q] = (floatx4){0.f, 0.f, 0.f, 0.f};
  rolling_contraction<3, false, RB, NW, W>(W_hh + g * s_rep + (long)j0 * H, (long)H * H, hp + (long)r0 * H, H, B - r0,
                                staged_lds, acc);
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        red[((kw * 3 * RB + (rsel * RBW + rb) * 3 + q) * 4 + v) * 64 + lane] = acc[rb][q][v];
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    const int rbg = rsel * RBW + rb;
    const int row = r0 + rbg * 16 + 4 * lg + kw;
    float gh[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int o = ((rbg * 3 + q) * 4 + kw) * 64 + lane;
      gh[q] = ((red[o] + red[o + 3 * RB * 256]) + (red[o + 6 * RB * 256] + red[o + 9 * RB * 256])) + bias[q];
    }
    if (row < B) {
      const float r = sigm(gxv[rb][0] + gh[0]);
      const float z = sigm(gxv[rb][1] + gh[1]);
      const float qv = gh[2];
      const float n = tanhf(gxv[rb][2] + r * qv);
      h_out[g * s_hs + (long)row * H + j] = (1.0f - z) * n + z * hpv[rb];
      float* sv = sv_t + g * s_sv + (long)row * 4 * H;
      sv[j] = r;
      sv[H + j] = z;
      sv[2 * H + j] = n;
      sv[3 * H + j] = qv;
    }
  }
}

// bf16 variants: 64-word slabs, so that two or three workgroups fit on a CU (config 3 launches
// two workgroups per CU; resident together they cover each other's load latency)
static constexpr int SKB = 64;
static constexpr int TTP = 40;  // pitch (bf16) of a staged transposed-output row of 32 batch rows
static constexpr size_t kFwdBf16Lds = (2 * 80 * (SKB + 4) + 4 * 6 * 4 * 64) * sizeof(float);
static constexpr size_t kBwdBf16Lds = (2 * 48 * (SKB + 4) + 4 * 2 * 4 * 64) * sizeof(float);

// Up to one workgroup per CU: 8 waves per workgroup and 128-word slabs (two waves on every
// SIMD cover each other's LDS and barrier latency; 84 KB of LDS, one workgroup per CU).
// More workgroups than CUs: 4 waves and 64-word slabs, so that several fit on a CU.
static bool step_wide(int B, int H, int groups) {
  return (long)(H / FJ) * ((B + FR - 1) / FR) * groups <= 256;
}

template <int RB, int NW, int W>
static hipError_t launch_fwd_rb(const float* W_hh, const float* b_hh, long s_rep, const float* gx_t, long s_gx,
                                const float* h_prev, float* h_out, long s_hs, float* sv_t, long s_sv, int B,
                                int H, int groups, hipStream_t s) {
  constexpr size_t slabs = 2 * (48 + 16 * RB) * (W + 4), redn = 4 * 3 * RB * 4 * 64;
  constexpr size_t lds = (slabs > redn ? slabs : redn) * sizeof(float);
  static bool ready = false;  // allow the dynamic LDS allocation above 64 KB once
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gru_fwd_step_kernel<RB, NW, W>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ready = true;
  }
  dim3 grid((H / FJ) * ((B + 16 * RB - 1) / (16 * RB)) * groups);
  KernelTimer kt(KID_GRU_STEP, 2.0 * B * 3 * H * (double)H * groups, s);
  hipLaunchKernelGGL((gru_fwd_step_kernel<RB, NW, W>), grid, dim3(64 * NW), lds, s, W_hh, b_hh, s_rep, gx_t, s_gx, h_prev,
                     h_out, s_hs, sv_t, s_sv, B, H, groups);
  return hipGetLastError();
}

hipError_t launch_gru_fwd_step(const float* W_hh, const float* b_hh, long s_rep, const float* gx_t,
                                      long s_gx, const float* h_prev, float* h_out, long s_hs,
                                      float* sv_t, long s_sv, int B, int H, int groups, hipStream_t s) {
  return step_wide(B, H, groups)
             ? launch_fwd_rb<2, 8, 128>(W_hh, b_hh, s_rep, gx_t, s_gx, h_prev, h_out, s_hs, sv_t, s_sv, B, H,
                                        groups, s)
             : launch_fwd_rb<2, 4, 64>(W_hh, b_hh, s_rep, gx_t, s_gx, h_prev, h_out, s_hs, sv_t, s_sv, B, H,
                                       groups, s);
}

// Backward step.  WT is W_hh transposed: WT[j][n] = W_hh[n][j], row pitch 3H (unit-stride along
// the contraction).  D holds dh_{t+1} * z_{t+1} on entry (or the head's gradient at the last
// step) and dh_t * z_t on exit.  dgh_next == nullptr at the last step (no recurrent term yet).
template <int RB, int NW, int W>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, 2)))
gru_bwd_step_kernel(const float* __restrict__ WT, long s_wt, const float* __restrict__ dgh_next,
                           long s_dg, float* __restrict__ D, long s_D, const float* __restrict__ above,
                           long s_above, const float* __restrict__ sv_t, long s_sv,
                           const float* __restrict__ h_prev, long s_hs, float* __restrict__ dgx_t,
                           float* __restrict__ dgh_t, int B, int H, int groups) {
  extern __shared__ __attribute__((aligned(16))) float staged_lds[];
  float* red = staged_lds;  // [4][RB][4][64], over the slab buffers once the contraction is done
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, rsel = wave >> 2;
  constexpr int RBW = RB * 4 / NW;  // row blocks per wave
  // the recurrence is the critical path: its waves issue ahead of any throughput kernel
  // (weight-gradient GEMMs, merge) that shares the SIMD
  __builtin_amdgcn_s_setprio(3);
  const int lr = lane & 15, lg = lane >> 4;
  int g, tx, ty;
  constexpr int FRB = 16 * RB;  // batch rows per workgroup
  step_tile(H / FJ, (B + FRB - 1) / FRB, groups, g, tx, ty);
  const int j0 = tx * FJ, r0 = ty * FRB;
  const int H3 = 3 * H;
  const int j = j0 + lr;
  float r_[RBW], z_[RBW], n_[RBW], q_[RBW], hp_[RBW], dh_[RBW], ab_[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    // unconditional loads from a row clamped into the batch (a select on a loaded value
    // would make the wave wait for it here, ahead of the slab loads); rows >= B are not stored
    const int row = min(r0 + (rsel * RBW + rb) * 16 + 4 * lg + kw, B - 1);
    const long e = (long)row * H + j;
    const float* sv = sv_t + g * s_sv + (long)row * 4 * H;
    r_[rb] = sv[j];
    z_[rb] = sv[H + j];
    n_[rb] = sv[2 * H + j];
    q_[rb] = sv[3 * H + j];
    hp_[rb] = h_prev[g * s_hs + e];
    dh_[rb] = D[g * s_D + e];
    ab_[rb] = above ? above[g * s_above + e] : 0.f;
  }
  floatx4 acc[RBW][1];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) acc[rb][0] = (floatx4){0.f, 0.f, 0.f, 0.f};
  if (dgh_next)
    rolling_contraction<1, false, RB, NW, W>(WT + g * s_wt + (long)j0 * H3, 0, dgh_next + g * s_dg + (long)r0 * H3, H3,
                                  B - r0, staged_lds, acc);
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[((kw * RB + rsel * RBW + rb) * 4 + v) * 64 + lane] = acc[rb][0][v];
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    const int rbg = rsel * RBW + rb;
    const int row = r0 + rbg * 16 + 4 * lg + kw;
    const int o = (rbg * 4 + kw) * 64 + lane;
    const float rec = (red[o] + red[o + RB * 256]) + (red[o + 2 * RB * 256] + red[o + 3 * RB * 256]);
    if (row < B) {
      const long e = (long)row * H + j;
      const float dh = (dh_[rb] + ab_[rb]) + rec;
      const float r = r_[rb], z = z_[rb], n = n_[rb], q = q_[rb];
      const float dn = dh * (1.0f - z);
      const float dz = dh * (hp_[rb] - n);
      const float da_n = dn * (1.0f - n * n);
      const float dq = da_n * r;
      const float da_r = da_n * q * r * (1.0f - r);
      const float da_z = dz * z * (1.0f - z);
      float* ox = dgx_t + g * s_dg + (long)row * H3;
      float* oh = dgh_t + g * s_dg + (long)row * H3;
      ox[j] = da_r;
      ox[H + j] = da_z;
      ox[2 * H + j] = da_n;
      oh[j] = da_r;
      oh[H + j] = da_z;
      oh[2 * H + j] = dq;
      D[g * s_D + e] = dh * z;
    }
  }
}

template <int RB, int NW, int W>
static hipError_t launch_bwd_rb(const float* WT, long s_wt, const float* dgh_next, long s_dg, float* D, long s_D,
                                const float* above, long s_above, const float* sv_t, long s_sv,
                                const float* h_prev, long s_hs, float* dgx_t, float* dgh_t, int B, int H,
                                int groups, hipStream_t s) {
  constexpr size_t slabs = 2 * (16 + 16 * RB) * (W + 4), redn = 4 * RB * 4 * 64;
  constexpr size_t lds = (slabs > redn ? slabs : redn) * sizeof(float);
  static bool ready = false;  // allow the dynamic LDS allocation above 64 KB once
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gru_bwd_step_kernel<RB, NW, W>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ready = true;
  }
  dim3 grid((H / FJ) * ((B + 16 * RB - 1) / (16 * RB)) * groups);
  KernelTimer kt(KID_GRU_STEP, 2.0 * B * 3 * H * (double)H * groups, s);
  hipLaunchKernelGGL((gru_bwd_step_kernel<RB, NW, W>), grid, dim3(64 * NW), lds, s, WT, s_wt, dgh_next, s_dg, D, s_D, above,
                     s_above, sv_t, s_sv, h_prev, s_hs, dgx_t, dgh_t, B, H, groups);
  return hipGetLastError();
}

hipError_t launch_gru_bwd_step(const float* WT, long s_wt, const float* dgh_next, long s_dg,
                                      float* D, long s_D, const float* above, long s_above,
                                      const float* sv_t, long s_sv, const float* h_prev, long s_hs,
                                      float* dgx_t, float* dgh_t, int B, int H, int groups, hipStream_t s) {
  return step_wide(B, H, groups)
             ? launch_bwd_rb<2, 8, 128>(WT, s_wt, dgh_next, s_dg, D, s_D, above, s_above, sv_t, s_sv, h_prev, s_hs,
                                        dgx_t, dgh_t, B, H, groups, s)
             : launch_bwd_rb<2, 4, 64>(WT, s_wt, dgh_next, s_dg, D, s_D, above, s_above, sv_t, s_sv, h_prev, s_hs,
                                       dgx_t, dgh_t, B, H, groups, s);
}

// ---------------------------------------------------------------------------- bf16 variants
// Same tiling and the same staged data path with v_mfma_f32_16x16x32_bf16: A lane l holds
// A[m = l%16][k = 8*(l/16) .. +7], B lane l holds B[k = 8*(l/16) .. +7][n = l%16]: one 16-byte
// fragment per operand per 32-wide contraction chunk.  The operands come from bf16 copies (weights converted once per local
// step, h_t / dgh_t written in both precisions by the previous step's epilogue), i.e. every
// GEMM operand is the nearest-even bf16 rounding of the fp32 value; accumulation, the cell
// math and everything stored for later use stay fp32.
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
gru_fwd_step_bf16_kernel(const __bf16* __restrict__ Wb, long s_wb, const float* __restrict__ b_hh,
                         long s_rep, const float* __restrict__ gx_t, long s_gx,
                         const float* __restrict__ h_prev, float* __restrict__ h_out, long s_hs,
                         const __bf16* __restrict__ hb_prev, __bf16* __restrict__ hb_out, long s_hb,
                         float* __restrict__ sv_t, long s_sv, __bf16* __restrict__ hT_out, long ld_hT,
                         long s_hT, int B, int H, int groups) {
  extern __shared__ __attribute__((aligned(16))) float staged_lds[];
  float* red = staged_lds + 2 * 80 * (SKB + 4);  // [4][6][4][64]
  // transposed output tile [16 units][32 rows] (the slab buffers are free by then)
  __bf16* tt = reinterpret_cast<__bf16*>(staged_lds);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the recurrence is the critical path: its waves issue ahead of any throughput kernel
  // (weight-gradient GEMMs, merge) that shares the SIMD
  __builtin_amdgcn_s_setprio(3);
  const int lr = lane & 15, lg = lane >> 4;
  int g, tx, ty;
  step_tile(H / FJ, (B + FR - 1) / FR, groups, g, tx, ty);
  const int j0 = tx * FJ, r0 = ty * FR;
  const float* hp = h_prev + g * s_hs;
  const float* bh = b_hh + g * s_rep;
  const int j = j0 + lr;
  float gxv[2][3], hpv[2], bias[3];
#pragma unroll
  for (int q = 0; q < 3; ++q) bias[q] = bh[q * H + j];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    // unconditional loads from a row clamped into the batch (a select on a loaded value
    // would make the wave wait for it here, ahead of the slab loads); rows >= B are not stored
    const int row = min(r0 + rb * 16 + 4 * lg + wave, B - 1);
    const float* gxr = gx_t + g * s_gx + (long)row * 3 * H;
#pragma unroll
    for (int q = 0; q < 3; ++q) gxv[rb][q] = gxr[q * H + j];
    hpv[rb] = hp[(long)row * H + j];
  }
  floatx4 acc[2][3];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int q = 0; q < 3; ++q) acc[rb][q] = (floatx4){0.f, 0.f, 0.f, 0.f};
  // rows of bf16 pairs, addressed in 4-byte words
  rolling_contraction<3, true>(reinterpret_cast<const float*>(Wb + g * s_wb + (long)j0 * H), (long)H * H / 2,
                                 reinterpret_cast<const float*>(hb_prev + g * s_hb + (long)r0 * H), H / 2,
                                 B - r0, staged_lds, acc);
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[((wave * 6 + rb * 3 + q) * 4 + v) * 64 + lane] = acc[rb][q][v];
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int row = r0 + rb * 16 + 4 * lg + wave;
    float gh[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int o = ((rb * 3 + q) * 4 + wave) * 64 + lane;
      gh[q] = ((red[o] + red[o + 6 * 256]) + (red[o + 12 * 256] + red[o + 18 * 256])) + bias[q];
    }
    if (row < B) {
      const float r = sigm(gxv[rb][0] + gh[0]);
      const float z = sigm(gxv[rb][1] + gh[1]);
      const float qv = gh[2];
      const float n = tanhf(gxv[rb][2] + r * qv);
      const float hn = (1.0f - z) * n + z * hpv[rb];
      h_out[g * s_hs + (long)row * H + j] = hn;
      hb_out[g * s_hb + (long)row * H + j] = (__bf16)hn;
      if (hT_out) tt[lr * TTP + rb * 16 + 4 * lg + wave] = (__bf16)hn;
      float* sv = sv_t + g * s_sv + (long)row * 4 * H;
      sv[j] = r;
      sv[H + j] = z;
      sv[2 * H + j] = n;
      sv[3 * H + j] = qv;
    }
  }
  if (hT_out) {
    // 64-byte row segments of the transposed copy [unit][time*B + row], 16 bytes per thread
    __syncthreads();
    if (tid < 64) {
      const int u = tid >> 2, part = tid & 3;
      if (r0 + 8 * part < B)  // B is a multiple of 8: a chunk of 8 rows is all in or all out
        *reinterpret_cast<uint4*>(hT_out + g * s_hT + (long)(j0 + u) * ld_hT + r0 + 8 * part) =
            *reinterpret_cast<const uint4*>(tt + u * TTP + 8 * part);
    }
  }
}

hipError_t launch_gru_fwd_step_bf16(const void* Wb, long s_wb, const float* b_hh, long s_rep,
                                    const float* gx_t, long s_gx, const float* h_prev, float* h_out,
                                    long s_hs, const void* hb_prev, void* hb_out, long s_hb, float* sv_t,
                                    long s_sv, void* hT_out, long ld_hT, long s_hT, int B, int H,
                                    int groups, hipStream_t s) {
  static bool ready = false;  // allow the dynamic LDS allocation above 64 KB once
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gru_fwd_step_bf16_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFwdBf16Lds);
    if (e != hipSuccess) return e;
    ready = true;
  }
  dim3 grid((H / FJ) * ((B + FR - 1) / FR) * groups);
  KernelTimer kt(KID_GRU_STEP, 2.0 * B * 3 * H * (double)H * groups, s);
  hipLaunchKernelGGL(gru_fwd_step_bf16_kernel, grid, dim3(256), kFwdBf16Lds, s, (const __bf16*)Wb, s_wb,
                     b_hh, s_rep, gx_t, s_gx, h_prev, h_out, s_hs, (const __bf16*)hb_prev, (__bf16*)hb_out,
                     s_hb, sv_t, s_sv, (__bf16*)hT_out, ld_hT, s_hT, B, H, groups);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
gru_bwd_step_bf16_kernel(const __bf16* __restrict__ WTb, long s_wt,
                         const __bf16* __restrict__ dghb_next, __bf16* __restrict__ dghb_t, long s_dgb,
                         float* __restrict__ D, long s_D, const float* __restrict__ above,
                         long s_above, const float* __restrict__ sv_t, long s_sv,
                         const float* __restrict__ h_prev, long s_hs, float* __restrict__ dgx_t,
                         float* __restrict__ dgh_t, long s_dg, __bf16* __restrict__ dgxb_t,
                         __bf16* __restrict__ dgxT_t, __bf16* __restrict__ dghT_t, long ld_T, long s_T,
                         int B, int H, int groups) {
  extern __shared__ __attribute__((aligned(16))) float staged_lds[];
  float* red = staged_lds + 2 * 48 * (SKB + 4);  // [4][2][4][64]
  // transposed output tile [da_r | da_z | da_n | dq][16 units][32 rows] (the slab buffers are free by then)
  __bf16* tt = reinterpret_cast<__bf16*>(staged_lds);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the recurrence is the critical path: its waves issue ahead of any throughput kernel
  // (weight-gradient GEMMs, merge) that shares the SIMD
  __builtin_amdgcn_s_setprio(3);
  const int lr = lane & 15, lg = lane >> 4;
  int g, tx, ty;
  step_tile(H / FJ, (B + FR - 1) / FR, groups, g, tx, ty);
  const int j0 = tx * FJ, r0 = ty * FR;
  const int H3 = 3 * H;
  const int j = j0 + lr;
  float r_[2], z_[2], n_[2], q_[2], hp_[2], dh_[2], ab_[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    // unconditional loads from a row clamped into the batch (a select on a loaded value
    // would make the wave wait for it here, ahead of the slab loads); rows >= B are not stored
    const int row = min(r0 + rb * 16 + 4 * lg + wave, B - 1);
    const long e = (long)row * H + j;
    const float* sv = sv_t + g * s_sv + (long)row * 4 * H;
    r_[rb] = sv[j];
    z_[rb] = sv[H + j];
    n_[rb] = sv[2 * H + j];
    q_[rb] = sv[3 * H + j];
    hp_[rb] = h_prev[g * s_hs + e];
    dh_[rb] = D[g * s_D + e];
    ab_[rb] = above ? above[g * s_above + e] : 0.f;
  }
  floatx4 acc[2][1];
  acc[0][0] = (floatx4){0.f, 0.f, 0.f, 0.f};
  acc[1][0] = acc[0][0];
  if (dghb_next)
    rolling_contraction<1, true>(reinterpret_cast<const float*>(WTb + g * s_wt + (long)j0 * H3), 0,
                                    reinterpret_cast<const float*>(dghb_next + g * s_dgb + (long)r0 * H3),
                                    H3 / 2, B - r0, staged_lds, acc);
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[((wave * 2 + rb) * 4 + v) * 64 + lane] = acc[rb][0][v];
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int row = r0 + rb * 16 + 4 * lg + wave;
    const int o = (rb * 4 + wave) * 64 + lane;
    const float rec = (red[o] + red[o + 2 * 256]) + (red[o + 4 * 256] + red[o + 6 * 256]);
    if (row < B) {
      const long e = (long)row * H + j;
      const float dh = (dh_[rb] + ab_[rb]) + rec;
      const float r = r_[rb], z = z_[rb], n = n_[rb], q = q_[rb];
      const float dn = dh * (1.0f - z);
      const float dz = dh * (hp_[rb] - n);
      const float da_n = dn * (1.0f - n * n);
      const float dq = da_n * r;
      const float da_r = da_n * q * r * (1.0f - r);
      const float da_z = dz * z * (1.0f - z);
      float* ox = dgx_t + g * s_dg + (long)row * H3;
      float* oh = dgh_t + g * s_dg + (long)row * H3;
      __bf16* ob = dghb_t + g * s_dgb + (long)row * H3;
      ox[j] = da_r;
      ox[H + j] = da_z;
      ox[2 * H + j] = da_n;
      oh[j] = da_r;
      oh[H + j] = da_z;
      oh[2 * H + j] = dq;
      ob[j] = (__bf16)da_r;
      ob[H + j] = (__bf16)da_z;
      ob[2 * H + j] = (__bf16)dq;
      if (dgxb_t) {
        // bf16 copies for the time-batched GEMMs: dgx row-major (input gradient), and the
        // four distinct gate-gradient blocks staged for the transposed copies
        __bf16* oxb = dgxb_t + g * s_dgb + (long)row * H3;
        oxb[j] = (__bf16)da_r;
        oxb[H + j] = (__bf16)da_z;
        oxb[2 * H + j] = (__bf16)da_n;
        const int rl = rb * 16 + 4 * lg + wave;
        tt[(0 * 16 + lr) * TTP + rl] = (__bf16)da_r;
        tt[(1 * 16 + lr) * TTP + rl] = (__bf16)da_z;
        tt[(2 * 16 + lr) * TTP + rl] = (__bf16)da_n;
        tt[(3 * 16 + lr) * TTP + rl] = (__bf16)dq;
      }
      D[g * s_D + e] = dh * z;
    }
  }
  if (dgxb_t) {
    // transposed copies [gate unit][time*B + row] as 64-byte row segments, 16 bytes per
    // thread: dgx^T = (da_r, da_z, da_n), dgh^T = (da_r, da_z, dq)
    __syncthreads();
    const int blk = tid >> 6, u = (tid >> 2) & 15, part = tid & 3;  // blk: which staged block
    if (r0 + 8 * part < B) {  // B is a multiple of 8: a chunk of 8 rows is all in or all out
      const uint4 v = *reinterpret_cast<const uint4*>(tt + (blk * 16 + u) * TTP + 8 * part);
      const long col = r0 + 8 * part;
      const int gate = blk == 3 ? 2 : blk;
      const long o = g * s_T + (long)(gate * H + j0 + u) * ld_T + col;
      if (blk != 3) *reinterpret_cast<uint4*>(dgxT_t + o) = v;
      if (blk != 2) *reinterpret_cast<uint4*>(dghT_t + o) = v;
    }
  }
}

hipError_t launch_gru_bwd_step_bf16(const void* WTb, long s_wt, const void* dghb_next, void* dghb_t,
                                    long s_dgb, float* D, long s_D, const float* above, long s_above,
                                    const float* sv_t, long s_sv, const float* h_prev, long s_hs,
                                    float* dgx_t, float* dgh_t, long s_dg, void* dgxb_t, void* dgxT_t,
                                    void* dghT_t, long ld_T, long s_T, int B, int H, int groups,
                                    hipStream_t s) {
  dim3 grid((H / FJ) * ((B + FR - 1) / FR) * groups);
  KernelTimer kt(KID_GRU_STEP, 2.0 * B * 3 * H * (double)H * groups, s);
  hipLaunchKernelGGL(gru_bwd_step_bf16_kernel, grid, dim3(256), kBwdBf16Lds, s, (const __bf16*)WTb, s_wt,
                     (const __bf16*)dghb_next, (__bf16*)dghb_t, s_dgb, D, s_D, above, s_above, sv_t, s_sv,
                     h_prev, s_hs, dgx_t, dgh_t, s_dg, (__bf16*)dgxb_t, (__bf16*)dgxT_t, (__bf16*)dghT_t, ld_T,
                     s_T, B, H, groups);
  return hipGetLastError();
}

// out (bf16) = nearest-even rounding of in (fp32, R x C, row pitch ld_in) per group;
// TRANSPOSE: out[c][r] = in[r][c] with row pitch ld_out, else out[r][c] with row pitch ld_out.
// 64 x 64 tiles: rows are read 256 bytes at a time, and the transposed tile is written as
// packed pairs of bf16, 128 bytes per output row.
template <bool TRANSPOSE>
__global__ void __launch_bounds__(256)
cvt_bf16_kernel(const float* __restrict__ in, long ld_in, long s_in, __bf16* __restrict__ out,
                long ld_out, long s_out, int R, int C) {
  __shared__ float tile[64][65];
  const int g = blockIdx.z;
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
  const float* src = in + g * s_in;
  __bf16* dst = out + g * s_out;
  if (!TRANSPOSE) {
    for (int i = ty; i < 64; i += 4) {
      const int r = r0 + i, c = c0 + tx;
      if (r < R && c < C) dst[(long)r * ld_out + c] = (__bf16)src[(long)r * ld_in + c];
    }
    return;
  }
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < R && c < C) ? src[(long)r * ld_in + c] : 0.f;
  }
  __syncthreads();
  // output row = input column c0 + i; a lane writes input rows r0 + 2*px, +1 as one 4-byte pair
  const int px = threadIdx.x & 31, py = threadIdx.x >> 5;  // 32 pairs x 8
  const bool pair_ok = (ld_out & 1) == 0 && (s_out & 1) == 0 && ((uintptr_t)out & 3) == 0;
  for (int i = py; i < 64; i += 8) {
    const int c = c0 + i, r = r0 + 2 * px;
    if (c >= C || r >= R) continue;
    __bf16* o = dst + (long)c * ld_out + r;
    if (pair_ok && r + 1 < R) {
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      bf16x2 v;
      v[0] = (__bf16)tile[2 * px][i];
      v[1] = (__bf16)tile[2 * px + 1][i];
      *reinterpret_cast<bf16x2*>(o) = v;
    } else {
      o[0] = (__bf16)tile[2 * px][i];
      if (r + 1 < R) o[1] = (__bf16)tile[2 * px + 1][i];
    }
  }
}

hipError_t launch_cvt_bf16(const float* in, long ld_in, long s_in, void* out, long ld_out, long s_out,
                           int R, int C, bool transpose, int groups, hipStream_t s) {
  dim3 grid((C + 63) / 64, (R + 63) / 64, groups);
  if (transpose)
    hipLaunchKernelGGL(cvt_bf16_kernel<true>, grid, dim3(256), 0, s, in, ld_in, s_in, (__bf16*)out, ld_out,
                       s_out, R, C);
  else
    hipLaunchKernelGGL(cvt_bf16_kernel<false>, grid, dim3(256), 0, s, in, ld_in, s_in, (__bf16*)out, ld_out,
                       s_out, R, C);
  return hipGetLastError();
}

bool gru_fused_bf16_supported(int H) { return H % 32 == 0 && H >= 32 && H <= 2048; }

// ---------------------------------------------------------------------------- transpose
// out[c][r] = in[r][c] for an R x C matrix per group (32x32 tiles through LDS).
__global__ void __launch_bounds__(256)
transpose_kernel(const float* __restrict__ in, long s_in, float* __restrict__ out, long s_out, int R,
                 int C) {
  __shared__ float tile[32][33];
  const int g = blockIdx.z;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < R && c < C) ? in[g * s_in + (long)r * C + c] : 0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, r = r0 + tx;
    if (r < R && c < C) out[g * s_out + (long)c * R + r] = tile[tx][i];
  }
}

hipError_t launch_transpose(const float* in, long s_in, float* out, long s_out, int R, int C,
                            int groups, hipStream_t s) {
  dim3 grid((C + 31) / 32, (R + 31) / 32, groups);
  hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, s, in, s_in, out, s_out, R, C);
  return hipGetLastError();
}

// The fused kernels need 16-byte loads along the contraction: H a multiple of 16, operand
// bases 16-byte aligned, and at most 64*NCH_max contraction elements per wave quarter.
bool gru_fused_supported(int H) { return H % 16 == 0 && H >= 16 && H <= 1024; }

}  // namespace hpsgd
