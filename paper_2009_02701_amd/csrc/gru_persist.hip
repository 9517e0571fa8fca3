// Recurrence kernels that stay on the chip for a whole run of time steps (fp32).
//
// One launch per time step pays, at every step, a launch gap, a cold L2 and the transfer of
// the workgroup's slice of W_hh (the larger part of what a step reads).  Here a workgroup
// keeps its slice of W_hh (forward: the 3 x 16 gate rows of its 16 hidden units; backward:
// 16 rows of W_hh^T) in LDS for all the steps of the launch; the activations of the step
// (h_{t-1}, or the gate gradients of step t+1) go from memory straight into MFMA operand
// registers, every wave fetching exactly the fragments it multiplies, so that the matrix
// work of a step needs no barrier until the partial sums are combined.
//
// The steps of one launch depend on each other across workgroups: h_t of a 32-row batch tile
// is produced by the NJ = H/16 workgroups that own its hidden units, and every one of them
// needs all of it for step t+1.  Those NJ workgroups form a synchronisation group with one
// flag word per member in device memory.  Protocol (no cache-wide write-back or invalidate,
// which cost several microseconds per step when 32 workgroups of an XCD each ask for one):
//   producer: the exchanged values are stored with device-scope write-through stores (sc1);
//             the workgroup barrier waits until every wave's stores have completed; then
//             thread 0 stores the number of steps done into the member's flag (device scope);
//   consumer: wave 0 polls the group's flags (device-scope loads, one lane per member) until
//             all NJ producers have completed the step; workgroup barrier; the operand loads that follow are
//             device-scope loads (sc1), which are served from the level of the memory
//             hierarchy that all XCDs share, never from a stale line of this XCD's caches.
// Values nobody reads before the launch ends (the saved gates, dgx) take ordinary stores.
//
// Scope of the exchange.  A synchronisation group whose members all run on one XCD shares that
// XCD's L2, and the exchanged values and the counts need to get no further than that: ordinary
// stores (the CU's vector cache writes through to L2), the same sc1 loads on the consuming side
// (they bypass the vector cache, which is all that is needed of them there).  A hand-off among 32
// workgroups then takes 0.73 us instead of 1.92 us (measured).  Where a workgroup lands is the
// dispatcher's business (workgroup i of a launch is not always on XCD i % 8 when other launches
// are in flight), so a launch that wants this does not tie a workgroup's tile to its index: when
// the launch fills the chip with one workgroup per CU, every XCD necessarily receives as many
// workgroups as it has CUs, and a workgroup takes its place from where it runs - it draws a
// ticket from the counter of its XCD (HW_REG_XCC_ID) and is member `ticket` there, of the groups
// that the tile order gives to that XCD.  A ticket beyond the XCD's share (it cannot happen while
// one workgroup fills a CU) sets the abort word: the launch fails loudly.  Otherwise the tile is
// that of the workgroup index and the exchange is at device scope as described above.
//
// Waiting needs every workgroup of the grid resident at the same time: the launcher refuses
// grids with more workgroups than the device has compute units (a workgroup takes most of a
// CU's LDS, so there is one per CU), and launches of these kernels from different streams are
// ordered against each other by the caller.  Every wait is bounded: when the spin limit runs
// out, or another workgroup has given up, the workgroup sets the abort word and the whole
// workgroup leaves the kernel, so every wave reaches its end whatever happens.
//
// Tiling: 8 waves, 32 batch rows x 16 hidden units per workgroup, v_mfma_f32_16x16x4_f32.
// The contraction is cut into 32-wide chunks, chunk c belongs to waves with (wave & 3) == c % 4,
// the two 16-row blocks to the wave halves (wave >> 2); partial sums are combined through LDS.
// MFMA 16x16x4 lane layout: A lane l holds A[m = l%16][k = l/16], B lane l holds
// B[k = l/16][n = l%16], accumulator register v holds C[4*(l/16) + v][l%16].  The order of the
// contraction index is free as long as both operands agree: for the chunk's MFMA number
// e = 0..7 lane group lg = l/16 takes k = 32c + 16*(e/4) + 4*lg + e%4, i.e. two 16-byte pieces
// of its row per chunk, and one load instruction reads 64 contiguous bytes of each of 16 rows.
#include "kernels.h"

namespace hpsgd {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int PNT = 512;     // threads per workgroup
constexpr int PR = 32;       // batch rows per workgroup
constexpr int PJ = 16;       // hidden units per workgroup
constexpr int PC = 32;       // contraction chunk
constexpr int SP = 80;       // pitch of the staged dgh tile: 4 batch rows x 16 gate rows hit 64 banks

__device__ __forceinline__ float sigm_p(float a) { return 1.0f / (1.0f + expf(-a)); }
// The gates of the bf16 forward launch, whose cell math is a fifth of a step: the hardware's
// exp2 and reciprocal (1 ulp each) in place of the library's expf, tanhf and division.  Absolute
// error about 1e-7 (tanh near 0 included: 1 - 2 / (e^2a + 1) loses relative, not absolute, accuracy),
// against gate values that are then rounded to bf16 (4e-3 relative) as operands.
__device__ __forceinline__ float sigm_fast(float a) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * a));
}
__device__ __forceinline__ float tanh_fast(float a) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.88539008f * a));
}

// Workgroup i runs on XCD i % 8; a synchronisation group (worker g, row tile ty) is kept on
// one XCD when the number of groups allows it.  sg = g * RT + ty.
__device__ __forceinline__ void persist_tile(int i, int NJ, int RT, int groups, int& g, int& tx, int& ty, int& sg) {
  const int SG = groups * RT;
  if (SG % 8 == 0) {
    const int c = i & 7, li = i >> 3;
    sg = c + 8 * (li / NJ);
    tx = li % NJ;
  } else {
    sg = i / NJ;
    tx = i % NJ;
  }
  g = sg / RT;
  ty = sg % RT;
}

// A synchronisation group owns PF flag words, one per member: a member stores the number of
// steps it has completed into its own word (plain device-scope stores to distinct words: no
// read-modify-write that the group's members would queue up for), and the waiting side reads
// all of them with one load instruction of wave 0, lane l looking at member l.
constexpr int PF = 64;  // flag words per group (a group has H/16 or H/32 <= 42 members)

// Wave 0 polls the group's flags until every member has reached `target` (wrap-safe), then the
// whole workgroup passes a barrier.  Returns false, for every thread alike, if the wait was
// given up; the abort word is then set.  limit == 0 makes every wait fail (the host-forced
// way to exercise the abort path).
__device__ __forceinline__ bool group_wait(unsigned* flags, int members, unsigned target, unsigned* abort_w,
                                           unsigned limit, int* lds_flag) {
  if (threadIdx.x < 64) {
    const int l = threadIdx.x;
    int ok = limit != 0;
    unsigned n = 0;
    while (ok) {
      const unsigned v = __hip_atomic_load(flags + (l < members ? l : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__all((int)(v - target) >= 0)) break;
      if (++n > limit || __hip_atomic_load(abort_w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) ok = 0;
      else __builtin_amdgcn_s_sleep(1);
    }
    if (l == 0) {
      if (!ok) __hip_atomic_store(abort_w, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *lds_flag = ok;
    }
  }
  __syncthreads();
  return *lds_flag != 0;
}

// Publishes the number of steps this member has completed, after the step's exchanged values.
// Order of data and count, by construction:
//   1. every wave waits until the vector-memory counter of its own accesses is zero
//      (s_waitcnt vmcnt(0): on this target stores count in vmcnt too, and a device-scope
//      write-through store is counted out only when the level of the memory hierarchy that all
//      XCDs share has acknowledged it);
//   2. the workgroup barrier: every wave of the workgroup has passed step 1;
//   3. thread 0 stores the count (device scope).
// A consumer that reads the count (device-scope load) and then issues its operand loads
// (device-scope, behind a barrier of its own workgroup) therefore reads the data of the step.
// The wait is written out: a workgroup-scope fence would only have to order LDS traffic here,
// and an agent-scope release would write back the XCD's whole L2.
// (l2x: the group shares one L2 and an ordinary store, acknowledged by that L2, takes the place of
// the write-through store in steps 1 and 3.)
__device__ __forceinline__ void group_signal(unsigned* my_flag, unsigned steps_done, bool l2x) {
  // vmcnt = 0 (bits 3:0 and 15:14), expcnt and lgkmcnt left at their maxima (no wait)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  if (threadIdx.x == 0) {
    if (l2x) __hip_atomic_store(my_flag, steps_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_store(my_flag, steps_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// The XCD this wave runs on (HW_REG_XCC_ID, bits 3:0)
__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15u; }

// The index that names this workgroup's tile, and whether its group exchanges through one L2.
// tickets == nullptr: the workgroup index, device scope.  Else (8 counters behind the flag words,
// zero at the start of the step; this launch is the one whose tickets start at ticket_base, per_xcd
// workgroups per XCD): member `ticket` of XCD x is index 8 ticket + x, which persist_tile puts into
// a group of workgroups with the same x.  Returns false, for every thread alike and with the abort
// word set, if the ticket is beyond the XCD's share.  Contains a barrier.
__device__ __forceinline__ bool persist_place(unsigned* tickets, unsigned ticket_base, unsigned per_xcd, unsigned* abort_w,
                                              int* lds_word, int& index, bool& l2x) {
  index = blockIdx.x;
  l2x = tickets != nullptr;
  if (!l2x) return true;
  if (threadIdx.x == 0) {
    const unsigned x = xcc_id();
    unsigned t = per_xcd;
    if (x < 8u) t = __hip_atomic_fetch_add(tickets + x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ticket_base;
    const bool ok = t < per_xcd;
    if (!ok) __hip_atomic_store(abort_w, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_word = ok ? (int)(8u * t + x) : -1;
  }
  __syncthreads();
  index = *lds_word;
  __syncthreads();  // (the word is used again by the first wait)
  return index >= 0;
}

// 16 bytes at byte offset `off` of the buffer, as a device-scope load
__device__ __forceinline__ float4 ld16_dev(__amdgpu_buffer_rsrc_t rs, int off) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 16 /* sc1 */);
  return __builtin_bit_cast(float4, v);
}
// store of an exchanged value: device-scope (write-through), or ordinary when the group shares one L2
__device__ __forceinline__ void st_dev(float* p, float v, bool l2x) {
  if (l2x) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Copies `rows` weight rows of KD words (row r at src + row_off(r)) into LDS at pitch wp and
// zeroes the columns from KD up to the next multiple of the chunk.
template <typename RowOff>
__device__ __forceinline__ void load_resident(float* wres, int wp, const float* src, int rows, int KD,
                                              RowOff row_off) {
  const int KDp = (KD + PC - 1) / PC * PC, ur = KDp >> 2;
  for (int u = threadIdx.x; u < rows * ur; u += PNT) {
    const int row = u / ur, c4 = u - row * ur;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (4 * c4 < KD) v = *reinterpret_cast<const float4*>(src + row_off(row) + 4 * c4);
    *reinterpret_cast<float4*>(&wres[row * wp + 4 * c4]) = v;
  }
}

// The loads of NB chunks of this wave, first chunk c0 (= wave & 3, + 4 per chunk).  rs: buffer
// over the workgroup's activation tile (row pitch KD words); rows >= rows_valid are read from
// row 0 (their results are never stored), columns beyond KD from column 0 (they meet a zero weight).
template <int NB>
__device__ __forceinline__ void fragment_loads(__amdgpu_buffer_rsrc_t rs, int KD, int rows_valid, int c0,
                                               float4 (&a)[NB][2]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rsel = wave >> 2, lr = lane & 15, lg = lane >> 4;
  const int row = rsel * 16 + lr;
  const int rowoff = (row < rows_valid ? row : 0) * KD;
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int k0 = PC * (c0 + 4 * i) + 4 * lg;
    // (KD is a multiple of 16: each piece is all in or all out)
    a[i][0] = ld16_dev(rs, (rowoff + (k0 < KD ? k0 : 0)) * 4);
    a[i][1] = ld16_dev(rs, (rowoff + (k0 + 16 < KD ? k0 + 16 : 0)) * 4);
  }
}

// ... and their products with the resident rows
template <int NQ, int NB>
__device__ __forceinline__ void fragment_mfmas(const float* wres, int wp, int KD, int c0, const float4 (&a)[NB][2],
                                               floatx4 (&acc)[2][NQ]) {
  const int lane = threadIdx.x & 63;
  const int lr = lane & 15, lg = lane >> 4;
  const int nch = (KD + PC - 1) / PC;
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    // branch-free (a branch would pull the loads of its chunk in behind it): a chunk slot
    // beyond the contraction reads weight column 0 and gets zeros instead
    const int c = c0 + 4 * i;
    const bool cv = c < nch;  // uniform over the wave
    const int cc = cv ? c : 0;
    float4 w[NQ][2];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const float* wr = &wres[(q * 16 + lr) * wp + PC * cc + 4 * lg];
      const float4 w0 = *reinterpret_cast<const float4*>(wr);
      const float4 w1 = *reinterpret_cast<const float4*>(wr + 16);
      w[q][0] = make_float4(cv ? w0.x : 0.f, cv ? w0.y : 0.f, cv ? w0.z : 0.f, cv ? w0.w : 0.f);
      w[q][1] = make_float4(cv ? w1.x : 0.f, cv ? w1.y : 0.f, cv ? w1.z : 0.f, cv ? w1.w : 0.f);
    }
    // consecutive MFMAs update different accumulators
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const float4 av = a[i][e >> 2], wv = w[q][e >> 2];
        const float as = (e & 3) == 0 ? av.x : (e & 3) == 1 ? av.y : (e & 3) == 2 ? av.z : av.w;
        const float ws = (e & 3) == 0 ? wv.x : (e & 3) == 1 ? wv.y : (e & 3) == 2 ? wv.z : wv.w;
        acc[e & 1][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(as, ws, acc[e & 1][q], 0, 0, 0);
      }
  }
}

// The exchanged operands (h_t, the gate gradients) are not read from a row-major matrix: there a
// load instruction fetches 64 bytes of each of 16 rows, half a cache line per row, which a CU
// does 2.8 times slower than whole lines (see the bf16 part below).  They are kept
// fragment-major: per step a block of ceil(B/16) row blocks x ceil(KD/32) chunks x 2 halves,
// each the 1 KB one load instruction reads, lane l's 16 bytes at byte 16 l (lane l: row l % 16,
// contraction indices 16 half + 4 (l / 16) .. + 3 of the chunk).  xoff: word offset of (row, k)
// inside a step's block; halves beyond KD are never written and never read.
__device__ __forceinline__ long xoff(int row, int nch, int k) {
  return ((((long)(row >> 4) * nch + (k >> 5)) * 2 + ((k >> 4) & 1)) * 64 + (((k & 15) >> 2) << 4) + (row & 15)) * 4 + (k & 3);
}
// words of a step's block
__host__ __device__ __forceinline__ long xblock_words(int B, int KD) {
  return (long)((B + 15) / 16) * 16 * ((KD + PC - 1) / PC) * PC;
}
// fragment_loads from a step's fragment-major block (rs), row block rbx of it
template <int NB>
__device__ __forceinline__ void fragment_loads_x(__amdgpu_buffer_rsrc_t rs, int KD, int rbx, int c0, float4 (&a)[NB][2]) {
  const int lane = threadIdx.x & 63;
  const int nch = (KD + PC - 1) / PC;
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int c = c0 + 4 * i;
    // (KD is a multiple of 16: a half is all in or all out; one that is out meets zero weights and
    // is read from the block's first fragment)
    const bool v0 = PC * c < KD, v1 = PC * c + 16 < KD;
    a[i][0] = ld16_dev(rs, ((rbx * nch + (v0 ? c : 0)) * 2) * 1024 + lane * 16);
    a[i][1] = ld16_dev(rs, ((rbx * nch + (v1 ? c : 0)) * 2 + (v1 ? 1 : 0)) * 1024 + lane * 16);
  }
}

// acc[i][q] (i = 0, 1: two accumulators per gate block, summed by the caller) +=
// sum over this wave's chunks of A[rsel*16 + ..][k] * Wres[q*16 + ..][k].
// wres: the resident weight rows (pitch wp words, zero beyond KD).  NB: chunks per wave whose
// loads are in flight together.
template <int NQ, int NB>
__device__ __forceinline__ void resident_contraction(const float* wres, int wp, __amdgpu_buffer_rsrc_t rs, int KD,
                                                     int rows_valid, floatx4 (&acc)[2][NQ]) {
  const int kw = (threadIdx.x >> 6) & 3;
  const int nch = (KD + PC - 1) / PC;
  for (int c0 = kw; c0 < nch; c0 += 4 * NB) {
    float4 a[NB][2];
    fragment_loads<NB>(rs, KD, rows_valid, c0, a);
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before anything waits for one
    fragment_mfmas<NQ, NB>(wres, wp, KD, c0, a, acc);
  }
}

// ... with the activations in a fragment-major block
// behind(): called once, behind the first trip's loads - where a step requests what it needs one
// step later from memory (requested in front of the flag wait, such loads would sit between the
// polling wave and its view of the flags: a wave's loads return in order).
template <int NQ, int NB, typename Behind>
__device__ __forceinline__ void resident_contraction_x(const float* wres, int wp, __amdgpu_buffer_rsrc_t rs, int KD,
                                                       int rbx, floatx4 (&acc)[2][NQ], Behind behind) {
  const int kw = (threadIdx.x >> 6) & 3;
  const int nch = (KD + PC - 1) / PC;
  bool first = true;
  for (int c0 = kw; c0 < nch; c0 += 4 * NB) {
    float4 a[NB][2];
    fragment_loads_x<NB>(rs, KD, rbx, c0, a);
    __builtin_amdgcn_sched_barrier(0);
    if (first) behind();
    first = false;
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before anything waits for one
    fragment_mfmas<NQ, NB>(wres, wp, KD, c0, a, acc);
  }
  if (first) behind();
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const float* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, 0x7fffffff, 0x00020000);
}

// Forward: steps t = 0 .. T-1.  hs holds h_0 .. h_T ((T+1) blocks of B x H per worker, h_0
// given), gx the input projections of all steps, sv receives r|z|n|q of every step.
// sync: the abort word, then 64 flag words per synchronisation group; `base` is what the
// flags read when the kernel starts.
// XP: the kernel computes the input projection itself, gx_t = x_t W_ih^T + b_ih, from the
// layer input xin (blocks of B x width per step) with its 48 rows of W_ih resident in LDS too;
// that part of a step does not depend on the other workgroups and is done before the wait.
// The r and z gates then take one sum over both contractions; gx is not used.
template <int XNB>  // chunks of the layer input per wave (width <= 128 * XNB); 0: gx is given
__global__ void __launch_bounds__(PNT) __attribute__((amdgpu_waves_per_eu(1, 2)))
gru_fwd_persist_kernel(const float* __restrict__ W_hh, const float* __restrict__ b_hh, long s_rep,
                       const float* __restrict__ gx, long s_gx, float* __restrict__ hs, long s_hs, float* hx, long s_hx,
                       float* __restrict__ sv, long s_sv, int B, int H, int T, int groups, unsigned* sync, unsigned base,
                       unsigned spin_limit, unsigned* tickets, unsigned ticket_base, unsigned per_xcd,
                       const float* __restrict__ xin, long s_x, int width,
                       const float* __restrict__ W_ih, const float* __restrict__ b_ih) {
  extern __shared__ __attribute__((aligned(16))) float persist_lds[];
  constexpr bool XP = XNB > 0;
  constexpr int XB = XP ? XNB : 1;
  constexpr int NP = XP ? 4 : 3;             // planes of partial sums: r, z, q (+ the x part of n)
  const int wp = (H + PC - 1) / PC * PC + 4;
  const int wp2 = XP ? (width + PC - 1) / PC * PC + 4 : 0;
  float* wres = persist_lds;                 // [48][wp]
  float* red = wres + 48 * wp;               // [4][2][NP][4][64]
  float* wres2 = red + 4 * 2 * NP * 4 * 64;  // [48][wp2]
  int* lds_flag = reinterpret_cast<int*>(wres2 + 48 * wp2);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, rsel = wave >> 2;
  const int lr = lane & 15, lg = lane >> 4;
  const int NJ = H / PJ, RT = (B + PR - 1) / PR;
  unsigned* abort_w = sync;
  int vi;
  bool l2x;
  if (!persist_place(tickets, ticket_base, per_xcd, abort_w, lds_flag, vi, l2x)) return;
  int g, tx, ty, sg;
  persist_tile(vi, NJ, RT, groups, g, tx, ty, sg);
  const int j0 = tx * PJ, r0 = ty * PR;
  unsigned* flags = sync + 1 + sg * PF;
  __builtin_amdgcn_s_setprio(3);
  // the resident slices: rows q*16 + r = W_hh[q*H + j0 + r][:] (and the same rows of W_ih)
  load_resident(wres, wp, W_hh + g * s_rep, 48, H,
                [&](int row) { return ((long)(row >> 4) * H + j0 + (row & 15)) * H; });
  if (XP)
    load_resident(wres2, wp2, W_ih + g * s_rep, 48, width,
                  [&](int row) { return ((long)(row >> 4) * H + j0 + (row & 15)) * width; });
  const int j = j0 + lr;
  const int row = r0 + rsel * 16 + 4 * lg + kw;     // this thread's element of the tile
  const int rowc = min(row, B - 1);                 // loads are clamped, stores guarded
  const float* bh = b_hh + g * s_rep;
  float bias[3], biasx[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int q = 0; q < 3; ++q) bias[q] = bh[q * H + j];
  if (XP) {
#pragma unroll
    for (int q = 0; q < 3; ++q) biasx[q] = (b_ih + g * s_rep)[q * H + j];
  }
  float* hsg = hs + g * s_hs;
  float* hxg = hx + g * s_hx;                 // h_0 .. h_T as the workgroups exchange them
  const long xblk = xblock_words(B, H);
  const int rbx = (r0 + rsel * 16 < B ? r0 + rsel * 16 : r0) >> 4;  // this wave's row block (one beyond the batch: the tile's first)
  float hpv = hsg[(long)rowc * H + j];
  float4 xa[XB][2];  // this step's fragments of the layer input, loaded one step ahead
  float gxn[3] = {0.f, 0.f, 0.f};  // ... or its input projection
  if (XP) {
    fragment_loads<XB>(tile_rsrc(xin + g * s_x + (long)r0 * width), width, B - r0, kw, xa);
  } else {
    const float* gxr = gx + g * s_gx + (long)rowc * 3 * H;
#pragma unroll
    for (int q = 0; q < 3; ++q) gxn[q] = gxr[q * H + j];
  }
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    // what does not depend on the recurrence is computed in front of the wait
    float gxv[3] = {gxn[0], gxn[1], gxn[2]};
    floatx4 acc[2][3], accx[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int q = 0; q < 3; ++q) acc[i][q] = (floatx4){0.f, 0.f, 0.f, 0.f};
      accx[i] = (floatx4){0.f, 0.f, 0.f, 0.f};
    }
    if (XP) {
      fragment_mfmas<3, XB>(wres2, wp2, width, kw, xa, acc);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        accx[i] = acc[i][2];  // n keeps its two parts apart: n = tanh(x part + r * (h part))
        acc[i][2] = (floatx4){0.f, 0.f, 0.f, 0.f};
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (t > 0 && !group_wait(flags, NJ, base + (unsigned)t, abort_w, spin_limit, lds_flag)) return;
    resident_contraction_x<3, 4>(wres, wp, tile_rsrc(hxg + (long)t * xblk), H, rbx, acc, [&]() {
      // step t+1's layer input (or input projection) travels during this step's product
      if (XP) {
        fragment_loads<XB>(tile_rsrc(xin + g * s_x + ((long)min(t + 1, T - 1) * B + r0) * width), width, B - r0, kw, xa);
      } else {
        const float* gxr = gx + g * s_gx + ((long)min(t + 1, T - 1) * B + rowc) * 3 * H;
#pragma unroll
        for (int q = 0; q < 3; ++q) gxn[q] = gxr[q * H + j];
      }
    });
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
      for (int q = 0; q < 3; ++q)
        red[(((kw * 2 + rsel) * NP + q) * 4 + v) * 64 + lane] = acc[0][q][v] + acc[1][q][v];
      if (XP) red[(((kw * 2 + rsel) * NP + 3) * 4 + v) * 64 + lane] = accx[0][v] + accx[1][v];
    }
    __syncthreads();
    float gh[NP];
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      const int o = ((rsel * NP + q) * 4 + kw) * 64 + lane;
      constexpr int PL = 2 * NP * 256;  // one wave quarter's partial sums
      gh[q] = (red[o] + red[o + PL]) + (red[o + 2 * PL] + red[o + 3 * PL]);
    }
    const float r = sigm_p(gxv[0] + biasx[0] + (gh[0] + bias[0]));
    const float z = sigm_p(gxv[1] + biasx[1] + (gh[1] + bias[1]));
    const float qv = gh[2] + bias[2];
    const float n = tanhf((XP ? gh[NP - 1] + biasx[2] : gxv[2]) + r * qv);
    const float hn = (1.0f - z) * n + z * hpv;
    if (row < B) {
      hsg[((long)(t + 1) * B + row) * H + j] = hn;
      st_dev(hxg + (long)(t + 1) * xblk + xoff(row, (H + PC - 1) / PC, j), hn, l2x);
      float* svr = sv + g * s_sv + ((long)t * B + row) * 4 * H;
      svr[j] = r;
      svr[H + j] = z;
      svr[2 * H + j] = n;
      svr[3 * H + j] = qv;
    }
    hpv = hn;
    group_signal(flags + tx, base + (unsigned)t + 1u, l2x);  // (its barrier also separates the reads of red from the next step's writes)
  }
}

// Backward: steps t = t_hi-1 down to t_lo.  The workgroup's resident slice is 16 columns of
// W_hh (3H x H), kept transposed in LDS (16 rows of 3H, unit stride along the contraction).  dgh and
// dgx hold the gate gradients of all steps (blocks of B x 3H); block t+1 of dgh is the
// contraction operand of step t (none at t = T-1).  D holds dh_{t_hi} * z_{t_hi} on entry (the
// head's gradient when t_hi == T; d_zero: it is zero and D is not read) and dh_{t_lo} * z_{t_lo}
// on exit.  above: per-step gradient from the layer above (blocks of B x H) or nullptr.
//
// dWp (nullable, H <= 512): the workgroup also accumulates its share of the recurrent weight
// gradient over the steps of the launch, dW_hh[q*H + j0 + m][:] += sum over its 32 batch rows
// of dgh_t[row][q*H + j0 + m] * h_{t-1}[row][:], and stores it at the end to
// dWp[(g * RT + ty)][3H][H] (one partial sum per batch-row tile; the caller adds the RT of
// them).  That work does not depend on the other workgroups: it is done between counting
// the step in and waiting for the next one, in the time the chain of waits leaves idle.
// Wave w owns columns 64w .. 64w+63 and all 48 gate rows (3 x 4 accumulator tiles); tile
// (mt, jt) holds the columns 64w + 4*lane%16 + jt, so that a lane fetches h as one float4 per
// batch row and stores its results as float4s.
//
// Register cap: two waves of this kernel share a SIMD, and at 256 registers each they would own
// its whole register file, so that no wave of any other kernel (the merge of the other stream,
// a short kernel queued behind) could start on a CU before this launch has ended.  The
// attribute counts in halves of the unified VGPR/AGPR file on this target: 124 caps the wave at
// 248 registers (2 dwords per lane are spilled), which leaves 16 per SIMD for a co-tenant.
__global__ void __launch_bounds__(PNT) __attribute__((amdgpu_num_vgpr(124)))
gru_bwd_persist_kernel(const float* __restrict__ W_hh, long s_rep, float* __restrict__ dgh, float* dghx, long s_dghx,
                       float* __restrict__ dgx, long s_dg,
                       float* __restrict__ D, long s_D, int d_zero, const float* __restrict__ above, long s_above,
                       const float* __restrict__ sv, long s_sv, const float* __restrict__ hs, long s_hs,
                       int B, int H, int T, int t_hi, int t_lo, int groups, unsigned* sync, unsigned base,
                       unsigned spin_limit, unsigned* tickets, unsigned ticket_base, unsigned per_xcd,
                       float* __restrict__ dWp, float* __restrict__ dbp) {
  extern __shared__ __attribute__((aligned(16))) float persist_lds[];
  const int H3 = 3 * H;
  const int wp = (H3 + PC - 1) / PC * PC + 4;
  float* wres = persist_lds;                 // [16][wp]
  float* red = wres + 16 * wp;               // [4][2][4][64]
  float* stage = red + 4 * 2 * 4 * 64;       // [32][SP]: the step's dgh tile, batch row x gate row
  int* lds_flag = reinterpret_cast<int*>(stage + PR * SP);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, rsel = wave >> 2;
  const int lr = lane & 15, lg = lane >> 4;
  const int NJ = H / PJ, RT = (B + PR - 1) / PR;
  unsigned* abort_w = sync;
  int vi;
  bool l2x;
  if (!persist_place(tickets, ticket_base, per_xcd, abort_w, lds_flag, vi, l2x)) return;
  int g, tx, ty, sg;
  persist_tile(vi, NJ, RT, groups, g, tx, ty, sg);
  const int j0 = tx * PJ, r0 = ty * PR;
  unsigned* flags = sync + 1 + sg * PF;
  __builtin_amdgcn_s_setprio(3);
  // weight-gradient share: this lane's 4 columns (clamped: results outside H are not stored)
  const int wn = 64 * wave + 4 * lr;
  const bool wn_ok = dWp != nullptr && wn < H;
  const int wnc = wn < H ? wn : 0;
  floatx4 dw[3][4];
#pragma unroll
  for (int mt = 0; mt < 3; ++mt)
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) dw[mt][jt] = (floatx4){0.f, 0.f, 0.f, 0.f};
  {
    // wres[m][k] = W_hh[k][j0 + m]: 64-byte pieces of 3H rows, transposed on the way into LDS
    const float* Wg = W_hh + g * s_rep + j0;
    for (int u = tid; u < H3 * 4; u += PNT) {
      const int k = u >> 2, c4 = u & 3;
      const float4 v = *reinterpret_cast<const float4*>(Wg + (long)k * H + 4 * c4);
      wres[(4 * c4 + 0) * wp + k] = v.x;
      wres[(4 * c4 + 1) * wp + k] = v.y;
      wres[(4 * c4 + 2) * wp + k] = v.z;
      wres[(4 * c4 + 3) * wp + k] = v.w;
    }
    const int padk = wp - 4 - H3;  // zero columns up to the next multiple of the chunk
    for (int u = tid; u < 16 * padk; u += PNT) wres[(u / padk) * wp + H3 + u % padk] = 0.f;
  }
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};  // this thread's da_r, da_z, da_n, dq summed over the steps
  const int j = j0 + lr;
  const int row = r0 + rsel * 16 + 4 * lg + kw;
  const int rowc = min(row, B - 1);
  float* Dg = D + g * s_D;
  float dcar = d_zero ? 0.f : Dg[(long)rowc * H + j];  // dh_{t+1} * z_{t+1}, carried in a register
  float* dghg = dgh ? dgh + g * s_dg : nullptr;  // row-major, for later launches (nullptr: nobody reads it)
  float* dgxg = dghx + g * s_dghx;               // the gate gradients as the workgroups exchange them
  const long xblk = xblock_words(B, H3);
  const int nchx = (H3 + PC - 1) / PC;
  const int rbx = (r0 + rsel * 16 < B ? r0 + rsel * 16 : r0) >> 4;
  __syncthreads();
  int it = 0;
  for (int t = t_hi - 1; t >= t_lo; --t, ++it) {
    // (loaded in front of the wait: one step ahead they would cost this kernel, which is held at 248
    // registers, spills - measured, 400 -> 620 us)
    const long e = ((long)t * B + rowc) * H + j;
    const float* svr = sv + g * s_sv + ((long)t * B + rowc) * 4 * H;
    const float r = svr[j], z = svr[H + j], n = svr[2 * H + j], q = svr[3 * H + j];
    const float hp = hs[g * s_hs + e];
    const float ab = above ? above[g * s_above + e] : 0.f;
    if (it > 0 && !group_wait(flags, NJ, base + (unsigned)it, abort_w, spin_limit, lds_flag)) return;
    floatx4 acc[2][1];
    acc[0][0] = (floatx4){0.f, 0.f, 0.f, 0.f};
    acc[1][0] = (floatx4){0.f, 0.f, 0.f, 0.f};
    if (t + 1 < T)  // uniform over the grid
      resident_contraction_x<1, 12>(wres, wp, tile_rsrc(dgxg + (long)(t + 1) * xblk), H3, rbx, acc, []() {});
#pragma unroll
    for (int v = 0; v < 4; ++v) red[((kw * 2 + rsel) * 4 + v) * 64 + lane] = acc[0][0][v] + acc[1][0][v];
    __syncthreads();
    const int o = (rsel * 4 + kw) * 64 + lane;
    const float rec = (red[o] + red[o + 512]) + (red[o + 1024] + red[o + 1536]);
    const float dh = (dcar + ab) + rec;
    const float dn = dh * (1.0f - z);
    const float dz = dh * (hp - n);
    const float da_n = dn * (1.0f - n * n);
    const float dq = da_n * r;
    const float da_r = da_n * q * r * (1.0f - r);
    const float da_z = dz * z * (1.0f - z);
    if (row < B) {
      float* ox = dgx + g * s_dg + ((long)t * B + row) * H3;
      ox[j] = da_r;
      ox[H + j] = da_z;
      ox[2 * H + j] = da_n;
      float* oe = dgxg + (long)t * xblk;
      st_dev(oe + xoff(row, nchx, j), da_r, l2x);
      st_dev(oe + xoff(row, nchx, H + j), da_z, l2x);
      st_dev(oe + xoff(row, nchx, 2 * H + j), dq, l2x);
      if (dghg) {
        float* oh = dghg + ((long)t * B + row) * H3;
        oh[j] = da_r;
        oh[H + j] = da_z;
        oh[2 * H + j] = dq;
      }
    }
    dcar = dh * z;
    if (row < B) {
      bsum[0] += da_r;
      bsum[1] += da_z;
      bsum[2] += da_n;
      bsum[3] += dq;
    }
    float4 hv[8];
    if (dWp) {  // uniform
      // rows beyond the batch contribute nothing: their staged gradients are zero, their h is
      // read from a valid row
      const bool rv = row < B;
      float* st = stage + (rsel * 16 + 4 * lg + kw) * SP + lr;
      st[0] = rv ? da_r : 0.f;
      st[16] = rv ? da_z : 0.f;
      st[32] = rv ? dq : 0.f;
      const float* hrow = hs + g * s_hs + (long)t * B * H + wnc;
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8)
        hv[s8] = *reinterpret_cast<const float4*>(hrow + (long)min(r0 + 4 * s8 + lg, B - 1) * H);
    }
    group_signal(flags + tx, base + (unsigned)it + 1u, l2x);  // (its barrier also publishes the staged tile to the workgroup)
    if (dWp) {
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8) {
        float am[3];
#pragma unroll
        for (int mt = 0; mt < 3; ++mt) am[mt] = stage[(4 * s8 + lg) * SP + mt * 16 + lr];
#pragma unroll
        for (int mt = 0; mt < 3; ++mt) {
          dw[mt][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(am[mt], hv[s8].x, dw[mt][0], 0, 0, 0);
          dw[mt][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(am[mt], hv[s8].y, dw[mt][1], 0, 0, 0);
          dw[mt][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(am[mt], hv[s8].z, dw[mt][2], 0, 0, 0);
          dw[mt][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(am[mt], hv[s8].w, dw[mt][3], 0, 0, 0);
        }
      }
    }
  }
  if (row < B) Dg[(long)row * H + j] = dcar;
  if (dbp) {  // uniform
    // bias gradients: sums over the tile's 32 batch rows, in row order; one partial sum per
    // batch-row tile: [b_ih: r | z | n][b_hh: r | z | q], 6H floats
    __syncthreads();
    float* bs = stage;  // [32][64]: row, then 4 sums x 16 units
#pragma unroll
    for (int i = 0; i < 4; ++i) bs[(rsel * 16 + 4 * lg + kw) * 64 + i * 16 + lr] = bsum[i];
    __syncthreads();
    if (tid < 64) {
      float tot = 0.f;
      for (int r32 = 0; r32 < PR; ++r32) tot += bs[r32 * 64 + tid];
      const int i = tid >> 4, jj = j0 + (tid & 15);
      float* out = dbp + (long)(g * RT + ty) * 6 * H;
      if (i == 0) out[jj] = out[H3 + jj] = tot;
      if (i == 1) out[H + jj] = out[H3 + H + jj] = tot;
      if (i == 2) out[2 * H + jj] = tot;
      if (i == 3) out[H3 + 2 * H + jj] = tot;
    }
  }
  if (wn_ok) {
    // accumulator register v of tile (mt, jt): gate row mt*16 + 4*lg + v, column wn + jt
    float* out = dWp + ((long)(g * RT + ty) * H3) * H;
#pragma unroll
    for (int mt = 0; mt < 3; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        *reinterpret_cast<float4*>(out + ((long)mt * H + j0 + 4 * lg + v) * H + wn) =
            make_float4(dw[mt][0][v], dw[mt][1][v], dw[mt][2][v], dw[mt][3][v]);
  }
}

// ---------------------------------------------------------------------------- bf16 operands
// The same scheme with v_mfma_f32_16x16x32_bf16 on the bf16 copies of W_hh and of the exchanged
// activations (every operand is the nearest-even bf16 rounding of the fp32 value; accumulation,
// cell math and everything stored for later use stay fp32).  A workgroup owns 32 batch rows x
// 32 hidden units.  Its slice of the weights (forward: 96 gate rows x H; backward: 32 rows of
// W_hh^T x 3H; 192 KB at H = 1024) stays in REGISTERS for the whole launch: the contraction is
// cut into 32-wide chunks, wave w owns the chunks w, w + 8, .. with all the column blocks, i.e.
// up to 24 B-operand fragments of 16 bytes per lane.  Per step a wave fetches only its own A
// fragments (16 bytes per lane per chunk and row block); the 8 partial sums of every output
// meet in LDS.  MFMA 16x16x32 lane layout: A lane l holds A[m = l%16][k = 8*(l/16) .. +7],
// B lane l holds B[k = 8*(l/16) .. +7][n = l%16], accumulator as for 16x16x4.
// Epilogue: thread t owns batch row t/16 and the two units 2*(t%16), +1 of the tile, so that
// bf16 values are stored in pairs.
//
// Layout of the exchanged operand.  A wave's A fragment is 16 rows x 32 contraction indices,
// 16 bytes per lane.  Read from a row-major matrix that is 64 bytes of each of 16 rows, half a
// cache line per row, and a CU then takes 5.3 us to fetch the 196 KB a backward step needs
// (measured: the same whether the lines come from L2 or past it, whatever the cache policy of the
// load and however few CUs read at once), against 1.9 us when every load instruction reads whole
// lines.  So the exchange buffers are kept fragment-major: per step, row block (16 batch rows) and
// chunk, the 1 KB that one load instruction reads, lane l's 16 bytes at byte 16 l (lane l holds row
// l % 16, contraction indices 8 (l / 16) .. + 7 of the chunk).  A workgroup's 32 units are exactly
// one chunk (per gate), so a workgroup writes whole fragments and nobody else writes into them.
// Rows of the last row block beyond the batch are never written: what a consumer reads there goes
// into output rows that are never stored.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

constexpr int QJ = 32;       // hidden units per workgroup
constexpr int TP = 40;       // pitch (bf16) of a staged transposed row of 32 batch rows

__device__ __forceinline__ bf16x8 ld_frag(const __bf16* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4_t*>(p));
}
__device__ __forceinline__ bf16x8 ld_frag_dev(__amdgpu_buffer_rsrc_t rs, int byte_off) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs, byte_off, 0, 16 /* sc1 */));
}
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  const __bf16 x = (__bf16)a, y = (__bf16)b;
  return (unsigned)__builtin_bit_cast(unsigned short, x) | ((unsigned)__builtin_bit_cast(unsigned short, y) << 16);
}
__device__ __forceinline__ void st_dev_u32(void* p, unsigned v, bool l2x) {
  if (l2x) __hip_atomic_store(reinterpret_cast<unsigned*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(reinterpret_cast<unsigned*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Element offset, inside a step's block of a fragment-major exchange buffer with nch chunks per
// row, of (row, chunk c, index u within the chunk)
__device__ __forceinline__ long xfrag(int row, int nch, int c, int u) {
  return ((long)(row >> 4) * nch + c) * 512 + (((u >> 3) << 4) + (row & 15)) * 8 + (u & 7);
}

// What a launch reads once (input projections, saved gates, the gradient from above) or leaves for
// later launches (saved gates, h, the copies for the GEMMs) goes past the L2 with the non-temporal
// hint: the L2 is where the exchanged operand lives between its stores and its loads.
typedef float f2nt_t __attribute__((ext_vector_type(2)));
typedef unsigned u4nt_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float2 ld2_nt(const float* p) {
  const f2nt_t v = __builtin_nontemporal_load(reinterpret_cast<const f2nt_t*>(p));
  return make_float2(v.x, v.y);
}
__device__ __forceinline__ void st2_nt(float* p, float2 v) {
  const f2nt_t t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<f2nt_t*>(p));
}
__device__ __forceinline__ void st_u32_nt(void* p, unsigned v) { __builtin_nontemporal_store(v, reinterpret_cast<unsigned*>(p)); }
__device__ __forceinline__ void st16_nt(void* p, uint4 v) {
  const u4nt_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u4nt_t*>(p));
}

// Forward.  Wb: bf16 W_hh [3H][H]; hx: bf16 h_0 .. h_T fragment-major (blocks of 16 ceil(B/16) x H,
// h_0 given), the exchanged operand; hb: the same row-major (blocks of B x H; written, not read);
// hs: the same in fp32; hT (nullable): bf16 transposed copy [H][ld_hT], column (t+1)*B + row.
// NCF: chunks per wave (H <= 256 * NCF).
template <int NCF>
__global__ void __launch_bounds__(PNT) __attribute__((amdgpu_waves_per_eu(1, 2)))
gru_fwd_persist_bf16_kernel(const __bf16* __restrict__ Wb, long s_wb, const float* __restrict__ b_hh, long s_rep,
                            const float* __restrict__ gx, long s_gx, float* __restrict__ hs, long s_hs,
                            __bf16* __restrict__ hb, long s_hb, __bf16* hx, long s_hx, float* __restrict__ sv, long s_sv, __bf16* __restrict__ hT, long ld_hT,
                            long s_hT, int B, int H, int T, int groups, unsigned* sync, unsigned base,
                            unsigned spin_limit, unsigned* tickets, unsigned ticket_base, unsigned per_xcd) {
  extern __shared__ __attribute__((aligned(16))) float persist_lds[];
  float* red = persist_lds;                                     // [8][2][6][4][64]
  __bf16* tt = reinterpret_cast<__bf16*>(red + 8 * 12 * 256);   // [32 units][TP]
  int* lds_flag = reinterpret_cast<int*>(tt + QJ * TP);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int NJ = H / QJ, RT = (B + PR - 1) / PR;
  unsigned* abort_w = sync;
  int vi;
  bool l2x;
  if (!persist_place(tickets, ticket_base, per_xcd, abort_w, lds_flag, vi, l2x)) return;
  int g, tx, ty, sg;
  persist_tile(vi, NJ, RT, groups, g, tx, ty, sg);
  const int j0 = tx * QJ, r0 = ty * PR;
  unsigned* flags = sync + 1 + sg * PF;
  __builtin_amdgcn_s_setprio(3);
  const int nch = H / PC;
  // resident fragments: chunk wave + 8i, column block cb = 2q + half: rows q*H + j0 + 16*half + lr
  bf16x8 wf[NCF][6];
#pragma unroll
  for (int i = 0; i < NCF; ++i) {
    const int c = wave + 8 * i;
#pragma unroll
    for (int cb = 0; cb < 6; ++cb) {
      const long wrow = (long)(cb >> 1) * H + j0 + 16 * (cb & 1) + lr;
      const bf16x8 v = ld_frag(Wb + g * s_wb + wrow * H + PC * (c < nch ? c : 0) + 8 * lg);
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      wf[i][cb] = c < nch ? v : zero;  // a chunk slot beyond the contraction multiplies by zero
    }
  }
  // epilogue element: row rl of the tile, units u0, u0 + 1
  const int rl = tid >> 4, u0 = 2 * (tid & 15);
  const int row = r0 + rl, rowc = min(row, B - 1);
  const int j = j0 + u0;
  const int ro = ((rl >> 4) * 6) * 256 + (rl & 3) * 64 + ((rl >> 2) & 3) * 16 + (u0 & 15);  // + cb * 256 + w * 3072
  const int half = u0 >> 4;
  float2 bias[3];
#pragma unroll
  for (int q = 0; q < 3; ++q) bias[q] = *reinterpret_cast<const float2*>(b_hh + g * s_rep + q * H + j);
  float* hsg = hs + g * s_hs;
  __bf16* hbg = hb + g * s_hb;
  __bf16* hxg = hx + g * s_hx;
  const long xblk = (long)((B + 15) / 16) * 16 * H;  // elements of a step's block of hx
  float2 hpv = *reinterpret_cast<const float2*>(hsg + (long)rowc * H + j);
  // A fragments: row blocks r0/16 + rb (one that lies beyond the batch is read from the tile's first)
  int aoff[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) aoff[rb] = (((r0 + rb * 16 < B ? r0 + rb * 16 : r0) >> 4) * nch) * 1024 + lane * 16;
  // The step's input projection is loaded one step ahead, behind the operand loads of the step
  // before: requested in front of the wait, it would sit between the polling wave and its view
  // of the flags (a wave's loads return in order, and these come from memory, not from the L2).
  float2 gxn[3];
  {
    const float* gxr = gx + g * s_gx + (long)rowc * 3 * H + j;
#pragma unroll
    for (int q = 0; q < 3; ++q) gxn[q] = ld2_nt(gxr + q * H);
  }
  for (int t = 0; t < T; ++t) {
    float2 gxv[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) gxv[q] = gxn[q];
    if (t > 0 && !group_wait(flags, NJ, base + (unsigned)t, abort_w, spin_limit, lds_flag)) return;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(hxg + (long)t * xblk, 0, 0x7fffffff, 0x00020000);
    bf16x8 a[NCF][2];
#pragma unroll
    for (int i = 0; i < NCF; ++i) {
      const int c = wave + 8 * i;
      const int co = (c < nch ? c : 0) * 1024;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) a[i][rb] = ld_frag_dev(rs, aoff[rb] + co);
    }
    __builtin_amdgcn_sched_barrier(0);
    {
      const float* gxr = gx + g * s_gx + ((long)min(t + 1, T - 1) * B + rowc) * 3 * H + j;
#pragma unroll
      for (int q = 0; q < 3; ++q) gxn[q] = ld2_nt(gxr + q * H);
    }
    floatx4 acc[2][6];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < 6; ++cb) acc[rb][cb] = (floatx4){0.f, 0.f, 0.f, 0.f};
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before anything waits for one
#pragma unroll
    for (int i = 0; i < NCF; ++i)
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 6; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i][rb], wf[i][cb], acc[rb][cb], 0, 0, 0);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < 6; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[(((wave * 2 + rb) * 6 + cb) * 4 + v) * 64 + lane] = acc[rb][cb][v];
    __syncthreads();
    float2 gh[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const float* rp = red + ro + (2 * q + half) * 256;
      float2 p[8];
#pragma unroll
      for (int w = 0; w < 8; ++w) p[w] = *reinterpret_cast<const float2*>(rp + w * 3072);
      gh[q].x = (((p[0].x + p[1].x) + (p[2].x + p[3].x)) + ((p[4].x + p[5].x) + (p[6].x + p[7].x))) + bias[q].x;
      gh[q].y = (((p[0].y + p[1].y) + (p[2].y + p[3].y)) + ((p[4].y + p[5].y) + (p[6].y + p[7].y))) + bias[q].y;
    }
    const float r0v = sigm_fast(gxv[0].x + gh[0].x), r1v = sigm_fast(gxv[0].y + gh[0].y);
    const float z0v = sigm_fast(gxv[1].x + gh[1].x), z1v = sigm_fast(gxv[1].y + gh[1].y);
    const float n0v = tanh_fast(gxv[2].x + r0v * gh[2].x), n1v = tanh_fast(gxv[2].y + r1v * gh[2].y);
    const float2 hn = make_float2((1.0f - z0v) * n0v + z0v * hpv.x, (1.0f - z1v) * n1v + z1v * hpv.y);
    if (row < B) {
      const long e = ((long)(t + 1) * B + row) * H + j;
      const unsigned hp2 = pack_bf16(hn.x, hn.y);
      st_dev_u32(hxg + (long)(t + 1) * xblk + xfrag(row, nch, tx, u0), hp2, l2x);
      st2_nt(hsg + e, hn);
      st_u32_nt(hbg + e, hp2);
      float* svr = sv + g * s_sv + ((long)t * B + row) * 4 * H + j;
      st2_nt(svr, make_float2(r0v, r1v));
      st2_nt(svr + H, make_float2(z0v, z1v));
      st2_nt(svr + 2 * H, make_float2(n0v, n1v));
      st2_nt(svr + 3 * H, gh[2]);
    }
    if (hT) {
      tt[u0 * TP + rl] = (__bf16)hn.x;
      tt[(u0 + 1) * TP + rl] = (__bf16)hn.y;
    }
    hpv = hn;
    group_signal(flags + tx, base + (unsigned)t + 1u, l2x);  // (its barrier also separates the reads of red from the next step's writes)
    if (hT && tid >= PNT - 128) {
      // 64-byte row segments of the transposed copy, 16 bytes per thread (the last two waves: the
      // first one polls the flags next, and would see them only behind its own stores)
      const int u = (tid - (PNT - 128)) >> 2, part = tid & 3;
      if (r0 + 8 * part < B)  // B is a multiple of 8: a piece of 8 rows is all in or all out
        st16_nt(hT + g * s_hT + (long)(j0 + u) * ld_hT + (long)(t + 1) * B + r0 + 8 * part,
                *reinterpret_cast<const uint4*>(tt + u * TP + 8 * part));
    }
  }
}

// Backward.  WT: bf16 W_hh^T [H][3H]; dghx: bf16 gate gradients of all steps, fragment-major
// (blocks of 16 ceil(B/16) x 3H), the exchanged operand; dgxb: bf16 dgx row-major; dgxT / dghT: bf16 transposed copies
// [3H][ld_T], column t*B + row; dbp: partial bias-gradient sums [(g*RT + ty)][6H] (b_ih | b_hh).
// D: dh_T * z_T on entry (the head's gradient; d_zero: zero, D is not read), dh_0 * z_0 on exit.  NCB: chunks per wave
// (3H <= 256 * NCB).  The fragments of the first half of a wave's chunks stay in registers,
// those of the second half in LDS (each wave reads back only its own): with all of them in
// registers the two waves of a SIMD would fill its register file, and no wave of any other
// kernel (a merge on the second stream) could ever share the CU.
template <int NCB>
__global__ void __launch_bounds__(PNT) __attribute__((amdgpu_waves_per_eu(1, 2)))
gru_bwd_persist_bf16_kernel(const __bf16* __restrict__ WT, long s_wt, __bf16* dghx, long s_dgh, long s_dgb, float* __restrict__ D,
                            long s_D, int d_zero, const float* __restrict__ above, long s_above, const float* __restrict__ sv,
                            long s_sv, const float* __restrict__ hs, long s_hs, __bf16* __restrict__ dgxb,
                            __bf16* __restrict__ dgxT, __bf16* __restrict__ dghT, long ld_T, long s_T,
                            float* __restrict__ dbp, int B, int H, int T, int groups, unsigned* sync, unsigned base,
                            unsigned spin_limit, unsigned* tickets, unsigned ticket_base, unsigned per_xcd) {
  extern __shared__ __attribute__((aligned(16))) float persist_lds[];
  constexpr int NCR = NCB / 2, NCL = NCB - NCR;                 // chunks in registers / in LDS
  float* red = persist_lds;                                     // [8][2][2][4][64]
  __bf16* tt = reinterpret_cast<__bf16*>(red + 8 * 4 * 256);    // [da_r | da_z | da_n | dq][32 units][TP]
  u32x4_t* wl = reinterpret_cast<u32x4_t*>(tt + 4 * QJ * TP);   // [8 waves][NCL][2][64 lanes] fragments
  int* lds_flag = reinterpret_cast<int*>(wl + 8 * NCL * 2 * 64);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int NJ = H / QJ, RT = (B + PR - 1) / PR;
  unsigned* abort_w = sync;
  int vi;
  bool l2x;
  if (!persist_place(tickets, ticket_base, per_xcd, abort_w, lds_flag, vi, l2x)) return;
  int g, tx, ty, sg;
  persist_tile(vi, NJ, RT, groups, g, tx, ty, sg);
  const int j0 = tx * QJ, r0 = ty * PR;
  unsigned* flags = sync + 1 + sg * PF;
  __builtin_amdgcn_s_setprio(3);
  const int H3 = 3 * H;
  const int nch = H3 / PC;
  // resident fragments: chunk wave + 8i, column block = half: rows j0 + 16*half + lr of W_hh^T
  bf16x8 wf[NCR][2];
#pragma unroll
  for (int i = 0; i < NCB; ++i) {
    const int c = wave + 8 * i;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const bf16x8 v = ld_frag(WT + g * s_wt + (long)(j0 + 16 * cb + lr) * H3 + PC * (c < nch ? c : 0) + 8 * lg);
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      const bf16x8 f = c < nch ? v : zero;
      if (i < NCR)
        wf[i][cb] = f;
      else
        wl[((wave * NCL + (i - NCR)) * 2 + cb) * 64 + lane] = __builtin_bit_cast(u32x4_t, f);
    }
  }
  const int rl = tid >> 4, u0 = 2 * (tid & 15);
  const int row = r0 + rl, rowc = min(row, B - 1);
  const int j = j0 + u0;
  const int ro = ((rl >> 4) * 2 + (u0 >> 4)) * 256 + (rl & 3) * 64 + ((rl >> 2) & 3) * 16 + (u0 & 15);  // + w * 1024
  float* Dg = D + g * s_D;
  float2 dcar = make_float2(0.f, 0.f);
  if (!d_zero) dcar = *reinterpret_cast<const float2*>(Dg + (long)rowc * H + j);
  __bf16* dghg = dghx + g * s_dgh;
  const long xblk = (long)((B + 15) / 16) * 16 * H3;  // elements of a step's block of dghx
  float2 bsum[4] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};  // da_r, da_z, da_n, dq over the steps
  int aoff[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) aoff[rb] = (((r0 + rb * 16 < B ? r0 + rb * 16 : r0) >> 4) * nch) * 1024 + lane * 16;
  // The step's saved gates, h and the gradient from above are loaded one step ahead, behind the
  // operand loads of the step before (see the forward kernel: in front of the wait they would
  // delay the polling wave's view of the flags by a trip to memory).
  float2 nr, nz, nn, nq, nhp, nab;
  auto prefetch = [&](int tn) {
    const long e = ((long)tn * B + rowc) * H + j;
    const float* svr = sv + g * s_sv + ((long)tn * B + rowc) * 4 * H + j;
    nr = ld2_nt(svr), nz = ld2_nt(svr + H);
    nn = ld2_nt(svr + 2 * H), nq = ld2_nt(svr + 3 * H);
    nhp = ld2_nt(hs + g * s_hs + e);
    nab = above ? ld2_nt(above + g * s_above + e) : make_float2(0.f, 0.f);
  };
  prefetch(T - 1);
  int it = 0;
  for (int t = T - 1; t >= 0; --t, ++it) {
    const float2 r = nr, z = nz, n = nn, q = nq, hp = nhp, ab = nab;
    if (it > 0 && !group_wait(flags, NJ, base + (unsigned)it, abort_w, spin_limit, lds_flag)) return;
    floatx4 acc[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) acc[rb][cb] = (floatx4){0.f, 0.f, 0.f, 0.f};
    if (t + 1 < T) {  // uniform over the grid
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(dghg + (long)(t + 1) * xblk, 0, 0x7fffffff,
                                                                          0x00020000);
      bf16x8 a[NCB][2];
#pragma unroll
      for (int i = 0; i < NCB; ++i) {
        const int c = wave + 8 * i;
        const int co = (c < nch ? c : 0) * 1024;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) a[i][rb] = ld_frag_dev(rs, aoff[rb] + co);
      }
      __builtin_amdgcn_sched_barrier(0);
      prefetch(max(t - 1, 0));
      __builtin_amdgcn_sched_barrier(0);  // every load is issued before anything waits for one
#pragma unroll
      for (int i = 0; i < NCB; ++i) {
        bf16x8 w2[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
          w2[cb] = i < NCR ? wf[i < NCR ? i : 0][cb]
                           : __builtin_bit_cast(bf16x8, wl[((wave * NCL + (i - NCR)) * 2 + cb) * 64 + lane]);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb)
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i][rb], w2[cb], acc[rb][cb], 0, 0, 0);
      }
    } else {
      prefetch(max(t - 1, 0));
    }
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[(((wave * 2 + rb) * 2 + cb) * 4 + v) * 64 + lane] = acc[rb][cb][v];
    __syncthreads();
    float2 p[8];
#pragma unroll
    for (int w = 0; w < 8; ++w) p[w] = *reinterpret_cast<const float2*>(red + ro + w * 1024);
    const float recx = ((p[0].x + p[1].x) + (p[2].x + p[3].x)) + ((p[4].x + p[5].x) + (p[6].x + p[7].x));
    const float recy = ((p[0].y + p[1].y) + (p[2].y + p[3].y)) + ((p[4].y + p[5].y) + (p[6].y + p[7].y));
    const float2 dh = make_float2((dcar.x + ab.x) + recx, (dcar.y + ab.y) + recy);
    const float2 dn = make_float2(dh.x * (1.0f - z.x), dh.y * (1.0f - z.y));
    const float2 dz = make_float2(dh.x * (hp.x - n.x), dh.y * (hp.y - n.y));
    const float2 da_n = make_float2(dn.x * (1.0f - n.x * n.x), dn.y * (1.0f - n.y * n.y));
    const float2 dq = make_float2(da_n.x * r.x, da_n.y * r.y);
    const float2 da_r = make_float2(da_n.x * q.x * r.x * (1.0f - r.x), da_n.y * q.y * r.y * (1.0f - r.y));
    const float2 da_z = make_float2(dz.x * z.x * (1.0f - z.x), dz.y * z.y * (1.0f - z.y));
    if (row < B) {
      const long o = ((long)t * B + row) * H3 + j;
      const unsigned pr = pack_bf16(da_r.x, da_r.y), pz = pack_bf16(da_z.x, da_z.y);
      const long ox3 = (long)t * xblk + xfrag(row, nch, tx, u0);  // gate q: chunk q H/32 + tx
      st_dev_u32(dghg + ox3, pr, l2x);
      st_dev_u32(dghg + ox3 + (long)(H / PC) * 512, pz, l2x);
      st_dev_u32(dghg + ox3 + (long)(2 * H / PC) * 512, pack_bf16(dq.x, dq.y), l2x);
      __bf16* ox = dgxb + g * s_dgb + o;
      st_u32_nt(ox, pr);
      st_u32_nt(ox + H, pz);
      st_u32_nt(ox + 2 * H, pack_bf16(da_n.x, da_n.y));
      bsum[0].x += da_r.x; bsum[0].y += da_r.y;
      bsum[1].x += da_z.x; bsum[1].y += da_z.y;
      bsum[2].x += da_n.x; bsum[2].y += da_n.y;
      bsum[3].x += dq.x;   bsum[3].y += dq.y;
    }
    // the four distinct gate-gradient blocks, staged for the transposed copies
    tt[(0 * QJ + u0) * TP + rl] = (__bf16)da_r.x;
    tt[(0 * QJ + u0 + 1) * TP + rl] = (__bf16)da_r.y;
    tt[(1 * QJ + u0) * TP + rl] = (__bf16)da_z.x;
    tt[(1 * QJ + u0 + 1) * TP + rl] = (__bf16)da_z.y;
    tt[(2 * QJ + u0) * TP + rl] = (__bf16)da_n.x;
    tt[(2 * QJ + u0 + 1) * TP + rl] = (__bf16)da_n.y;
    tt[(3 * QJ + u0) * TP + rl] = (__bf16)dq.x;
    tt[(3 * QJ + u0 + 1) * TP + rl] = (__bf16)dq.y;
    dcar = make_float2(dh.x * z.x, dh.y * z.y);
    group_signal(flags + tx, base + (unsigned)it + 1u, l2x);
    // transposed copies [gate unit][t*B + row] as 64-byte row segments, 16 bytes per piece:
    // dgx^T = (da_r, da_z, da_n), dgh^T = (da_r, da_z, dq).  512 pieces, by the waves 1 .. 7: wave
    // 0 polls the flags next, and would see them only behind its own stores
    for (int idx = tid - 64; idx >= 0 && idx < PNT; idx += PNT - 64) {
      const int blk = idx >> 7, u = (idx >> 2) & 31, part = idx & 3;
      if (r0 + 8 * part < B) {  // B is a multiple of 8
        const uint4 v = *reinterpret_cast<const uint4*>(tt + (blk * QJ + u) * TP + 8 * part);
        const int gate = blk == 3 ? 2 : blk;
        const long o = g * s_T + (long)(gate * H + j0 + u) * ld_T + (long)t * B + r0 + 8 * part;
        if (blk != 3) st16_nt(dgxT + o, v);
        if (blk != 2) st16_nt(dghT + o, v);
      }
    }
  }
  if (row < B) *reinterpret_cast<float2*>(Dg + (long)row * H + j) = dcar;
  // bias gradients: sums over the tile's 32 batch rows, in row order
  __syncthreads();
  float* bs = red;  // [32 rows][4 sums][32 units]
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<float2*>(bs + (rl * 4 + i) * QJ + u0) = bsum[i];
  __syncthreads();
  if (tid < 128) {
    float tot = 0.f;
    for (int r32 = 0; r32 < PR; ++r32) tot += bs[r32 * 128 + tid];
    const int i = tid >> 5, jj = j0 + (tid & 31);
    float* out = dbp + (long)(g * RT + ty) * 6 * H;
    if (i == 0) out[jj] = out[H3 + jj] = tot;
    if (i == 1) out[H + jj] = out[H3 + H + jj] = tot;
    if (i == 2) out[2 * H + jj] = tot;
    if (i == 3) out[H3 + 2 * H + jj] = tot;
  }
}

// How a launch places its workgroups (persist_place).  By ticket, with the exchange through the
// XCDs' L2s, when: the caller allows it; the launch has exactly one workgroup per CU of the device
// (a workgroup that needs more than half of a CU's LDS has a CU to itself, so each of the 8 XCDs
// receives cus / 8 of them); and the synchronisation groups divide evenly over the XCDs.
struct Placement { unsigned* tickets; unsigned ticket_base, per_xcd; };
int device_cus();
// ticket_launches: how many launches of this step have drawn tickets so far (counted here)
Placement placement(unsigned* sync, int sync_groups, long grid, size_t lds, bool device_scope, unsigned* ticket_launches) {
  const int cus = device_cus();
  if (device_scope || !ticket_launches || cus <= 0 || cus % 8 != 0 || grid != cus || sync_groups % 8 != 0 ||
      lds <= 80 * 1024)
    return Placement{nullptr, 0u, 0u};
  const unsigned per_xcd = (unsigned)(cus / 8);
  return Placement{sync + 1 + (size_t)sync_groups * PF, (*ticket_launches)++ * per_xcd, per_xcd};
}

int device_cus() {
  static int cus = -1;
  if (cus < 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return 0;
    cus = n;
  }
  return cus;
}

constexpr size_t kLdsLimit = 160 * 1024;
// forward: 48 rows of H (rounded up to the chunk) + 4 words, the partial sums, the flag;
// backward: 16 rows of 3H (rounded up) + 4 words and fewer partial sums: never more
size_t persist_lds_bytes(int H) {
  return ((size_t)48 * ((H + PC - 1) / PC * PC + 4) + 4 * 6 * 4 * 64 + 4) * sizeof(float);
}
// forward with the input projection: a fourth plane of partial sums and 48 rows of W_ih
size_t persist_xp_lds_bytes(int H, int width) {
  return ((size_t)48 * ((H + PC - 1) / PC * PC + 4) + 4 * 8 * 4 * 64 + (size_t)48 * ((width + PC - 1) / PC * PC + 4) +
          4) * sizeof(float);
}

}  // namespace

// One workgroup per CU and all of them resident: the grid may not exceed the CU count, and
// the resident slice plus the partial sums must fit the 160 KB of LDS.
bool gru_persist_supported(int B, int H, int groups) {
  if (H % 16 != 0 || H < 16 || B < 1 || groups < 1) return false;
  if (persist_lds_bytes(H) > kLdsLimit) return false;
  const long grid = (long)(H / PJ) * ((B + PR - 1) / PR) * groups;
  return grid <= device_cus();
}

// The backward kernel can accumulate dW_hh itself when 8 waves x 64 columns cover H.
bool gru_persist_dw_supported(int H) { return H <= 512; }

// Words of device memory the kernels synchronise through: the abort word + 64 flag words per group.
size_t gru_persist_sync_words(int B, int groups) { return (size_t)groups * ((B + PR - 1) / PR) * PF + 1 + 8; }

// How much every flag advances per time step of a launch.
unsigned gru_persist_count_per_step(int) { return 1u; }

// The forward kernel can do the input projection itself when the layer input is narrow enough
// for the 48 rows of W_ih to fit the LDS beside those of W_hh (at most 2 x 4 chunks of 32).
bool gru_persist_xproj_supported(int H, int width) {
  return width >= 16 && width % 16 == 0 && width <= 256 && persist_xp_lds_bytes(H, width) <= kLdsLimit;
}

size_t gru_persist_exchange_words(int B, int width) { return (size_t)xblock_words(B, width); }

hipError_t launch_gru_fwd_persist(const float* W_hh, const float* b_hh, long s_rep, const float* gx, long s_gx,
                                  float* hs, long s_hs, float* hx, long s_hx, float* sv, long s_sv, int B, int H, int T,
                                  int groups,
                                  unsigned* sync, unsigned base, unsigned spin_limit, const float* xin, long s_x,
                                  int width, const float* W_ih, const float* b_ih, bool device_scope, unsigned* ticket_launches, hipStream_t s) {
  if (!gru_persist_supported(B, H, groups) || T < 1) return hipErrorInvalidValue;
  if (((uintptr_t)hs & 15) != 0 || (s_hs & 3) != 0 || ((uintptr_t)W_hh & 15) != 0 || (s_rep & 3) != 0 || !hx ||
      ((uintptr_t)hx & 15) != 0 || (s_hx & 3) != 0)
    return hipErrorInvalidValue;
  if (xin && (!gru_persist_xproj_supported(H, width) || !W_ih || !b_ih || ((uintptr_t)xin & 15) != 0 ||
              (s_x & 3) != 0 || ((uintptr_t)W_ih & 15) != 0))
    return hipErrorInvalidValue;
  if (!xin && !gx) return hipErrorInvalidValue;
  const size_t lds = xin ? persist_xp_lds_bytes(H, width) : persist_lds_bytes(H);
  const int xnb = !xin ? 0 : width <= 128 ? 1 : 2;
  static size_t allowed[3] = {0, 0, 0};
  const void* fn = xnb == 0   ? (const void*)gru_fwd_persist_kernel<0>
                   : xnb == 1 ? (const void*)gru_fwd_persist_kernel<1>
                              : (const void*)gru_fwd_persist_kernel<2>;
  if (lds > allowed[xnb]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    allowed[xnb] = lds;
  }
  dim3 grid((H / PJ) * ((B + PR - 1) / PR) * groups);
  const Placement pl = placement(sync, groups * ((B + PR - 1) / PR), (long)grid.x, lds, device_scope, ticket_launches);
  KernelTimer kt(KID_GRU_FWD_PERSIST, 2.0 * B * 3 * H * ((double)H + (xin ? width : 0)) * T * groups, s);
#define HPSGD_FWD_PERSIST(N)                                                                                    \
  hipLaunchKernelGGL(gru_fwd_persist_kernel<N>, grid, dim3(PNT), lds, s, W_hh, b_hh, s_rep, gx, s_gx, hs, s_hs, \
                     hx, s_hx, sv, s_sv, B, H, T, groups, sync, base, spin_limit, pl.tickets, pl.ticket_base, pl.per_xcd, xin, s_x,  \
                     width, W_ih, b_ih)
  if (xnb == 0) HPSGD_FWD_PERSIST(0);
  else if (xnb == 1) HPSGD_FWD_PERSIST(1);
  else HPSGD_FWD_PERSIST(2);
#undef HPSGD_FWD_PERSIST
  return hipGetLastError();
}

hipError_t launch_gru_bwd_persist(const float* W_hh, long s_rep, float* dgh, float* dghx, long s_dghx, float* dgx,
                                  long s_dg, float* D,
                                  long s_D, bool d_zero, const float* above, long s_above, const float* sv, long s_sv,
                                  const float* hs, long s_hs, int B, int H, int T, int t_hi, int t_lo,
                                  int groups, unsigned* sync, unsigned base, unsigned spin_limit, float* dWp,
                                  float* dbp, bool device_scope, unsigned* ticket_launches, hipStream_t s) {
  if (!gru_persist_supported(B, H, groups) || t_lo < 0 || t_hi > T || t_lo >= t_hi) return hipErrorInvalidValue;
  if (dWp && (!gru_persist_dw_supported(H) || ((uintptr_t)dWp & 15) != 0 || ((uintptr_t)hs & 15) != 0 ||
              (s_hs & 3) != 0))
    return hipErrorInvalidValue;
  if (((uintptr_t)dgh & 15) != 0 || (s_dg & 3) != 0 || ((uintptr_t)W_hh & 15) != 0 || (s_rep & 3) != 0 || !dghx ||
      ((uintptr_t)dghx & 15) != 0 || (s_dghx & 3) != 0)
    return hipErrorInvalidValue;
  const size_t lds = persist_lds_bytes(H);
  static size_t allowed = 0;
  if (lds > allowed) {
    hipError_t e = hipFuncSetAttribute((const void*)gru_bwd_persist_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    allowed = lds;
  }
  dim3 grid((H / PJ) * ((B + PR - 1) / PR) * groups);
  const Placement pl = placement(sync, groups * ((B + PR - 1) / PR), (long)grid.x, lds, device_scope, ticket_launches);
  KernelTimer kt(KID_GRU_BWD_PERSIST, 2.0 * B * 3 * H * (double)H * (t_hi - t_lo) * groups * (dWp ? 2 : 1), s);
  hipLaunchKernelGGL(gru_bwd_persist_kernel, grid, dim3(PNT), lds, s, W_hh, s_rep, dgh, dghx, s_dghx, dgx, s_dg, D, s_D,
                     d_zero ? 1 : 0, above, s_above, sv, s_sv, hs, s_hs, B, H, T, t_hi, t_lo, groups, sync, base, spin_limit,
                     pl.tickets, pl.ticket_base, pl.per_xcd, dWp, dbp);
  return hipGetLastError();
}

// Makes a given-up recurrence visible in the results: NaN in the losses and in the first
// parameter of every output replica.
__global__ void poison_on_abort_kernel(const unsigned* abort_w, float* loss, int n_loss, float* rout, long s_rout,
                                       int groups) {
  if (*abort_w == 0u) return;
  const float nan = __builtin_nanf("");
  for (int i = threadIdx.x; i < groups; i += blockDim.x) {
    rout[i * s_rout] = nan;
    if (loss && i < n_loss) loss[i] = nan;
  }
}

hipError_t launch_poison_on_abort(const unsigned* abort_w, float* loss, int n_loss, float* rout, long s_rout,
                                  int groups, hipStream_t s) {
  hipLaunchKernelGGL(poison_on_abort_kernel, dim3(1), dim3(64), 0, s, abort_w, loss, n_loss, rout, s_rout, groups);
  return hipGetLastError();
}

// bf16 operands: 32 units per workgroup, the weight slice in registers (24 fragments per wave at most)
bool gru_persist_bf16_supported(int B, int H, int groups) {
  if (H % 32 != 0 || H < 32 || H > 1024 || B < 8 || B % 8 != 0 || groups < 1) return false;
  const long grid = (long)(H / QJ) * ((B + PR - 1) / PR) * groups;
  return grid <= device_cus();
}

unsigned gru_persist_bf16_count_per_step(int) { return 1u; }

size_t gru_persist_bf16_exchange_elems(int B, int width) { return (size_t)((B + 15) / 16) * 16 * (size_t)width; }

hipError_t launch_gru_fwd_persist_bf16(const void* Wb, long s_wb, const float* b_hh, long s_rep, const float* gx,
                                       long s_gx, float* hs, long s_hs, void* hb, long s_hb, void* hx, long s_hx,
                                       float* sv, long s_sv, void* hT, long ld_hT, long s_hT, int B, int H, int T,
                                       int groups, unsigned* sync, unsigned base, unsigned spin_limit, bool device_scope,
                                       unsigned* ticket_launches, hipStream_t s) {
  if (!gru_persist_bf16_supported(B, H, groups) || T < 1) return hipErrorInvalidValue;
  auto a16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  if (!hx || !a16(hx) || (s_hx & 7) != 0) return hipErrorInvalidValue;
  if (!a16(Wb) || !a16(hb) || !a16(hs) || !a16(gx) || !a16(sv) || !a16(b_hh) || (hT && !a16(hT)) || (s_wb & 7) != 0 ||
      (s_hb & 7) != 0 || (s_hs & 3) != 0 || (s_gx & 3) != 0 || (s_sv & 3) != 0 || (s_rep & 3) != 0 ||
      (hT && ((ld_hT & 7) != 0 || (s_hT & 7) != 0)))
    return hipErrorInvalidValue;
  const size_t lds = (size_t)8 * 12 * 256 * sizeof(float) + (size_t)QJ * TP * 2 + 16;
  const int ncf = H <= 256 ? 1 : H <= 512 ? 2 : 4;
  static bool ready[3] = {false, false, false};
  const int slot = ncf == 1 ? 0 : ncf == 2 ? 1 : 2;
  const void* fn = ncf == 1   ? (const void*)gru_fwd_persist_bf16_kernel<1>
                   : ncf == 2 ? (const void*)gru_fwd_persist_bf16_kernel<2>
                              : (const void*)gru_fwd_persist_bf16_kernel<4>;
  if (!ready[slot]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ready[slot] = true;
  }
  dim3 grid((H / QJ) * ((B + PR - 1) / PR) * groups);
  const Placement pl = placement(sync, groups * ((B + PR - 1) / PR), (long)grid.x, lds, device_scope, ticket_launches);
  KernelTimer kt(KID_GRU_FWD_PERSIST_BF16, 2.0 * B * 3 * H * (double)H * T * groups, s);
#define HPSGD_FWD_PB(N)                                                                                            \
  hipLaunchKernelGGL(gru_fwd_persist_bf16_kernel<N>, grid, dim3(PNT), lds, s, (const __bf16*)Wb, s_wb, b_hh, s_rep, \
                     gx, s_gx, hs, s_hs, (__bf16*)hb, s_hb, (__bf16*)hx, s_hx, sv, s_sv, (__bf16*)hT, ld_hT, s_hT, B, H, T, groups,    \
                     sync, base, spin_limit, pl.tickets, pl.ticket_base, pl.per_xcd)
  if (ncf == 1) HPSGD_FWD_PB(1);
  else if (ncf == 2) HPSGD_FWD_PB(2);
  else HPSGD_FWD_PB(4);
#undef HPSGD_FWD_PB
  return hipGetLastError();
}

hipError_t launch_gru_bwd_persist_bf16(const void* WT, long s_wt, void* dghx, long s_dgh, long s_dgb, float* D, long s_D,
                                       bool d_zero, const float* above, long s_above, const float* sv, long s_sv, const float* hs,
                                       long s_hs, void* dgxb, void* dgxT, void* dghT, long ld_T, long s_T, float* dbp,
                                       int B, int H, int T, int groups, unsigned* sync, unsigned base,
                                       unsigned spin_limit, bool device_scope, unsigned* ticket_launches, hipStream_t s) {
  if (!gru_persist_bf16_supported(B, H, groups) || T < 1 || !dbp || !dgxb || !dgxT || !dghT || !dghx)
    return hipErrorInvalidValue;
  auto a16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  if ((s_dgh & 7) != 0) return hipErrorInvalidValue;
  if (!a16(WT) || !a16(dghx) || !a16(dgxb) || !a16(dgxT) || !a16(dghT) || !a16(D) || !a16(sv) || !a16(hs) ||
      (above && !a16(above)) || (s_wt & 7) != 0 || (s_dgb & 7) != 0 || (ld_T & 7) != 0 || (s_T & 7) != 0 ||
      (s_D & 3) != 0 || (s_above & 3) != 0 || (s_sv & 3) != 0 || (s_hs & 3) != 0)
    return hipErrorInvalidValue;
  const int ncf = H <= 256 ? 1 : H <= 512 ? 2 : 4;
  const int ncl = 3 * ncf - 3 * ncf / 2;
  const size_t lds = (size_t)8 * 4 * 256 * sizeof(float) + (size_t)4 * QJ * TP * 2 + (size_t)8 * ncl * 2 * 64 * 16 + 16;
  static bool ready[3] = {false, false, false};
  const int slot = ncf == 1 ? 0 : ncf == 2 ? 1 : 2;
  const void* fn = ncf == 1   ? (const void*)gru_bwd_persist_bf16_kernel<3>
                   : ncf == 2 ? (const void*)gru_bwd_persist_bf16_kernel<6>
                              : (const void*)gru_bwd_persist_bf16_kernel<12>;
  if (!ready[slot]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ready[slot] = true;
  }
  dim3 grid((H / QJ) * ((B + PR - 1) / PR) * groups);
  const Placement pl = placement(sync, groups * ((B + PR - 1) / PR), (long)grid.x, lds, device_scope, ticket_launches);
  KernelTimer kt(KID_GRU_BWD_PERSIST_BF16, 2.0 * B * 3 * H * (double)H * T * groups, s);
#define HPSGD_BWD_PB(N)                                                                                            \
  hipLaunchKernelGGL(gru_bwd_persist_bf16_kernel<N>, grid, dim3(PNT), lds, s, (const __bf16*)WT, s_wt,              \
                     (__bf16*)dghx, s_dgh, s_dgb, D, s_D, d_zero ? 1 : 0, above, s_above, sv, s_sv, hs, s_hs, (__bf16*)dgxb, (__bf16*)dgxT, \
                     (__bf16*)dghT, ld_T, s_T, dbp, B, H, T, groups, sync, base, spin_limit,                        \
                     pl.tickets, pl.ticket_base, pl.per_xcd)
  if (ncf == 1) HPSGD_BWD_PB(3);
  else if (ncf == 2) HPSGD_BWD_PB(6);
  else HPSGD_BWD_PB(12);
#undef HPSGD_BWD_PB
  return hipGetLastError();
}

}  // namespace hpsgd
