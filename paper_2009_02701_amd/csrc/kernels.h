// Internal launch interface between the C-ABI layer and the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#define HPSGD_KMAX 32

namespace hpsgd {

struct PtrPack {  // K device pointers passed by value as a kernel argument
  float* p[HPSGD_KMAX];
};

// ---- per-kernel timing (benchmarks) ----
// The kernels whose launches can be timed one by one (enum hpsgd_kernel in hpsgd.h has the
// same numbering).  A launcher creates a KernelTimer around its launch: when the calling
// thread is inside a local step whose context has that kernel's timing enabled, a HIP event
// pair is recorded on the launch's own stream, together with the launch's algorithmic work
// (flops for the contractions, bytes for the streaming kernels); otherwise it does nothing.
enum KernelId : int {
  KID_NONE = 0,
  KID_GRU_FWD_PERSIST = 1,        // gru_fwd_persist_kernel (fp32, any input-projection form)
  KID_GRU_BWD_PERSIST = 2,        // gru_bwd_persist_kernel
  KID_GRU_FWD_PERSIST_BF16 = 3,   // gru_fwd_persist_bf16_kernel
  KID_GRU_BWD_PERSIST_BF16 = 4,   // gru_bwd_persist_bf16_kernel
  KID_GEMM_BF16_DL = 5,           // gemm_bf16_dl_kernel<false>   (128 x 128)
  KID_GEMM_BF16_DL_COMMIT = 6,    // gemm_bf16_dl_kernel<true>
  KID_GEMM_BF16_DLX128 = 7,       // gemm_bf16_dlx_kernel<false, 2, 4, 2, 2, 3>  (128 x 256)
  KID_GEMM_BF16_DLX128_COMMIT = 8,
  KID_GEMM_BF16_DLX192 = 9,       // gemm_bf16_dlx_kernel<false, 2, 4, 3, 2, 2>  (192 x 256)
  KID_GEMM_BF16_DLX192_COMMIT = 10,  // (also gemm_bf16_dlx_pair_kernel<true, 2, 4, 3, 2, 2>: two such products in one launch)
  KID_GEMM_BF16_DLX256 = 11,      // gemm_bf16_dlx_kernel<false, 2, 4, 4, 2, 2>  (256 x 256)
  KID_GEMM_BF16_DLX256_COMMIT = 12,
  KID_GEMM_BF16_NT = 13,          // gemm_bf16_nt_kernel (an fp32 operand rounded while staged)
  KID_GEMM_F32_FAST = 14,         // gemm_f32_fast_kernel (all tile forms)
  KID_GEMM_F32 = 15,              // gemm_f32_kernel / gemm_bf16_kernel (generic fallbacks)
  KID_CVT2 = 16,                  // cvt2_kernel (bf16 copy + transposed copy)
  KID_SOFTMAX_CE_BF16 = 17,       // softmax_ce_bf16_rows_kernel / softmax_ce_bf16_kernel
  KID_GRU_STEP = 18,              // gru_{fwd,bwd}_step(_bf16)_kernel: one launch per time step
  KID_COMMIT_ACC = 19,            // commit_acc4_kernel / commit_acc_kernel (update + accumulate, 20 B/param)
  KID_COMMIT = 20,                // commit_kernel (update of what no GEMM epilogue updated, 12 B/param)
  KID_CVT2_PACK = 21,             // cvt2_pack_kernel (the copies of several matrices in one launch)
  KID_COUNT = 22
};
struct KernelTimer {
  KernelTimer(int kid, double work, hipStream_t s);
  ~KernelTimer();
  KernelTimer(const KernelTimer&) = delete;
  KernelTimer& operator=(const KernelTimer&) = delete;
 private:
  void* ctx_;  // the context that holds the open stamp, or nullptr
  int idx_;    // its index there
  hipStream_t s_;
};

// ---- HBM-streaming kernels over flat parameter buffers ----
hipError_t launch_merge(float* global, const PtrPack& replicas, const float* snapshot, int K,
                        size_t P, hipStream_t s);
hipError_t launch_sync_all(const float* global, const PtrPack& replicas, int K, float* snapshot,
                           size_t P, hipStream_t s);
// merge, then sync of the same replicas and snapshot, in one pass
// (clone = false: the replicas are only read, the snapshot alone is taken)
hipError_t launch_merge_sync(float* global, const PtrPack& replicas, float* snapshot, int K, size_t P,
                             hipStream_t s, bool clone = true);
// out[k] = in[k] - lr * grad[k] for K strided slices of P floats (in_stride 0: one model for all)
hipError_t launch_commit(const float* in, size_t in_stride, float* out, size_t stride, const float* grad,
                         size_t grad_stride, float lr, int K, size_t P, hipStream_t s);
// p[g*stride + i] = 0 for i < n (p 16-byte aligned, stride a multiple of 4)
hipError_t launch_commit_acc(const float* in, size_t in_stride, float* out, size_t stride, const float* grad,
                             size_t grad_stride, float* acc, size_t acc_stride, float lr, int K, size_t P, hipStream_t s);
hipError_t launch_merge_grad(float* global, const PtrPack& accs, float lr, int K, size_t P, hipStream_t s);
hipError_t launch_fill_zero(float* p, size_t n, size_t stride, int groups, hipStream_t s, float* extra = nullptr,
                            size_t n_extra = 0);
// p[g*stride + r*ld + c] = 0 for r < rows, c < cols (4-byte words)
// Up to MAXSEG clears in one launch.  pk.n = 0, pk.blk0[0] = 0, pk.max_groups = 0 are set by the caller.
struct FillSeg {
  float* p; long ld; int rows; long cols; size_t stride; int groups;
};
struct FillPack {
  static constexpr int MAXSEG = 12;
  FillSeg seg[MAXSEG];
  unsigned blk0[MAXSEG + 1];
  int n, max_groups;
};
bool fill_pack_push(FillPack& pk, float* p, long ld, int rows, long cols, size_t stride, int groups);
hipError_t launch_fill_pack(const FillPack& pk, hipStream_t s);
hipError_t launch_fill_zero_2d(float* p, long ld, int rows, int cols, size_t stride, int groups,
                               hipStream_t s);
hipError_t launch_gather(const void* shard, const int32_t* idx, int n_idx, size_t row_bytes,
                         int n_chunks, size_t chunk_bytes, void* out, hipStream_t s);

hipError_t launch_gather_all(const void* const* shards, const int32_t* const* idx, int K, int n_idx,
                             size_t row_bytes, int n_chunks, size_t chunk_bytes, void* const* outs,
                             hipStream_t s);

// ---- grouped GEMM on the fp32 / bf16 matrix cores ----
enum Epilogue : int {
  EPI_STORE = 0,      // C = acc
  EPI_BIAS = 1,       // C = acc + bias[n]
  EPI_BIAS_RELU = 2,  // C = max(acc + bias[n], 0)
  EPI_ACCUM = 3,      // C += acc
  EPI_RELU_MASK = 4,  // C = acc * (mask[m,n] > 0)      (mask has C's layout)
  EPI_COMMIT = 5      // C = W[m,n] - alpha * acc       (W = aux, C's layout; C may be W itself):
                      // the SGD update of a weight matrix applied where its gradient is produced
};

struct GemmDesc {
  // C[g] (M x N, row-major, ldc) = op(A[g]) (M x Kd) * op(B[g]) (Kd x N)
  const float* A; long lda; long strideA; int transA;  // transA=0: A stored [M][Kd]; 1: stored [Kd][M]
  const float* B; long ldb; long strideB; int transB;  // transB=0: B stored [Kd][N]; 1: stored [N][Kd]
  float* C; long ldc; long strideC;
  const float* aux; long strideAux;                    // bias [N] or mask [M][N] (ldc)
  int M, N, Kd, groups;
  // splits > 1 (pipelined fp32 kernel only; the caller checks launch_gemm_f32_split_supported):
  // the contraction is cut into `splits` equal parts of Kd each, part p of group g reads A and B
  // advanced by p * Kd along the contraction and writes its own C at C + (g * splits + p) * strideC
  // (strideC is then the distance between two parts; the epilogue must be EPI_STORE)
  int splits;
  int epilogue;
  int bf16;                                            // round operands to bf16, use the bf16 MFMA
  float alpha;                                         // EPI_COMMIT: the learning rate
  int background;                                      // runs beside latency-critical kernels: keep the
                                                       // LDS footprint small so both fit on a CU
};
hipError_t launch_gemm(const GemmDesc& d, hipStream_t s);

// ---- classifier head with few classes in two small launches (fp32), see cls_head.hip ----
bool cls_head_supported(int N, int C, int H);
hipError_t launch_cls_head(const float* feats, long s_feats, const float* W_in, const float* b_in, long s_in,
                           const int32_t* y, long s_y, float* dlog, long s_dlog, float* rowloss, long s_rowloss,
                           float* dfeat, long s_dfeat, float* W_out, float* b_out, long s_out, float lr, int commit,
                           float* loss, int N, int C, int H, int groups, hipStream_t s, int relu_mask = 0);

// ---- GRU cell, loss, reductions ----
// forward cell for one time step of all groups:
//   gx [B][3H] (b_ih included), gh [B][3H] (b_hh included), h_prev [B][H] -> h [B][H], saved [B][4H] = r|z|n|q
hipError_t launch_gru_cell_fwd(const float* gx, long s_gx, const float* gh, long s_gh,
                               const float* h_prev, float* h, long s_h, float* saved, long s_saved,
                               int B, int H, int groups, hipStream_t s);
// backward cell: dh = D + above (above nullable); writes dgx [B][3H], dgh [B][3H], D = dh*z
hipError_t launch_gru_cell_bwd(float* D, long s_D, const float* above, long s_above,
                               const float* saved, long s_saved, const float* h_prev, long s_h,
                               float* dgx, float* dgh, long s_dg, int B, int H, int groups,
                               hipStream_t s);
// ---- fused recurrent steps (recurrent GEMM + cell math in one launch), see gru_fused.hip ----
bool gru_fused_supported(int H);
hipError_t launch_gru_fwd_step(const float* W_hh, const float* b_hh, long s_rep, const float* gx_t,
                               long s_gx, const float* h_prev, float* h_out, long s_hs, float* sv_t,
                               long s_sv, int B, int H, int groups, hipStream_t s);
hipError_t launch_gru_bwd_step(const float* WT, long s_wt, const float* dgh_next, long s_dg, float* D,
                               long s_D, const float* above, long s_above, const float* sv_t,
                               long s_sv, const float* h_prev, long s_hs, float* dgx_t, float* dgh_t,
                               int B, int H, int groups, hipStream_t s);
// ---- whole runs of time steps in one launch, W_hh resident in LDS (fp32), see gru_persist.hip ----
// sync: gru_persist_sync_words() words of device memory (the abort word, the flag words of the
// synchronisation groups, 8 ticket counters); base: what the flags read when the launch starts; every launch
// advances them by steps * gru_persist_count_per_step().  spin_limit bounds every wait.
bool gru_persist_supported(int B, int H, int groups);
size_t gru_persist_sync_words(int B, int groups);
unsigned gru_persist_count_per_step(int H);
// device_scope: the workgroups exchange through memory that every XCD sees; false lets a launch
// that fills the chip with one workgroup per CU exchange through the L2 of the XCD a
// synchronisation group runs on (the workgroups then take their tiles by where they run: they draw
// tickets from 8 counters at the end of the sync words, zero at the start of a step).
// ticket_launches: the step's count of launches that have drawn tickets (advanced by the launcher;
// all launches of a step that share the sync words must share it).
// hx / dghx: h_0 .. h_T and the gate gradients of all steps as the workgroups exchange them,
// fragment-major, gru_persist_exchange_words(B, H) resp. (B, 3H) floats per time step (hx: T + 1
// steps, the first one, h_0, given); hs / dgh are the row-major copies for the other kernels
// (dgh may be nullptr in the backward launch when nothing reads it later).
size_t gru_persist_exchange_words(int B, int width);
hipError_t launch_gru_fwd_persist(const float* W_hh, const float* b_hh, long s_rep, const float* gx, long s_gx,
                                  float* hs, long s_hs, float* hx, long s_hx, float* sv, long s_sv, int B, int H, int T,
                                  int groups,
                                  unsigned* sync, unsigned base, unsigned spin_limit, const float* xin, long s_x,
                                  int width, const float* W_ih, const float* b_ih, bool device_scope, unsigned* ticket_launches, hipStream_t s);
// xin != nullptr (allowed when gru_persist_xproj_supported(H, width)): the launch computes the input
// projection itself from the layer input xin (T blocks of B x width per worker, stride s_x) and W_ih,
// b_ih (in the replica, like W_hh); gx is then unused and may be nullptr.
bool gru_persist_xproj_supported(int H, int width);
// steps t_hi-1 .. t_lo of BPTT (a range: a caller may cut BPTT into several launches);
// d_zero: the gradient carried into step t_hi-1 is zero (D is written at the end, not read)
hipError_t launch_gru_bwd_persist(const float* W_hh, long s_rep, float* dgh, float* dghx, long s_dghx, float* dgx,
                                  long s_dg, float* D,
                                  long s_D, bool d_zero, const float* above, long s_above, const float* sv, long s_sv,
                                  const float* hs, long s_hs, int B, int H, int T, int t_hi, int t_lo,
                                  int groups, unsigned* sync, unsigned base, unsigned spin_limit, float* dWp,
                                  float* dbp, bool device_scope, unsigned* ticket_launches, hipStream_t s);
// dbp != nullptr: the launch also leaves dbp[(g * RT + ty)][6H], partial sums over its steps of the
// bias gradients (b_ih: sum of dgx, then b_hh: sum of dgh)
// dWp != nullptr (allowed when gru_persist_dw_supported(H)): the launch also leaves
// dWp[(g * RT + ty)][3H][H], RT = ceil(B / 32) partial sums of dW_hh over its steps per worker.
bool gru_persist_dw_supported(int H);
// out[g][i] = in[g][i] - lr * sum_p parts[(g * n_parts + p)][i]  (commit != 0; in may be out)
// out[g][i] = sum_p parts[(g * n_parts + p)][i]                   (commit == 0)
// Up to MAXSEG sums of partial results in one launch: reduce_pack_push (false: the segment does
// not meet the alignment rules of launch_reduce_parts or the pack is full; nothing is added),
// then launch_reduce_pack.  pk.n = 0, pk.blk0[0] = 0 and pk.lr are set by the caller.
struct ReduceSeg {
  const float* parts; int n_parts; size_t n4;
  const float* in; size_t s_in; float* out; size_t s_out; int commit;
};
struct ReducePack {
  static constexpr int MAXSEG = 4;
  ReduceSeg seg[MAXSEG];
  unsigned blk0[MAXSEG + 1];
  int n;
  float lr;
};
bool reduce_pack_push(ReducePack& pk, const float* parts, int n_parts, size_t n, const float* in, size_t s_in,
                      float* out, size_t s_out, int commit);
hipError_t launch_reduce_pack(const ReducePack& pk, int groups, hipStream_t s);
hipError_t launch_reduce_parts(const float* parts, int n_parts, size_t n, const float* in, size_t s_in,
                               float* out, size_t s_out, float lr, int commit, int groups, hipStream_t s);
// bf16 operands (strides of bf16 buffers in bf16 elements): hx / dghx hold all time steps and are the
// operands the workgroups exchange, kept fragment-major (per step a block of 16 ceil(B/16) rows;
// gru_persist_bf16_exchange_elems gives a step's block); hb is the row-major copy of h for the
// GEMMs; hT, dgxT, dghT are the transposed copies [unit][time * B + row].
// The backward launch always leaves the partial bias-gradient sums in dbp and writes no fp32
// gate gradients.  Counters advance by steps * gru_persist_bf16_count_per_step().
bool gru_persist_bf16_supported(int B, int H, int groups);
unsigned gru_persist_bf16_count_per_step(int H);
hipError_t launch_gru_fwd_persist_bf16(const void* Wb, long s_wb, const float* b_hh, long s_rep, const float* gx,
                                       long s_gx, float* hs, long s_hs, void* hb, long s_hb, void* hx, long s_hx,
                                       float* sv, long s_sv, void* hT, long ld_hT, long s_hT, int B, int H, int T,
                                       int groups, unsigned* sync, unsigned base, unsigned spin_limit, bool device_scope,
                                       unsigned* ticket_launches, hipStream_t s);
// bf16 elements of one time step's block of an exchange buffer whose rows are `width` wide
size_t gru_persist_bf16_exchange_elems(int B, int width);
hipError_t launch_gru_bwd_persist_bf16(const void* WT, long s_wt, void* dghx, long s_dgh, long s_dgb, float* D, long s_D,
                                       bool d_zero, const float* above, long s_above, const float* sv, long s_sv, const float* hs,
                                       long s_hs, void* dgxb, void* dgxT, void* dghT, long ld_T, long s_T, float* dbp,
                                       int B, int H, int T, int groups, unsigned* sync, unsigned base,
                                       unsigned spin_limit, bool device_scope, unsigned* ticket_launches, hipStream_t s);
// NaN into loss[0..n_loss) and into rout[g * s_rout] for every group if *abort_w != 0
hipError_t launch_poison_on_abort(const unsigned* abort_w, float* loss, int n_loss, float* rout, long s_rout,
                                  int groups, hipStream_t s);
// bf16-operand variants (strides of bf16 buffers are in bf16 elements)
bool gru_fused_bf16_supported(int H);
hipError_t launch_gru_fwd_step_bf16(const void* Wb, long s_wb, const float* b_hh, long s_rep,
                                    const float* gx_t, long s_gx, const float* h_prev, float* h_out,
                                    long s_hs, const void* hb_prev, void* hb_out, long s_hb, float* sv_t,
                                    long s_sv, void* hT_out, long ld_hT, long s_hT, int B, int H,
                                    int groups, hipStream_t s);
hipError_t launch_gru_bwd_step_bf16(const void* WTb, long s_wt, const void* dghb_next, void* dghb_t,
                                    long s_dgb, float* D, long s_D, const float* above, long s_above,
                                    const float* sv_t, long s_sv, const float* h_prev, long s_hs,
                                    float* dgx_t, float* dgh_t, long s_dg, void* dgxb_t, void* dgxT_t,
                                    void* dghT_t, long ld_T, long s_T, int B, int H, int groups,
                                    hipStream_t s);
// out(bf16) = round(in), in is R x C with row pitch ld_in; transpose: out[c][r] = in[r][c];
// ld_out is the row pitch of out, strides of out in bf16 elements
hipError_t launch_cvt_bf16(const float* in, long ld_in, long s_in, void* out, long ld_out, long s_out,
                           int R, int C, bool transpose, int groups, hipStream_t s);
// in (fp32, or bf16 when in_bf16) R x C -> out_p = bf16 rounding (nullable), out_t = its
// transpose (nullable), one read of `in`; strides of each buffer in its own elements
bool cvt2_supported(const void* in, int in_bf16, long ld_in, long s_in, const void* out_p, long ld_p,
                    long s_p, const void* out_t, long ld_t, long s_t, int R, int C);
hipError_t launch_cvt2(const void* in, int in_bf16, long ld_in, long s_in, void* out_p, long ld_p, long s_p,
                       void* out_t, long ld_t, long s_t, int R, int C, int groups, hipStream_t s);
// several fp32 matrices through one launch of the same copies (one group count for all of them)
struct Cvt2Job {
  const float* in;
  long ld_in, s_in;
  void* out_p;
  long ld_p, s_p;
  void* out_t;
  long ld_t, s_t;
  int R, C, tiles_x, pad;
};
struct Cvt2Pack {
  static constexpr int MAX = 8;
  int n = 0;
  int tile0[MAX + 1] = {0};  // first tile of job j in blockIdx.x; tile0[n] = all tiles
  double bytes = 0;          // per group, for the launch timer
  Cvt2Job job[MAX];
};
// false: the pack is full or the job is not one cvt2_supported takes (launch it by itself)
bool cvt2_pack_push(Cvt2Pack& p, const float* in, long ld_in, long s_in, void* out_p, long ld_p, long s_p,
                    void* out_t, long ld_t, long s_t, int R, int C);
hipError_t launch_cvt2_pack(const Cvt2Pack& p, int groups, hipStream_t s);
// mean softmax-CE whose logit gradient is written rounded to bf16 (row pitch ld_d); logits intact
bool softmax_ce_bf16_supported(const float* logits, long s_logits, const void* dlog, long ld_d, long s_d,
                               int C);
// rowstat: per row (max logit, 1 / sum of exponentials), two floats (group stride s_rowstat floats, even)
hipError_t launch_softmax_ce_bf16(const float* logits, long s_logits, const int32_t* y, long s_y, void* dlog,
                                  long ld_d, long s_d, float* rowloss, long s_rowloss, float* rowstat,
                                  long s_rowstat, int N, int C, int groups, hipStream_t s, float* colpart = nullptr,
                                  long s_colpart = 0, int sizing_groups = 0);
// colpart holds one partial sum per block of rows: softmax_ce_bf16_row_blocks(N, sizing_groups)
// blocks per group, where sizing_groups is the number of workers the launch is sized for (the
// same value must go to the launch); 0 gives the upper bound, for allocations
int softmax_ce_bf16_row_blocks(int N, int sizing_groups = 0, int C = 0);
// out[c] = mean over rows of (softmax - onehot), from the logits and the rows' rowstat pairs
hipError_t launch_colsum_softmax(const float* logits, long s_logits, const float* rowstat, long s_rowstat,
                                 const int32_t* y, long s_y, float* out, long s_out, int N, int C, int groups,
                                 hipStream_t s);
// one wave that sleeps until the wall clock has advanced by `us` microseconds
hipError_t launch_delay(unsigned us, hipStream_t s);
// pure-MFMA loop, one wave on every SIMD, operands from `operands` (16 KiB); see hpsgd.h
hipError_t launch_mfma_probe(bool bf16, const void* operands, int iterations, double* result, float* sink,
                             hipStream_t s);
// out[r] = sum_c in[r][c], in bf16 (R x C, row pitch ld), fp32 accumulation
hipError_t launch_rowsum_bf16(const void* in, long ld, long s_in, float* out, long s_out, int R, int C,
                              int groups, hipStream_t s);
// bf16 GEMM with both operands unit-stride along the contraction (gemm_bf16_nt.hip)
bool gemm_bf16_nt_supported(const void* p, int is_bf16, long ld, long stride, int Kd);
hipError_t launch_gemm_bf16_nt(const void* A, int a_bf16, long lda, long sA, const void* B, int b_bf16,
                               long ldb, long sB, float* C, long ldc, long sC, const float* bias,
                               long sBias, const float* win, long sWin, float lr, int M, int N, int Kd,
                               int groups, hipStream_t s, int form = 0);
// Two products with bf16 operands and the update epilogue (C = win - lr * A B^T) in ONE launch of
// the 192 x 256 form: for two that neither need each other nor fill the chip alone.  Strides in
// elements of each buffer's own type; the same conditions as launch_gemm_bf16_nt per product.
struct GemmBf16Args {
  const void* A; long lda, sA;
  const void* B; long ldb, sB;
  float* C; long ldc, sC;
  const float* win; long sWin;
  float lr;
  int M, N, Kd, groups;
};
bool gemm_bf16_update_pair_supported(const GemmBf16Args& p0, const GemmBf16Args& p1);
hipError_t launch_gemm_bf16_update_pair(const GemmBf16Args& p0, const GemmBf16Args& p1, hipStream_t s);

// out[c][r] = in[r][c], R x C per group
hipError_t launch_transpose(const float* in, long s_in, float* out, long s_out, int R, int C,
                            int groups, hipStream_t s);

// mean softmax cross-entropy over N rows of C logits; dlogits = (p - onehot)/N; row losses to rowloss
hipError_t launch_softmax_ce(const float* logits, long s_logits, const int32_t* y, long s_y,
                             float* dlogits, float* rowloss, long s_rowloss, int N, int C,
                             int groups, hipStream_t s);
// loss[g] = (1/N) sum_i rowloss[g][i], fixed order
hipError_t launch_loss_mean(const float* rowloss, long s_rowloss, float* loss, int N, int groups,
                            hipStream_t s);
// out[g][n] = sum_r in[g][r][n]
// Column sums of up to MAXSEG matrices in one launch, optionally applied as out = b_in - lr * sum.
// pk.n = 0, pk.blk0[0] = 0 and pk.lr are set by the caller.
struct ColsumSeg {
  const float* in; long ld, s_in;
  float* out; long s_out;
  const float* b_in; long s_bin;
  int R, N;
  float scale;  // applied when b_in is null
};
struct ColsumPack {
  static constexpr int MAXSEG = 8;
  ColsumSeg seg[MAXSEG];
  unsigned blk0[MAXSEG + 1];
  int n;
  float lr;
};
bool colsum_pack_push(ColsumPack& pk, const float* in, long ld, long s_in, float* out, long s_out, const float* b_in,
                      long s_bin, int R, int N, float scale = 1.0f);
hipError_t launch_colsum_pack(const ColsumPack& pk, int groups, hipStream_t s);
hipError_t launch_colsum(const float* in, long ld, long s_in, float* out, long s_out, int R, int N,
                         int groups, hipStream_t s);
// embedding rows: out[g][i][:] = E[g][tok[g][i]][:]
hipError_t launch_embed_fwd(const float* E, long s_E, const int32_t* tok, long s_tok, float* out,
                            long s_out, int N, int Ew, int groups, hipStream_t s);
// dE[g][v][:] = sum over positions i with tok[g][i]==v of dx[g][i][:], in increasing i; other rows untouched
hipError_t launch_embed_bwd(const float* dx, long s_dx, const int32_t* tok, long s_tok, float* dE,
                            long s_dE, int N, int Ew, int groups, hipStream_t s, const float* E_in = nullptr,
                            long s_E = 0, float lr = 0.f);

}  // namespace hpsgd
