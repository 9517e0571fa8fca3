// C-ABI layer: argument validation, the flat parameter layout, the workspace layout and
// the launch plan of one local training step.  Host code only; every arithmetic step runs
// in the kernels declared in kernels.h.
#include "../../include/hpsgd.h"

#include <string>
#include <mutex>
#include <cstring>
#include <vector>

#include "kernels.h"

using namespace hpsgd;

namespace {

struct Entry {
  std::string name;
  size_t offset;
  int rows, cols;
};

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int kWihSplits = 4;  // parts of the contraction of a narrow layer's dW_ih GEMM (fp32)

struct Region {  // one workspace buffer: K slices of `stride` floats
  size_t offset = 0, stride = 0;
};

}  // namespace

struct hpsgd_ctx {
  hpsgd_model_desc d;
  int K;
  std::vector<Entry> entries;
  size_t P = 0;
  size_t ws_floats = 0;
  // workspace regions (floats)
  Region grad, xe, gx, dgh, gh, D, dx, logits, rowloss, wt;
  Region psync;                 // abort word and flag words of the resident-weight recurrence kernels
  Region dwp, dbp;              // their partial sums of dW_hh and of the bias gradients, one per 32-row batch tile
  Region dwip;                  // partial sums of dW_ih of a narrow layer input (contraction cut into kWihSplits)
  Region hb, dghb, dgxb;        // bf16 copies of h, dgh and dgx (bf16 precision only)
  Region hx, dghx;              // h and dgh as the resident-weight launches exchange them (fragment-major)
  // transposed bf16 copies that bring the weight-gradient and input-gradient GEMMs into the
  // contraction-contiguous form (bf16 precision only); sizes in floats = bf16 count / 2
  Region dgxT, dghT, xT, dlogT, wihT, woT;
  Region xb, wihb, wob, dlogb;  // row-major bf16 copies: layer-0 input, W_ih, head.W, dlogits
  Region rowstat;               // per logits row: (max, 1 / sum of exponentials)
  Region colpart;               // per block of logits rows: column sums of the logit gradient
  std::vector<Region> hsT;
  std::vector<Region> whhT, wihTl;  // per layer: transposed bf16 W_hh and W_ih, made in the forward pass
  std::vector<Region> whhb, wihbl;  // per layer: row-major bf16 W_hh and W_ih
  // Marks left by hpsgd_prepare_replicas / hpsgd_prepare_clones, one per workspace (a schedule with
  // two generations of buffers prepares one while the other steps): the bf16 copies of these
  // replicas' weights are in that workspace.  clone_src (prepare_clones): ONE set of copies, made
  // from this model, serves every worker; head_done: the head's copies are among them (else the
  // step makes them from clone_src right before the logits GEMM).
  struct Mark { const float* rin; const float* ws; size_t stride; const float* clone_src; bool head_done; };
  std::vector<Mark> marks;
  void set_mark(const Mark& m) {
    drop_mark(m.ws);
    if (marks.size() >= 4) marks.erase(marks.begin());
    marks.push_back(m);
  }
  void drop_mark(const float* ws) {
    for (size_t i = 0; i < marks.size();)
      if (marks[i].ws == ws) marks.erase(marks.begin() + i);
      else ++i;
  }
  // the mark of this workspace if it was made for exactly these replicas; the workspace's mark is
  // gone afterwards either way (the step rewrites the copies, and changes the weights)
  bool take_mark(const float* rin, const float* ws, size_t stride, Mark& out) {
    bool found = false;
    for (const Mark& m : marks)
      if (m.ws == ws && m.rin == rin && m.stride == stride) { out = m; found = true; }
    drop_mark(ws);
    return found;
  }
  std::vector<Region> hs, sv;   // per GRU layer
  std::vector<Region> act;      // per MLP layer output
  std::vector<Region> dact;     // per MLP hidden layer: gradient w.r.t. its output
  // optional per-role kernel timing (benchmarks): event pairs recorded around launches
  // optional second stream for work that can run beside the recurrence, and the two events
  // that order it against the caller's stream
  hipStream_t aux = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool resident = true;         // fp32 recurrence: one launch per run of time steps when supported
  bool device_scope = false;    // resident-weight launches exchange at device scope even where an XCD's L2 would do
  unsigned spin_limit = 1u << 20;  // bound of every wait inside those launches
  size_t last_commit_params = 0;  // parameters per worker that the commit kernel handled last step
  int last_resident = 0, last_xproj = 0, last_dw = 0;  // GRU layers of the last step, see hpsgd_recurrence_info
  unsigned timer_mask = 0;
  bool timer_nested = false;    // an enclosing scope already brackets the current launches
  struct Stamp { int role; int launches; hipEvent_t a, b; };
  std::vector<Stamp> stamps;
  std::vector<hipEvent_t> free_events;
  double role_ms[HPSGD_ROLE_COUNT] = {0};
  long role_launches[HPSGD_ROLE_COUNT] = {0};
  // per-kernel timing: event pairs recorded by the launchers themselves (KernelTimer)
  unsigned kernel_mask = 0;
  struct KStamp { int kid; double work; hipEvent_t a, b; };
  std::vector<KStamp> kstamps;
  double kernel_ms[HPSGD_KERNEL_COUNT] = {0}, kernel_work[HPSGD_KERNEL_COUNT] = {0};
  long kernel_launches[HPSGD_KERNEL_COUNT] = {0};

  // entries of the flat layout by role, filled once by build_layout: the launch plan of a step looks
  // nothing up by name
  struct LayerIdx { int wih, whh, bih, bhh; };
  std::vector<LayerIdx> lidx;       // per GRU layer
  std::vector<int> fc_w, fc_b;      // per MLP layer
  int i_embed = -1, i_head_w = -1, i_head_b = -1;
  size_t eoff(int entry) const { return entries[entry].offset; }


  Region alloc(size_t per_worker) {
    Region r;
    r.stride = round_up(per_worker, 64);
    r.offset = ws_floats;
    ws_floats += r.stride * (size_t)K;
    return r;
  }
};

namespace {

void add_entry(hpsgd_ctx* c, const std::string& name, int rows, int cols) {
  c->entries.push_back({name, c->P, rows, cols});
  c->P += (size_t)rows * (size_t)cols;
}

int build_layout(hpsgd_ctx* c) {
  const hpsgd_model_desc& d = c->d;
  const long big = 1L << 30;
  if (d.kind == HPSGD_GRU_CLASSIFIER || d.kind == HPSGD_GRU_LM) {
    const bool lm = d.kind == HPSGD_GRU_LM;
    if (d.layers < 1 || d.layers > 16 || d.hidden < 1 || d.seq_len < 1 || d.batch < 1) return HPSGD_ESHAPE;
    if (lm ? (d.vocab < 2 || d.embed < 1) : (d.input < 1 || d.classes < 2)) return HPSGD_ESHAPE;
    if ((long)d.seq_len * d.batch * 4L * d.hidden >= big) return HPSGD_ESHAPE;
    if (d.seq_len > 65535) return HPSGD_ESHAPE;
    int width = lm ? d.embed : d.input;
    const int classes = lm ? d.vocab : d.classes;
    if ((long)d.seq_len * d.batch * (long)classes >= big) return HPSGD_ESHAPE;
    if (lm) {
      c->i_embed = (int)c->entries.size();
      add_entry(c, "embed.E", d.vocab, d.embed);
    }
    for (int l = 0; l < d.layers; ++l) {
      const std::string p = "l" + std::to_string(l);
      const int e0 = (int)c->entries.size();
      c->lidx.push_back({e0, e0 + 1, e0 + 2, e0 + 3});
      add_entry(c, p + ".W_ih", 3 * d.hidden, width);
      add_entry(c, p + ".W_hh", 3 * d.hidden, d.hidden);
      add_entry(c, p + ".b_ih", 3 * d.hidden, 1);
      add_entry(c, p + ".b_hh", 3 * d.hidden, 1);
      width = d.hidden;
    }
    c->i_head_w = (int)c->entries.size();
    add_entry(c, "head.W", classes, d.hidden);
    c->i_head_b = (int)c->entries.size();
    add_entry(c, "head.b", classes, 1);

    const size_t TB = (size_t)d.seq_len * d.batch, H = d.hidden;
    c->grad = c->alloc(c->P);
    if (lm) c->xe = c->alloc(TB * d.embed);
    for (int l = 0; l < d.layers; ++l) {
      c->hs.push_back(c->alloc((TB + d.batch) * H));
      c->sv.push_back(c->alloc(TB * 4 * H));
    }
    c->gx = c->alloc(TB * 3 * H);
    c->dgh = c->alloc(TB * 3 * H);
    c->gh = c->alloc((size_t)d.batch * 3 * H);
    c->D = c->alloc((size_t)d.batch * H);
    c->wt = c->alloc(3 * H * H);
    c->psync = c->alloc(gru_persist_sync_words(d.batch, 1));
    if (gru_fused_supported(d.hidden)) c->dbp = c->alloc((size_t)((d.batch + 31) / 32) * 6 * H);
    if (d.prec != HPSGD_BF16_MFMA && gru_fused_supported(d.hidden) && gru_persist_dw_supported(d.hidden))
      c->dwp = c->alloc((size_t)((d.batch + 31) / 32) * 3 * H * H);
    if (d.prec != HPSGD_BF16_MFMA) c->dwip = c->alloc((size_t)kWihSplits * 3 * H * (lm ? d.embed : d.input));
    if (d.prec != HPSGD_BF16_MFMA && gru_fused_supported(d.hidden)) {
      c->hx = c->alloc((size_t)(d.seq_len + 1) * gru_persist_exchange_words(d.batch, d.hidden));
      c->dghx = c->alloc((size_t)d.seq_len * gru_persist_exchange_words(d.batch, 3 * d.hidden));
    }
    if (d.prec == HPSGD_BF16_MFMA) {
      c->hb = c->alloc(((TB + d.batch) * H + 1) / 2);
      c->dghb = c->alloc((TB * 3 * H + 1) / 2);
      c->hx = c->alloc(((size_t)(d.seq_len + 1) * gru_persist_bf16_exchange_elems(d.batch, d.hidden) + 1) / 2);
      c->dghx = c->alloc(((size_t)d.seq_len * gru_persist_bf16_exchange_elems(d.batch, 3 * d.hidden) + 1) / 2);
      c->dgxb = c->alloc((TB * 3 * H + 1) / 2);
      const size_t TBp = round_up(TB, 64), TB1p = round_up(TB + d.batch, 64);
      const size_t win0 = lm ? d.embed : d.input;
      const size_t wmax = win0 > H ? win0 : H;
      c->dgxT = c->alloc(3 * H * TBp / 2);
      c->dghT = c->alloc(3 * H * TBp / 2);
      c->xT = c->alloc(win0 * TBp / 2);
      for (int l = 0; l < d.layers; ++l) {
        c->hsT.push_back(c->alloc(H * TB1p / 2));
        c->whhT.push_back(c->alloc((3 * H * H + 1) / 2));
        c->wihTl.push_back(c->alloc(((l == 0 ? win0 : H) * 3 * H + 1) / 2));
        c->whhb.push_back(c->alloc((3 * H * H + 1) / 2));
        c->wihbl.push_back(c->alloc(((l == 0 ? win0 : H) * 3 * H + 1) / 2));
      }
      const size_t nr = lm ? TB : (size_t)d.batch;
      c->dlogT = c->alloc((size_t)classes * round_up(nr, 64) / 2);
      c->wihT = c->alloc(wmax * 3 * H / 2);
      c->woT = c->alloc(H * round_up(classes, 64) / 2);
      c->xb = c->alloc((TB * win0 + 1) / 2);
      c->wihb = c->alloc((wmax * 3 * H + 1) / 2);
      c->wob = c->alloc(((size_t)classes * H + 1) / 2);
      c->dlogb = c->alloc((nr * round_up(classes, 64) + 1) / 2);
      c->rowstat = c->alloc(2 * nr);
      c->colpart = c->alloc(round_up((size_t)softmax_ce_bf16_row_blocks((int)nr) * classes, 4));
    }
    size_t wmax = H;
    if (lm && (size_t)d.embed > wmax) wmax = d.embed;
    c->dx = c->alloc(TB * wmax);
    const size_t nrows = lm ? TB : (size_t)d.batch;
    c->logits = c->alloc(nrows * classes);
    c->rowloss = c->alloc(nrows);
  } else if (d.kind == HPSGD_MLP) {
    if (d.n_mlp_dims < 2 || d.n_mlp_dims > HPSGD_MAX_MLP_DIMS || d.batch < 1) return HPSGD_ESHAPE;
    for (int i = 0; i < d.n_mlp_dims; ++i)
      if (d.mlp_dims[i] < 1 || (long)d.mlp_dims[i] * d.batch >= big) return HPSGD_ESHAPE;
    if (d.mlp_dims[d.n_mlp_dims - 1] < 2) return HPSGD_ESHAPE;
    for (int i = 0; i + 1 < d.n_mlp_dims; ++i) {
      const std::string p = "fc" + std::to_string(i);
      c->fc_w.push_back((int)c->entries.size());
      add_entry(c, p + ".W", d.mlp_dims[i + 1], d.mlp_dims[i]);
      c->fc_b.push_back((int)c->entries.size());
      add_entry(c, p + ".b", d.mlp_dims[i + 1], 1);
    }
    c->grad = c->alloc(c->P);
    for (int i = 1; i < d.n_mlp_dims; ++i) c->act.push_back(c->alloc((size_t)d.batch * d.mlp_dims[i]));
    for (int i = 1; i + 1 < d.n_mlp_dims; ++i) c->dact.push_back(c->alloc((size_t)d.batch * d.mlp_dims[i]));
    c->rowloss = c->alloc(d.batch);
  } else {
    return HPSGD_EINVAL;
  }
  return HPSGD_OK;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + nb && b0 < a0 + na;
}

// Records an event pair around the launches issued while it is alive, if its role is timed.
struct TimerScope {
  hpsgd_ctx* c;
  hipStream_t s;
  int idx = -1;
  static hipEvent_t get(hpsgd_ctx* c) {
    hipEvent_t e = nullptr;
    if (!c->free_events.empty()) {
      e = c->free_events.back();
      c->free_events.pop_back();
    } else if (hipEventCreate(&e) != hipSuccess) {
      e = nullptr;
    }
    return e;
  }
  // launches: how many kernel launches the pair brackets (a whole time loop is bracketed by
  // one pair: an event record between two dependent launches costs far more than the launch)
  TimerScope(hpsgd_ctx* c_, int role, hipStream_t s_, int launches = 1) : c(c_), s(s_) {
    if (launches <= 0 || !(c->timer_mask & (1u << role)) || c->timer_nested) return;
    hipEvent_t a = get(c), b = get(c);
    if (!a || !b) return;
    c->stamps.push_back({role, launches, a, b});
    idx = (int)c->stamps.size() - 1;
    (void)hipEventRecord(a, s);
  }
  ~TimerScope() {
    if (idx >= 0) (void)hipEventRecord(c->stamps[idx].b, s);
  }
  bool active() const { return idx >= 0; }
};

// The context whose local step the calling thread is issuing (KernelTimer looks here).
thread_local hpsgd_ctx* t_step_ctx = nullptr;
struct StepCtxScope {
  hpsgd_ctx* prev;
  explicit StepCtxScope(hpsgd_ctx* c) : prev(t_step_ctx) { t_step_ctx = c; }
  ~StepCtxScope() { t_step_ctx = prev; }
};

// inside run_step: `role` names what the next launches are for
#define HIP_TRY(expr)                              \
  do {                                             \
    TimerScope ts_(c, role, s);                    \
    if ((expr) != hipSuccess) return HPSGD_EHIP;   \
  } while (0)

// GEMM helper: C = op(A) op(B) for `groups` workers.
int gemm(hipStream_t s, int groups, int bf16, int M, int N, int Kd, const float* A, long lda,
         long sA, int tA, const float* B, long ldb, long sB, int tB, float* C, long ldc, long sC,
         int epi, const float* aux, long sAux, int background = 0, float alpha = 0.f, int splits = 1) {
  GemmDesc g;
  g.splits = splits;
  g.background = background;
  g.alpha = alpha;
  g.A = A; g.lda = lda; g.strideA = sA; g.transA = tA;
  g.B = B; g.ldb = ldb; g.strideB = sB; g.transB = tB;
  g.C = C; g.ldc = ldc; g.strideC = sC;
  g.aux = aux; g.strideAux = sAux;
  g.M = M; g.N = N; g.Kd = Kd; g.groups = groups;
  g.epilogue = epi; g.bf16 = bf16;
  return launch_gemm(g, s) == hipSuccess ? HPSGD_OK : HPSGD_EHIP;
}

// A k-contiguous view of a GEMM operand for the NT kernel (p == nullptr: none available).
struct NtView {
  const void* p = nullptr;
  int bf16 = 0;
  long ld = 0, stride = 0;
};

// bf16 precision: use the NT kernel when both operands have a usable contraction-contiguous
// view (C = a b^T), otherwise the generic kernel on the original fp32 operands.
int gemm2(hipStream_t s, int groups, int bf16, int M, int N, int Kd, const float* A, long lda, long sA,
          int tA, const float* B, long ldb, long sB, int tB, float* C, long ldc, long sC, int epi,
          const float* aux, long sAux, const NtView& a, const NtView& b, float alpha = 0.f,
          bool require_nt = false) {
  if (bf16 && a.p && b.p && (epi == EPI_STORE || epi == EPI_BIAS || epi == EPI_COMMIT) &&
      gemm_bf16_nt_supported(a.p, a.bf16, a.ld, a.stride, Kd) &&
      gemm_bf16_nt_supported(b.p, b.bf16, b.ld, b.stride, Kd) && ((uintptr_t)C & 3) == 0) {
    return launch_gemm_bf16_nt(a.p, a.bf16, a.ld, a.stride, b.p, b.bf16, b.ld, b.stride, C, ldc, sC,
                               epi == EPI_BIAS ? aux : nullptr, sAux, epi == EPI_COMMIT ? aux : nullptr, sAux,
                               alpha, M, N, Kd, groups, s) == hipSuccess
               ? HPSGD_OK
               : HPSGD_EHIP;
  }
  if (require_nt) return HPSGD_EINVAL;  // the fp32 operands of the fallback were not produced
  return gemm(s, groups, bf16, M, N, Kd, A, lda, sA, tA, B, ldb, sB, tB, C, ldc, sC, epi, aux, sAux, 0, alpha);
}

#define TRY(expr)                    \
  do {                               \
    TimerScope ts_(c, role, s);      \
    int rc_ = (expr);                \
    if (rc_ != HPSGD_OK) return rc_; \
  } while (0)
#define TRY0(expr)                   \
  do {                               \
    int rc_ = (expr);                \
    if (rc_ != HPSGD_OK) return rc_; \
  } while (0)

// The resident-weight recurrence kernels wait for each other inside a launch, which needs all
// their workgroups on the chip at once: two such launches running side by side (from two
// streams) could each hold CUs the other is waiting for.  Launches on one stream are ordered
// anyway.  Across streams, contexts and host threads they are ordered here: the one piece of
// per-process state of the library, per device, is the event recorded behind the most recent
// resident-weight launch and the stream it went to.  A local step that issues such launches
// holds the lock from its first one to its last (so that no other thread's launches fall in
// between) and, if the previous ones went to another stream, lets its stream wait for that
// event (hipStreamWaitEvent: the host never blocks).
// how far behind the training stream's product the auxiliary stream's starts where the former must
// be dispatched first (see the layers' backward pass)
constexpr unsigned kAuxHeadStartUs = 5;

struct ResidentOrder {
  std::mutex mu;
  hipEvent_t ev = nullptr;   // behind the last resident-weight launch issued on this device
  hipStream_t last = nullptr;
  bool have = false;
};
constexpr int kMaxDevices = 64;
ResidentOrder g_resident[kMaxDevices];

struct ResidentScope {
  ResidentOrder* o = nullptr;
  std::unique_lock<std::mutex> lock;
  hipStream_t s = nullptr;
  // Called before the step's first resident-weight launch.
  int begin(hipStream_t stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HPSGD_EHIP;
    o = &g_resident[dev];
    s = stream;
    lock = std::unique_lock<std::mutex>(o->mu);
    if (!o->ev && hipEventCreateWithFlags(&o->ev, hipEventDisableTiming) != hipSuccess) {
      o->ev = nullptr;
      return HPSGD_EHIP;
    }
    if (o->have && o->last != s && hipStreamWaitEvent(s, o->ev, 0) != hipSuccess) return HPSGD_EHIP;
    return HPSGD_OK;
  }
  // note(): a resident-weight launch was issued; mark(): ... and the event is recorded behind
  // it (the last record stands).  The step marks behind its backward launches; a launch that was
  // only noted is marked when the step has been issued, where the lock is released too.
  bool pending = false;
  void note() { pending = o != nullptr; }
  int mark() {
    if (!o) return HPSGD_OK;
    pending = false;
    if (hipEventRecord(o->ev, s) != hipSuccess) return HPSGD_EHIP;
    o->have = true;
    o->last = s;
    return HPSGD_OK;
  }
  ~ResidentScope() {
    if (pending) (void)mark();
  }
};

// bf16 precision: the rounded copies of the weight matrices that a local step's GEMMs and
// recurrence launches read (row-major, and transposed where an input gradient is needed), all
// made from the replicas `rin`.  what[l] / head say which copies exist; launch = false only
// reports.  The head's copies are made when with_head is set.
struct WeightCopies {
  bool wih[16] = {false}, wihT[16] = {false}, whh[16] = {false}, whhT[16] = {false};
  bool head = false;
};

int weight_copies(hpsgd_ctx* c, const float* rin, long sR, int k0, int groups, float* ws, hipStream_t st, bool launch,
                  bool with_head, WeightCopies& wc) {
  const hpsgd_model_desc& d = c->d;
  if (d.prec != HPSGD_BF16_MFMA || d.kind == HPSGD_MLP || c->whhb.empty()) return HPSGD_OK;
  auto reg = [&](const Region& r) { return ws + r.offset + (size_t)k0 * r.stride; };
  auto bfreg = [&](const Region& r) { return (__bf16*)reg(r); };
  const bool lm = d.kind == HPSGD_GRU_LM;
  const int B = d.batch, H = d.hidden, L = d.layers;
  const int classes = lm ? d.vocab : d.classes;
  const bool ntc = (B % 8 == 0) && (H % 8 == 0);
  const bool fused_b = gru_fused_bf16_supported(H);
  // the matrices go through one launch (each is a few hundred tiles); what the pack does not
  // take is launched by itself
  Cvt2Pack pack;
  auto copy2 = [&](const float* in, long ld_in, void* out_p, long ld_p, long s_p, void* out_t, long ld_t, long s_t,
                   int R, int C) -> bool {
    if (!launch || cvt2_pack_push(pack, in, ld_in, sR, out_p, ld_p, s_p, out_t, ld_t, s_t, R, C)) return true;
    return launch_cvt2(in, 0, ld_in, sR, out_p, ld_p, s_p, out_t, ld_t, s_t, R, C, groups, st) == hipSuccess;
  };
  for (int l = 0; l < L && l < 16; ++l) {
    const int width = l > 0 ? H : (lm ? d.embed : d.input);
    const float* Wih = rin + c->eoff(c->lidx[l].wih);
    const float* Whh = rin + c->eoff(c->lidx[l].whh);
    if (fused_b && ntc && width % 8 == 0) {
      const bool need_T = l > 0 || lm;  // the input gradient of this layer is needed
      __bf16* wT = need_T ? bfreg(c->wihTl[l]) : nullptr;
      const long s_wT = 2 * (long)c->wihTl[l].stride, s_wb2 = 2 * (long)c->wihbl[l].stride;
      if (cvt2_supported(Wih, 0, width, sR, bfreg(c->wihbl[l]), width, s_wb2, wT, 3 * H, s_wT, 3 * H, width)) {
        if (!copy2(Wih, width, bfreg(c->wihbl[l]), width, s_wb2, wT, 3 * H, s_wT, 3 * H, width)) return HPSGD_EHIP;
        wc.wih[l] = true;
        wc.wihT[l] = need_T;
      }
    }
    if (fused_b) {
      void* wb = reg(c->whhb[l]);
      const long s_wb = 2 * (long)c->whhb[l].stride, s_whT = 2 * (long)c->whhT[l].stride;
      if (cvt2_supported(Whh, 0, H, sR, wb, H, s_wb, bfreg(c->whhT[l]), 3 * H, s_whT, 3 * H, H)) {
        if (!copy2(Whh, H, wb, H, s_wb, bfreg(c->whhT[l]), 3 * H, s_whT, 3 * H, H)) return HPSGD_EHIP;
        wc.whhT[l] = true;
      } else if (launch && launch_cvt_bf16(Whh, H, sR, wb, H, s_wb, 3 * H, H, false, groups, st) != hipSuccess) {
        return HPSGD_EHIP;
      }
      wc.whh[l] = true;
    }
  }
  if (with_head) {
    const size_t oW = c->eoff(c->i_head_w);
    const long clp = (long)round_up(classes, 64);
    const long s_wob = 2 * (long)c->wob.stride, s_woT = 2 * (long)c->woT.stride;
    if (ntc && fused_b && classes % 8 == 0 &&
        cvt2_supported(rin + oW, 0, H, sR, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H)) {
      if (!copy2(rin + oW, H, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H)) return HPSGD_EHIP;
      wc.head = true;
    }
  }
  if (launch && launch_cvt2_pack(pack, groups, st) != hipSuccess) return HPSGD_EHIP;
  return HPSGD_OK;
}

// One local step for `groups` workers whose workspace slices start at worker k0.
// acc (nullable): per-worker gradient accumulators [groups][acc_stride]; the step's gradient
// is added to them (Alg. 2 "accumulate gradients").  Every gradient then goes through the
// gradient buffer: no weight matrix is updated in a GEMM epilogue.
// cloned: rin is ONE model that every worker's replica is a clone of (Alg. 2 "make replica" not
// yet written out): parameters are read from it with group stride 0, rout receives every
// parameter of every worker.
int run_step(hpsgd_ctx* c, int k0, int groups, const float* rin, float* rout, size_t rstride,
             const void* x, const int32_t* y, float lr, float* loss_out, float* ws, hipStream_t s,
             float* acc = nullptr, size_t acc_stride = 0, bool cloned = false) {
  const hpsgd_model_desc& d = c->d;
  const int bf = d.prec == HPSGD_BF16_MFMA ? 1 : 0;
  auto reg = [&](const Region& r) { return ws + r.offset + (size_t)k0 * r.stride; };
  float* grad = reg(c->grad);
  const long sG = (long)c->grad.stride;
  const long sR = (long)rstride;            // of rout
  const long sRi = cloned ? 0L : (long)rstride;  // of rin
  const int B = d.batch;
  int role = HPSGD_ROLE_OTHER;
  c->timer_nested = false;
  StepCtxScope step_scope(c);
  ResidentScope resident;  // orders this step's resident-weight launches against other streams
  // the bf16 copies of the weights are already in this workspace (hpsgd_prepare_replicas); the
  // step changes the weights, so the mark is used once
  hpsgd_ctx::Mark mark{nullptr, nullptr, 0, nullptr, false};
  // (a mark is kept under the replicas' address: rout when they are still clones of rin)
  const bool marked = c->take_mark(cloned ? rout : rin, ws, rstride, mark);
  const bool prepared = bf && marked && k0 == 0 && groups == c->K && (!cloned || mark.clone_src == rin);
  // clones without prepared copies: the step makes the one set itself, from rin
  const bool own_set = cloned && !prepared && bf && k0 == 0;
  const float* head_src = prepared ? mark.clone_src : own_set ? rin : nullptr;
  const bool head_done = prepared && mark.head_done;
  // the replicas are clones of one model (hpsgd_prepare_clones): one set of bf16 weight copies, in
  // worker 0's slice of the workspace, is every worker's operand (group stride 0)
  const bool shared = head_src != nullptr;
  auto wstride = [&](const Region& r) { return shared ? 0L : 2 * (long)r.stride; };
  const unsigned* abort_word = nullptr;  // set when resident-weight recurrence kernels were launched
  c->last_resident = c->last_xproj = c->last_dw = 0;
  // Weight matrices whose SGD update is applied by the epilogue of their own gradient GEMM
  // (replica_out = replica_in - lr * dW, no gradient buffer round trip); every other
  // parameter goes through the gradient buffer and the commit kernel at the end.  A matrix
  // is only updated after the last kernel that reads it (the input-gradient GEMM of its
  // layer) has been issued, so the step may run in place.
  std::vector<char> fused_commit(c->entries.size(), 0);
  // Where the weight-gradient GEMM of `name` writes: the updated matrix itself (epilogue
  // W_out = W_in - lr * dW), or, when gradients are accumulated as well, the gradient buffer.
  struct WgradTarget { float* C; long sC; int epi; const float* aux; };
  auto wgrad_target = [&](int entry) -> WgradTarget {
    const size_t o = c->eoff(entry);
    if (acc) return WgradTarget{grad + o, sG, EPI_STORE, nullptr};
    fused_commit[entry] = 1;
    return WgradTarget{rout + o, sR, EPI_COMMIT, rin + o};
  };

  if (d.kind == HPSGD_MLP) {
    const int L = d.n_mlp_dims - 1;
    const int* dims = d.mlp_dims;
    // A last layer with few classes (the softmax head): forward, loss, its three gradients and its
    // update as the two small launches of the classifier head instead of three GEMMs, the loss
    // kernel and a share of the column sums
    const bool small_head = !bf && L >= 2 && cls_head_supported(B, dims[L], dims[L - 1]) && c->dact.size() + 1 >= (size_t)L;
    // forward
    const float* a_in = (const float*)x;
    long s_in = (long)B * dims[0];
    for (int i = 0; i < (small_head ? L - 1 : L); ++i) {
      float* a_out = reg(c->act[i]);
      role = HPSGD_ROLE_MLP_FWD;
      TRY(gemm(s, groups, bf, B, dims[i + 1], dims[i], a_in, dims[i], s_in, 0, rin + c->eoff(c->fc_w[i]),
               dims[i], sRi, 1, a_out, dims[i + 1], (long)c->act[i].stride,
               i + 1 < L ? EPI_BIAS_RELU : EPI_BIAS, rin + c->eoff(c->fc_b[i]), sRi));
      a_in = a_out;
      s_in = (long)c->act[i].stride;
    }
    // loss; the logits buffer becomes the output delta
    float* delta = reg(c->act[L - 1]);
    float* rowloss = reg(c->rowloss);
    role = HPSGD_ROLE_LOSS;
    if (small_head) {
      const size_t oW = c->eoff(c->fc_w[L - 1]), ob = c->eoff(c->fc_b[L - 1]);
      float* dprev = reg(c->dact[L - 2]);
      if (acc) {
        HIP_TRY(launch_cls_head(a_in, s_in, rin + oW, rin + ob, sRi, y, B, delta, (long)c->act[L - 1].stride, rowloss,
                                (long)c->rowloss.stride, dprev, (long)c->dact[L - 2].stride, grad + oW, grad + ob, sG, lr,
                                0, loss_out, B, dims[L], dims[L - 1], groups, s, 1));
      } else {
        fused_commit[c->fc_w[L - 1]] = 1;
        fused_commit[c->fc_b[L - 1]] = 1;
        HIP_TRY(launch_cls_head(a_in, s_in, rin + oW, rin + ob, sRi, y, B, delta, (long)c->act[L - 1].stride, rowloss,
                                (long)c->rowloss.stride, dprev, (long)c->dact[L - 2].stride, rout + oW, rout + ob, sR, lr,
                                1, loss_out, B, dims[L], dims[L - 1], groups, s, 1));
      }
      delta = dprev;
    } else {
      HIP_TRY(launch_softmax_ce(delta, (long)c->act[L - 1].stride, y, B, delta, rowloss,
                                (long)c->rowloss.stride, B, dims[L], groups, s));
    }
    // backward
    // the bias gradients (column sums of every layer's delta) are taken in one launch behind the
    // last layer, which also applies them unless the gradients are accumulated as well
    ColsumPack cp;
    cp.n = 0;
    cp.blk0[0] = 0;
    cp.lr = lr;
    // (the mean of the per-row losses rides along: a column sum of a B x 1 matrix; the small head
    // has taken it already)
    if (loss_out && !small_head &&
        !colsum_pack_push(cp, rowloss, 1, (long)c->rowloss.stride, loss_out, 1, nullptr, 0, B, 1, 1.0f / (float)B))
      return HPSGD_ESHAPE;
    for (int i = (small_head ? L - 2 : L - 1); i >= 0; --i) {
      const float* a_prev = i > 0 ? reg(c->act[i - 1]) : (const float*)x;
      const long s_prev = i > 0 ? (long)c->act[i - 1].stride : (long)B * dims[0];
      const long s_delta = i == L - 1 ? (long)c->act[i].stride : (long)c->dact[i].stride;
      role = HPSGD_ROLE_MLP_BWD;  // (with the small head the loop starts at layer L-2, whose delta is dact[L-2])
      float* dprev = nullptr;
      if (i > 0) {
        // delta_prev = (delta W) * [a_prev > 0]: before W is updated
        dprev = reg(c->dact[i - 1]);
        TRY(gemm(s, groups, bf, B, dims[i], dims[i + 1], delta, dims[i + 1], s_delta, 0,
                 rin + c->eoff(c->fc_w[i]), dims[i], sRi, 0, dprev, dims[i], (long)c->dact[i - 1].stride,
                 EPI_RELU_MASK, a_prev, s_prev));
      }
      // W' = W - lr * delta^T a_prev
      const WgradTarget wt = wgrad_target(c->fc_w[i]);
      TRY(gemm(s, groups, bf, dims[i + 1], dims[i], B, delta, dims[i + 1], s_delta, 1, a_prev, dims[i],
               s_prev, 0, wt.C, dims[i], wt.sC, wt.epi, wt.aux, sRi, 0, lr));
      {
        const size_t ob = c->eoff(c->fc_b[i]);
        const bool pushed = acc ? colsum_pack_push(cp, delta, dims[i + 1], s_delta, grad + ob, sG, nullptr, 0, B, dims[i + 1])
                                : colsum_pack_push(cp, delta, dims[i + 1], s_delta, rout + ob, sR, rin + ob, sRi, B,
                                                   dims[i + 1]);
        if (pushed && !acc) fused_commit[c->fc_b[i]] = 1;
        if (!pushed)
          HIP_TRY(launch_colsum(delta, dims[i + 1], s_delta, grad + ob, sG, B, dims[i + 1], groups, s));
      }
      if (i > 0) delta = dprev;
    }
    HIP_TRY(launch_colsum_pack(cp, groups, s));
  } else {
    const bool lm = d.kind == HPSGD_GRU_LM;
    const int T = d.seq_len, H = d.hidden, L = d.layers;
    const int TB = T * B;
    const int classes = lm ? d.vocab : d.classes;
    const int32_t* tok = (const int32_t*)x;
    float* gx = reg(c->gx);
    float* dgh = reg(c->dgh);
    float* gh = reg(c->gh);
    float* D = reg(c->D);
    float* dx = reg(c->dx);
    float* logits = reg(c->logits);
    float* rowloss = reg(c->rowloss);
    const long s_gx = (long)c->gx.stride, s_gh = (long)c->gh.stride, s_D = (long)c->D.stride;
    const long s_dx = (long)c->dx.stride, s_log = (long)c->logits.stride;

    // bf16 precision: the weight-gradient and input-gradient GEMMs take contraction-contiguous
    // bf16 operands ("NT" form); the fused step kernels write those copies themselves
    const bool ntc = bf && (B % 8 == 0) && (H % 8 == 0);
    const long TBp = (long)round_up(TB, 64), TB1p = (long)round_up(TB + B, 64);
    auto bfreg = [&](const Region& r) { return (__bf16*)reg(r); };
    bool xT_ready = false;  // the transposed bf16 layer-0 input was made in the forward pass
    // per layer: the transposed bf16 W_hh / W_ih were made in the forward pass, in the same
    // read as the row-major copies
    bool whhT_ready[16] = {false}, wihT_ready[16] = {false};
    // fp32: the recurrence of a layer as one launch (a few for BPTT) with W_hh resident in LDS.
    // Its workgroups wait for each other through flag words in the workspace, zeroed here; pbase
    // follows what the flags read.  A given-up wait shows as NaN in the results (below).
    const bool use_persist = !bf && c->resident && gru_fused_supported(H) && gru_persist_supported(B, H, groups);
    // bf16: the same with the weight slices in registers; its backward launch writes only the bf16
    // copies of the gate gradients, so every GEMM that consumes them must be able to take those
    // (contraction-contiguous bf16 views: batch, hidden size and every layer width multiples of 8)
    bool use_persist_b = bf && c->resident && gru_fused_bf16_supported(H) && gru_persist_bf16_supported(B, H, groups) &&
                         ntc && (lm ? d.embed : d.input) % 8 == 0 && (sG & 3) == 0 &&
                         c->dbp.stride == (size_t)((B + 31) / 32) * 6 * H;
    for (int l = 0; l < L && use_persist_b; ++l) {
      use_persist_b = ((uintptr_t)(grad + c->eoff(c->lidx[l].bih)) & 15) == 0 &&
                      c->eoff(c->lidx[l].bhh) == c->eoff(c->lidx[l].bih) + (size_t)3 * H;
    }
    unsigned* psync = (use_persist || use_persist_b) ? (unsigned*)reg(c->psync) : nullptr;
    unsigned pbase = 0;
    unsigned ticket_launches = 0;  // launches of this step that placed their workgroups by ticket
    if (use_persist || use_persist_b) {
      TRY0(resident.begin(s));
      abort_word = psync;  // (cleared together with the first layer's h_0 below)
    }
    // ---- the head's operands
    const int nrows = lm ? TB : B;
    const size_t oW = c->eoff(c->i_head_w), ob = c->eoff(c->i_head_b);
    const long nrp = (long)round_up(nrows, 64), clp = (long)round_up(classes, 64);
    const long s_dlb = 2 * (long)c->dlogb.stride, s_wob = wstride(c->wob);
    const long s_woT = wstride(c->woT), s_dlT = 2 * (long)c->dlogT.stride;
    // bf16 precision with every head operand available as bf16: h of the top layer (written
    // by its step kernels), head.W rounded once (row-major and transposed in one pass), the
    // logit gradient emitted in bf16 by the loss kernel and transposed from there
    const bool headb =
        ntc && gru_fused_bf16_supported(H) && classes % 8 == 0 &&
        cvt2_supported(rin + oW, 0, H, sRi, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H) &&
        softmax_ce_bf16_supported(logits, s_log, bfreg(c->dlogb), clp, s_dlb, classes) &&
        cvt2_supported(bfreg(c->dlogb), 1, clp, s_dlb, nullptr, 0, 0, bfreg(c->dlogT), nrp, s_dlT, nrows, classes);
    // the layers' bf16 weight copies: all at the start (nothing but the replicas feeds them),
    // unless they were made before the step
    WeightCopies wc;
    role = HPSGD_ROLE_OTHER;
    TRY(weight_copies(c, rin, sRi, k0, own_set ? 1 : groups, ws, s, !prepared, false, wc));
    // ---- forward
    const float* lin = (const float*)x;
    long s_lin = (long)TB * d.input;
    int width = d.input;
    if (lm) {
      float* xe = reg(c->xe);
      role = HPSGD_ROLE_EMBED;
      HIP_TRY(launch_embed_fwd(rin + c->eoff(c->i_embed), sRi, tok, TB, xe, (long)c->xe.stride, TB,
                               d.embed, groups, s));
      lin = xe;
      s_lin = (long)c->xe.stride;
      width = d.embed;
    }
    // everything a step clears before its first layer, in one launch: the flag words of the
    // resident-weight launches, h_0 of every layer (fp32, and in bf16 precision the bf16 copy and
    // the first B columns of the transposed copy)
    bool cleared = false;
    bool head_early = false;
    {
      FillPack fp;
      fp.n = 0;
      fp.blk0[0] = 0;
      fp.max_groups = 0;
      bool ok = true;
      if (psync) ok = ok && fill_pack_push(fp, (float*)psync, 0, 1, (long)gru_persist_sync_words(B, groups), 0, 1);
      for (int l = 0; l < L && ok; ++l) {
        ok = ok && fill_pack_push(fp, reg(c->hs[l]), 0, 1, (long)B * H, c->hs[l].stride, groups);
        if (bf && gru_fused_bf16_supported(H) && ntc)
          ok = ok && fill_pack_push(fp, reg(c->hsT[l]), TB1p / 2, H, B / 2, c->hsT[l].stride, groups);
      }
      if (bf && gru_fused_bf16_supported(H))
        ok = ok && fill_pack_push(fp, reg(c->hb), 0, 1, (long)B * H / 2, c->hb.stride, groups);
      if (use_persist_b)
        ok = ok && fill_pack_push(fp, reg(c->hx), 0, 1, (long)(gru_persist_bf16_exchange_elems(B, H) / 2), c->hx.stride, groups);
      if (use_persist)
        ok = ok && fill_pack_push(fp, reg(c->hx), 0, 1, (long)gru_persist_exchange_words(B, H), c->hx.stride, groups);
      if (ok) {
        role = HPSGD_ROLE_OTHER;
        HIP_TRY(launch_fill_pack(fp, s));
        cleared = true;
      }
    }
    for (int l = 0; l < L; ++l) {
      float* hs = reg(c->hs[l]);
      float* sv = reg(c->sv[l]);
      const long s_hs = (long)c->hs[l].stride, s_sv = (long)c->sv[l].stride;
      role = HPSGD_ROLE_OTHER;
      if (!cleared) {
        HIP_TRY(launch_fill_zero(hs, (size_t)B * H, (size_t)s_hs, groups, s, l == 0 ? (float*)psync : nullptr,
                                 l == 0 && psync ? gru_persist_sync_words(B, groups) : 0));
        if (use_persist && l == 0)
          HIP_TRY(launch_fill_zero(reg(c->hx), gru_persist_exchange_words(B, H), c->hx.stride, groups, s));
      }
      const float* Whh = rin + c->eoff(c->lidx[l].whh);
      const bool fused = !bf && gru_fused_supported(H) && ((uintptr_t)Whh & 15) == 0 && (sRi & 3) == 0;
      const bool fused_b = bf && gru_fused_bf16_supported(H);
      const bool persist = fused && use_persist;
      // a narrow layer input: the resident-weight kernel does the input projection itself
      const float* Wih0 = rin + c->eoff(c->lidx[l].wih);
      const bool xproj = persist && gru_persist_xproj_supported(H, width) && ((uintptr_t)lin & 15) == 0 &&
                         (s_lin & 3) == 0 && ((uintptr_t)Wih0 & 15) == 0;
      if (!xproj) {
        const float* Wih = rin + c->eoff(c->lidx[l].wih);
        NtView va{lin, 0, width, s_lin}, vb{Wih, 0, width, sRi};
        // bf16 precision: both operands as row-major bf16 copies (the layer below wrote its
        // h in bf16; the layer-0 input and W_ih are rounded here, the input also transposed
        // for the weight-gradient GEMM)
        if (fused_b && ntc && width % 8 == 0) {
          role = HPSGD_ROLE_OTHER;
          const long s_xb = 2 * (long)c->xb.stride;
          if (l > 0) {
            va = NtView{(const __bf16*)reg(c->hb) + (size_t)B * H, 1, H, 2 * (long)c->hb.stride};
          } else if (cvt2_supported(lin, 0, width, s_lin, bfreg(c->xb), width, s_xb, bfreg(c->xT), TBp,
                                    2 * (long)c->xT.stride, TB, width)) {
            HIP_TRY(launch_cvt2(lin, 0, width, s_lin, bfreg(c->xb), width, s_xb, bfreg(c->xT), TBp,
                                2 * (long)c->xT.stride, TB, width, groups, s));
            va = NtView{bfreg(c->xb), 1, width, s_xb};
            xT_ready = true;
          }
          if (wc.wih[l]) {  // made at the start of the step, or before it
            vb = NtView{bfreg(c->wihbl[l]), 1, width, wstride(c->wihbl[l])};
            wihT_ready[l] = wc.wihT[l];
          }
        }
        // The one copy of the head matrix that serves cloned replicas: beside the top layer's
        // input projection (between two resident-weight launches, when the synchronising stream
        // has finished), joined before the recurrence starts.
        const bool early = l == L - 1 && l > 0 && headb && !head_done && head_src && c->aux && c->ev_fork && c->ev_join;
        if (early) {
          if (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess ||
              launch_cvt2(head_src + oW, 0, H, 0, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H, 1,
                          c->aux) != hipSuccess ||
              hipEventRecord(c->ev_join, c->aux) != hipSuccess)
            return HPSGD_EHIP;
          head_early = true;
        }
        role = HPSGD_ROLE_GEMM_INPUT;
        TRY(gemm2(s, groups, bf, TB, 3 * H, width, lin, width, s_lin, 0, Wih, width, sRi, 1, gx, 3 * H, s_gx,
                  EPI_BIAS, rin + c->eoff(c->lidx[l].bih), sRi, va, vb));
        if (early && hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess) return HPSGD_EHIP;
      }
      // bf16 path: bf16 copy of W_hh (kept in the W_hh^T region, which the forward pass does
      // not use) and of h
      void* wb = wc.whh[l] ? reg(c->whhb[l]) : reg(c->wt);
      const long s_wb = wc.whh[l] ? wstride(c->whhb[l]) : 2 * (long)c->wt.stride;
      __bf16* hb = fused_b ? (__bf16*)reg(c->hb) : nullptr;
      const long s_hb = 2 * (long)c->hb.stride;
      __bf16* hT = (fused_b && ntc) ? bfreg(c->hsT[l]) : nullptr;  // hsT exists in bf16 precision only
      const long s_hT = hT ? 2 * (long)c->hsT[l].stride : 0;
      if (fused_b) {
        role = HPSGD_ROLE_OTHER;
        if (!wc.whh[l]) return HPSGD_ESHAPE;  // (bf16 precision allocates the per-layer copies)
        whhT_ready[l] = wc.whhT[l];
        if (!cleared) {
          HIP_TRY(launch_fill_zero((float*)hb, (size_t)B * H / 2, (size_t)c->hb.stride, groups, s));
          if (use_persist_b)
            HIP_TRY(launch_fill_zero(reg(c->hx), gru_persist_bf16_exchange_elems(B, H) / 2, c->hx.stride, groups, s));
          if (hT)  // h_0 = 0: the first B columns of the transposed copy
            HIP_TRY(launch_fill_zero_2d((float*)hT, TB1p / 2, H, B / 2, c->hsT[l].stride, groups, s));
        }
      }
      // one event pair around the whole time loop when its launches are all of one role
      const bool persist_b = fused_b && use_persist_b && hT != nullptr;
      TimerScope loop_fwd(c, HPSGD_ROLE_GEMM_REC_FWD, s, (persist || persist_b) ? 1 : (fused || fused_b) ? T : 0);
      c->timer_nested = loop_fwd.active() && (fused || fused_b);
      if (persist) {
        role = HPSGD_ROLE_GEMM_REC_FWD;
        HIP_TRY(launch_gru_fwd_persist(Whh, rin + c->eoff(c->lidx[l].bhh), sRi, gx, s_gx, hs, s_hs, reg(c->hx),
                                       (long)c->hx.stride, sv, s_sv, B, H, T,
                                       groups, psync, pbase, c->spin_limit, xproj ? lin : nullptr, s_lin, width,
                                       Wih0, rin + c->eoff(c->lidx[l].bih), c->device_scope, &ticket_launches, s));
        pbase += (unsigned)T * gru_persist_count_per_step(H);
        ++c->last_resident;
        c->last_xproj += xproj ? 1 : 0;
        resident.note();
      }
      if (persist_b) {
        role = HPSGD_ROLE_GEMM_REC_FWD;
        HIP_TRY(launch_gru_fwd_persist_bf16(wb, s_wb, rin + c->eoff(c->lidx[l].bhh), sRi, gx, s_gx, hs, s_hs, hb, s_hb,
                                            bfreg(c->hx), 2 * (long)c->hx.stride, sv, s_sv, hT, TB1p, s_hT, B, H, T, groups,
                                            psync, pbase, c->spin_limit, c->device_scope, &ticket_launches, s));
        pbase += (unsigned)T * gru_persist_bf16_count_per_step(H);
        ++c->last_resident;
        resident.note();
      }
      for (int t = 0; t < T && !persist && !persist_b; ++t) {
        role = HPSGD_ROLE_GEMM_REC_FWD;
        if (fused_b) {
          HIP_TRY(launch_gru_fwd_step_bf16(wb, s_wb, rin + c->eoff(c->lidx[l].bhh), sRi, gx + (size_t)t * B * 3 * H,
                                           s_gx, hs + (size_t)t * B * H, hs + (size_t)(t + 1) * B * H, s_hs,
                                           hb + (size_t)t * B * H, hb + (size_t)(t + 1) * B * H, s_hb,
                                           sv + (size_t)t * B * 4 * H, s_sv,
                                           hT ? hT + (size_t)(t + 1) * B : nullptr, TB1p, s_hT, B, H, groups,
                                           s));
          continue;
        }
        if (fused) {
          HIP_TRY(launch_gru_fwd_step(Whh, rin + c->eoff(c->lidx[l].bhh), sRi, gx + (size_t)t * B * 3 * H, s_gx,
                                      hs + (size_t)t * B * H, hs + (size_t)(t + 1) * B * H, s_hs,
                                      sv + (size_t)t * B * 4 * H, s_sv, B, H, groups, s));
          continue;
        }
        TRY(gemm(s, groups, bf, B, 3 * H, H, hs + (size_t)t * B * H, H, s_hs, 0, Whh, H, sRi, 1, gh, 3 * H,
                 s_gh, EPI_BIAS, rin + c->eoff(c->lidx[l].bhh), sRi));
        role = HPSGD_ROLE_CELL_FWD;
        HIP_TRY(launch_gru_cell_fwd(gx + (size_t)t * B * 3 * H, s_gx, gh, s_gh, hs + (size_t)t * B * H,
                                    hs + (size_t)(t + 1) * B * H, s_hs, sv + (size_t)t * B * 4 * H,
                                    s_sv, B, H, groups, s));
      }
      c->timer_nested = false;
      lin = hs + (size_t)B * H;
      s_lin = s_hs;
      width = H;
    }
    // ---- head and loss
    const float* top = reg(c->hs[L - 1]);
    const long s_top = (long)c->hs[L - 1].stride;
    const float* feats = lm ? top + (size_t)B * H : top + (size_t)T * B * H;
    if (headb) {
      role = HPSGD_ROLE_OTHER;
      // the bf16 copies of the head's weights: here, when the synchronising stream has finished and
      // the copy has the memory system to itself (beside a resident-weight launch it takes 2.3
      // times as long and slows that launch by more than it takes alone; at the start of the step it
      // shares the bandwidth with the merge and the clone)
      if (head_done || head_early) {
        // made with the layers' copies, before the step, or beside the top layer's input projection
      } else if (head_src) {  // the replicas are clones of one model: one copy of its head matrix serves all workers
        HIP_TRY(launch_cvt2(head_src + oW, 0, H, 0, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H,
                            1, s));
      } else if (!prepared) {
        HIP_TRY(launch_cvt2(rin + oW, 0, H, sRi, bfreg(c->wob), H, s_wob, bfreg(c->woT), clp, s_woT, classes, H,
                            groups, s));
      }
      const long s_hb = 2 * (long)c->hb.stride;
      const NtView va{(const __bf16*)reg(c->hb) + (size_t)(lm ? B : T * B) * H, 1, H, s_hb};
      const NtView vb{bfreg(c->wob), 1, H, s_wob};
      role = HPSGD_ROLE_GEMM_HEAD;
      TRY(gemm2(s, groups, bf, nrows, classes, H, feats, H, s_top, 0, rin + oW, H, sRi, 1, logits, classes,
                s_log, EPI_BIAS, rin + ob, sRi, va, vb));
      role = HPSGD_ROLE_LOSS;
      // the head's bias gradient: column sums of the unrounded logit gradient, per block of rows
      // in the loss kernel, added up below (else recomputed from the logits in a pass of its own)
      // (the partial sums of the groups lie back to back, as the adding kernel reads them)
      // (sized for all K workers also when fewer are stepped: the sums then do not depend on the entry point)
      const int n_colparts = softmax_ce_bf16_row_blocks(nrows, c->K, classes);
      const long s_colpart = (long)n_colparts * classes;
      const bool colsum_fused = (((uintptr_t)(grad + ob) | (uintptr_t)reg(c->colpart)) & 15) == 0 && sG % 4 == 0 &&
                                s_colpart % 4 == 0 && (size_t)s_colpart <= c->colpart.stride;
      HIP_TRY(launch_softmax_ce_bf16(logits, s_log, y, nrows, bfreg(c->dlogb), clp, s_dlb, rowloss,
                                     (long)c->rowloss.stride, reg(c->rowstat), (long)c->rowstat.stride, nrows,
                                     classes, groups, s, colsum_fused ? reg(c->colpart) : nullptr, s_colpart, c->K));
      role = HPSGD_ROLE_GEMM_HEAD;
      const NtView vdl{bfreg(c->dlogb), 1, clp, s_dlb}, vwT{bfreg(c->woT), 1, clp, s_woT};
      const NtView vdT{bfreg(c->dlogT), 1, nrp, s_dlT};
      const NtView vhT{bfreg(c->hsT[L - 1]) + (lm ? B : T * B), 1, TB1p, 2 * (long)c->hsT[L - 1].stride};
      const WgradTarget wt = wgrad_target(c->i_head_w);
      // The head's input gradient and weight gradient need the same logit gradient and nothing of
      // each other.  The former has fewer tiles than the chip has CUs (a long contraction over
      // the classes): with an auxiliary stream the two run side by side and the tiles of the
      // weight gradient fill the CUs the other leaves idle.  One event pair brackets both.
      const bool side_by_side = c->aux && c->ev_fork && c->ev_join;
      // What needs the loss kernel's results only (the mean loss, the bias gradient from its
      // partial column sums): side by side, the weight gradient outlasts the input gradient, and
      // these follow the latter on this stream while the other stream is still busy.
      auto loss_followers = [&]() -> int {
        if (loss_out)
          HIP_TRY(launch_loss_mean(rowloss, (long)c->rowloss.stride, loss_out, nrows, groups, s));
        if (colsum_fused)
          HIP_TRY(launch_reduce_parts(reg(c->colpart), n_colparts, (size_t)classes, nullptr, 0,
                                      grad + ob, (size_t)sG, 0.f, 0, groups, s));
        else
          HIP_TRY(launch_colsum_softmax(logits, s_log, reg(c->rowstat), (long)c->rowstat.stride, y, nrows,
                                        grad + ob, sG, nrows, classes, groups, s));
        return HPSGD_OK;
      };
      if (!side_by_side) TRY0(loss_followers());
      // The transposed logit gradient is the weight gradient's operand only: side by side it is
      // made on that product's stream, under the start of the input gradient.
      if (side_by_side &&
          (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess))
        return HPSGD_EHIP;
      role = HPSGD_ROLE_OTHER;
      if (side_by_side) {
        if (launch_cvt2(bfreg(c->dlogb), 1, clp, s_dlb, nullptr, 0, 0, bfreg(c->dlogT), nrp, s_dlT, nrows, classes,
                        groups, c->aux) != hipSuccess)
          return HPSGD_EHIP;
      } else {
        HIP_TRY(launch_cvt2(bfreg(c->dlogb), 1, clp, s_dlb, nullptr, 0, 0, bfreg(c->dlogT), nrp, s_dlT, nrows,
                            classes, groups, s));
      }
      role = HPSGD_ROLE_GEMM_HEAD;
      {
        TimerScope pair(c, role, s, 2);
        const bool nested = c->timer_nested;
        c->timer_nested = c->timer_nested || pair.active();
        // (bf16 views only: the fp32 head matrix may be updated in place by the GEMM beside this one)
        TRY(gemm2(s, groups, bf, nrows, H, classes, logits, classes, s_log, 0, rin + oW, H, sRi, 0, lm ? dx : D, H,
                  lm ? s_dx : s_D, EPI_STORE, nullptr, 0, vdl, vwT, 0.f, true));
        TRY(gemm2(side_by_side ? c->aux : s, groups, bf, classes, H, nrows, logits, classes, s_log, 1, feats, H, s_top,
                  0, wt.C, H, wt.sC, wt.epi, wt.aux, sRi, vdT, vhT, lr));
        if (side_by_side) {
          const int saved_role = role;
          role = HPSGD_ROLE_OTHER;
          TRY0(loss_followers());
          role = saved_role;
        }
        if (side_by_side &&
            (hipEventRecord(c->ev_join, c->aux) != hipSuccess || hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess))
          return HPSGD_EHIP;
        c->timer_nested = nested;
      }
    } else if (!bf && !lm && cls_head_supported(nrows, classes, H)) {
      // a classifier head with few classes: forward and loss in one small launch, the three
      // gradients and the update (or the gradients, when they are accumulated as well) in another
      role = HPSGD_ROLE_GEMM_HEAD;
      TimerScope ts_(c, role, s);
      if (acc) {
        HIP_TRY(launch_cls_head(feats, s_top, rin + oW, rin + ob, sRi, y, nrows, logits, s_log, rowloss,
                                (long)c->rowloss.stride, D, s_D, grad + oW, grad + ob, sG, lr, 0, loss_out, nrows,
                                classes, H, groups, s));
      } else {
        fused_commit[c->i_head_w] = 1;
        fused_commit[c->i_head_b] = 1;
        HIP_TRY(launch_cls_head(feats, s_top, rin + oW, rin + ob, sRi, y, nrows, logits, s_log, rowloss,
                                (long)c->rowloss.stride, D, s_D, rout + oW, rout + ob, sR, lr, 1, loss_out, nrows,
                                classes, H, groups, s));
      }
    } else {
      role = HPSGD_ROLE_GEMM_HEAD;
      {
        const NtView va{feats, 0, H, s_top}, vb{rin + oW, 0, H, sRi};
        TRY(gemm2(s, groups, bf, nrows, classes, H, feats, H, s_top, 0, rin + oW, H, sRi, 1, logits, classes,
                  s_log, EPI_BIAS, rin + ob, sRi, va, vb));
      }
      role = HPSGD_ROLE_LOSS;
      HIP_TRY(launch_softmax_ce(logits, s_log, y, nrows, logits, rowloss, (long)c->rowloss.stride, nrows,
                                classes, groups, s));
      if (loss_out)
        HIP_TRY(launch_loss_mean(rowloss, (long)c->rowloss.stride, loss_out, nrows, groups, s));
      // ---- backward: head
      // bf16 precision: transposed bf16 copies (contraction-contiguous operands for the NT kernel)
      if (ntc) {
        role = HPSGD_ROLE_OTHER;
        if (!gru_fused_bf16_supported(H))  // else written by the forward step kernels
          for (int l = 0; l < L; ++l)      // hs^T of every layer: [H][(T+1)B]
            HIP_TRY(launch_cvt_bf16(reg(c->hs[l]), H, (long)c->hs[l].stride, bfreg(c->hsT[l]), TB1p,
                                    2 * (long)c->hsT[l].stride, TB + B, H, true, groups, s));
        HIP_TRY(launch_cvt_bf16(logits, classes, s_log, bfreg(c->dlogT), nrp, 2 * (long)c->dlogT.stride, nrows,
                                classes, true, groups, s));
        HIP_TRY(launch_cvt_bf16(rin + oW, H, sRi, bfreg(c->woT), clp, 2 * (long)c->woT.stride, classes, H, true,
                                groups, s));
      }
      role = HPSGD_ROLE_GEMM_HEAD;
      {
        NtView va, vb, vw;
        if (ntc) {
          va = NtView{bfreg(c->dlogT), 1, nrp, 2 * (long)c->dlogT.stride};
          vb = NtView{bfreg(c->hsT[L - 1]) + (lm ? B : T * B), 1, TB1p, 2 * (long)c->hsT[L - 1].stride};
          vw = NtView{bfreg(c->woT), 1, clp, 2 * (long)c->woT.stride};
        }
        const NtView vl{logits, 0, classes, s_log};
        if (lm) {
          TRY(gemm2(s, groups, bf, TB, H, classes, logits, classes, s_log, 0, rin + oW, H, sRi, 0, dx, H, s_dx,
                    EPI_STORE, nullptr, 0, vl, vw));
        } else {
          TRY(gemm2(s, groups, bf, B, H, classes, logits, classes, s_log, 0, rin + oW, H, sRi, 0, D, H, s_D,
                    EPI_STORE, nullptr, 0, vl, vw));
        }
        const WgradTarget wt = wgrad_target(c->i_head_w);
        TRY(gemm2(s, groups, bf, classes, H, nrows, logits, classes, s_log, 1, feats, H, s_top, 0, wt.C, H, wt.sC,
                  wt.epi, wt.aux, sRi, va, vb, lr));
        HIP_TRY(launch_colsum(logits, classes, s_log, grad + ob, sG, nrows, classes, groups, s));
      }
    }
    // the embedding gradient from the first layer's input gradient dx (Alg. 2 "update replica"
    // for the table, when the update is in place)
    bool embed_done = false;
    // clones: the table is written out first (one read, a write per worker), then updated like
    // one that is already there.  (Nothing of the step reads the output table, so the copy could be
    // issued earlier; beside the layer above's weight gradients it cost more than it saved here.)
    bool table_out = false;
    auto embed_table_out = [&](hipStream_t st) -> int {
      const size_t oE = c->eoff(c->i_embed);
      if (table_out || acc || !cloned || !lm || !aligned16(rin + oE) || !aligned16(rout + oE) || (sR & 3) != 0 ||
          groups > HPSGD_KMAX)
        return HPSGD_OK;
      PtrPack pk;
      for (int g = 0; g < groups; ++g) pk.p[g] = rout + oE + (size_t)g * sR;
      if (launch_sync_all(rin + oE, pk, groups, nullptr, (size_t)d.vocab * d.embed, st) != hipSuccess) return HPSGD_EHIP;
      table_out = true;
      return HPSGD_OK;
    };
    auto embed_grad = [&](hipStream_t st) -> int {
      const size_t oE = c->eoff(c->i_embed);
      TRY0(embed_table_out(st));
      if (!acc && (rin == rout || table_out)) {
        // an update in place: only the rows of the tokens of the batch change, and their owners
        // write them; no gradient table to clear, fill and stream through the commit kernel
        fused_commit[c->i_embed] = 1;
        if (launch_embed_bwd(dx, s_dx, tok, TB, rout + oE, sR, TB, d.embed, groups, st, rin + oE, sRi, lr) != hipSuccess)
          return HPSGD_EHIP;
      } else {
        if (launch_fill_zero(grad + oE, (size_t)d.vocab * d.embed, (size_t)sG, groups, st) != hipSuccess ||
            launch_embed_bwd(dx, s_dx, tok, TB, grad + oE, sG, TB, d.embed, groups, st) != hipSuccess)
          return HPSGD_EHIP;
      }
      return HPSGD_OK;
    };
    const float* above = nullptr;
    // the gradient carried into a layer's last step is zero unless the head wrote it (the
    // classifier on the top layer): a resident-weight launch is told so, any other path has D cleared
    bool d_zero = false;
    if (lm) {
      above = dx;
      d_zero = true;
    }
    // ---- backward: GRU layers, top to bottom
    for (int l = L - 1; l >= 0; --l) {
      const float* hs = reg(c->hs[l]);
      const float* sv = reg(c->sv[l]);
      const long s_hs = (long)c->hs[l].stride, s_sv = (long)c->sv[l].stride;
      const int win = l > 0 ? H : (lm ? d.embed : d.input);
      ReducePack rp;
      rp.n = 0;
      rp.blk0[0] = 0;
      rp.lr = lr;
      // queued for the layer's one adding launch; a segment that launch cannot take runs by itself
      auto queue_reduce = [&](const float* parts, int n_parts, size_t n, const float* in, size_t s_in, float* out,
                              size_t s_out, int commit) -> int {
        if (reduce_pack_push(rp, parts, n_parts, n, in, s_in, out, s_out, commit)) return HPSGD_OK;
        return launch_reduce_parts(parts, n_parts, n, in, s_in, out, s_out, lr, commit, groups, s) == hipSuccess
                   ? HPSGD_OK
                   : HPSGD_EHIP;
      };
      const float* layer_in;
      long s_layer_in;
      if (l > 0) {
        layer_in = reg(c->hs[l - 1]) + (size_t)B * H;
        s_layer_in = (long)c->hs[l - 1].stride;
      } else if (lm) {
        layer_in = reg(c->xe);
        s_layer_in = (long)c->xe.stride;
      } else {
        layer_in = (const float*)x;
        s_layer_in = (long)TB * d.input;
      }
      float* dgx = gx;  // the gate pre-activation buffer is free once the layer's forward is done
      const float* Whh = rin + c->eoff(c->lidx[l].whh);
      const bool fused = !bf && gru_fused_supported(H) && ((uintptr_t)Whh & 15) == 0 && (sRi & 3) == 0;
      const bool fused_b = bf && gru_fused_bf16_supported(H);
      float* wt = reg(c->wt);
      const long s_wt = (long)c->wt.stride;
      __bf16* dghb = fused_b ? (__bf16*)reg(c->dghb) : nullptr;
      const long s_dgb = 2 * (long)c->dghb.stride;
      const bool stepT = fused_b && ntc && win % 8 == 0;  // the step kernels write the bf16 copies
      __bf16* dgxb = stepT ? bfreg(c->dgxb) : nullptr;
      const long s_T = 2 * (long)c->dgxT.stride;
      if (fused && !(use_persist)) {
        role = HPSGD_ROLE_OTHER;
        HIP_TRY(launch_transpose(Whh, sRi, wt, s_wt, 3 * H, H, groups, s));
      }
      const void* wtb = wt;   // bf16 W_hh^T of this layer
      long s_wtb = 2 * s_wt;
      if (fused_b && whhT_ready[l]) {
        wtb = bfreg(c->whhT[l]);
        s_wtb = wstride(c->whhT[l]);
      } else if (fused_b) {
        role = HPSGD_ROLE_OTHER;
        HIP_TRY(launch_cvt_bf16(Whh, H, sRi, wt, 3 * H, 2 * s_wt, 3 * H, H, true, groups, s));
      }
      // fp32 path with an auxiliary stream: the weight-gradient GEMMs of the time steps that
      // BPTT has already finished run on that stream beside the rest of the recurrence (the
      // recurrence is latency-bound and leaves the matrix cores mostly idle).  The steps are
      // cut into chunks; chunk c's GEMMs are issued when BPTT has walked past it, the last
      // one follows on the main stream after the join.  Fixed chunking: deterministic.
      const bool persist = fused && use_persist;
      const bool persist_b = fused_b && use_persist_b && stepT;
      if (d_zero && !persist && !persist_b) {
        role = HPSGD_ROLE_OTHER;
        HIP_TRY(launch_fill_zero(D, (size_t)B * H, (size_t)s_D, groups, s));
      }
      // the resident-weight kernel accumulates dW_hh itself (one partial sum per batch-row tile)
      float* dwp = (persist && c->dwp.stride == (size_t)((B + 31) / 32) * 3 * H * H) ? reg(c->dwp) : nullptr;
      // ... and the bias gradients, when their partial sums can be added with 16-byte accesses
      float* dbp = persist_b ? reg(c->dbp)  // (its conditions were checked with use_persist_b)
                   : (persist && c->dbp.stride == (size_t)((B + 31) / 32) * 6 * H && (sG & 3) == 0 &&
                      ((uintptr_t)(grad + c->eoff(c->lidx[l].bih)) & 15) == 0 &&
                      c->eoff(c->lidx[l].bhh) == c->eoff(c->lidx[l].bih) + (size_t)3 * H)
                       ? reg(c->dbp)
                       : nullptr;
      const int NC = (c->aux && fused && !persist && T >= 8) ? 4 : 1;
      auto chunk_lo = [&](int ch) { return (int)((long)T * ch / NC); };
      auto wgrad_rows = [&](hipStream_t st, int t0, int t1, int epi) -> int {
        const size_t r0 = (size_t)t0 * B;
        const int rows = (t1 - t0) * B;
        const int bg = st != s;  // on the auxiliary stream: beside the recurrence
        int rc = gemm(st, groups, bf, 3 * H, win, rows, dgx + r0 * 3 * H, 3 * H, s_gx, 1, layer_in + r0 * win,
                      win, s_layer_in, 0, grad + c->eoff(c->lidx[l].wih), win, sG, epi, nullptr, 0, bg);
        if (rc != HPSGD_OK) return rc;
        return gemm(st, groups, bf, 3 * H, H, rows, dgh + r0 * 3 * H, 3 * H, s_gx, 1, hs + r0 * H, H, s_hs, 0,
                    grad + c->eoff(c->lidx[l].whh), H, sG, epi, nullptr, 0, bg);
      };
      {
      TimerScope loop_bwd(c, HPSGD_ROLE_GEMM_REC_BWD, s, (persist || persist_b) ? 1 : (fused || fused_b) ? T : 0);
      c->timer_nested = loop_bwd.active() && (fused || fused_b);
      int next_chunk = NC - 1;  // the chunk BPTT is walking through
      // resident weights: all of BPTT is one launch; its weight-gradient GEMMs follow it (work
      // that shares the CUs with this launch slows its chain of waits by more than it hides)
      if (persist) {
        role = HPSGD_ROLE_GEMM_REC_BWD;
        // (the row-major gate gradients only when a later launch reads them)
        HIP_TRY(launch_gru_bwd_persist(Whh, sRi, (dwp && dbp) ? nullptr : dgh, reg(c->dghx), (long)c->dghx.stride, dgx, s_gx,
                                       D, s_D, d_zero, above, s_dx, sv, s_sv, hs, s_hs, B, H, T,
                                       T, 0, groups, psync, pbase, c->spin_limit, dwp, dbp, c->device_scope, &ticket_launches, s));
        c->last_dw += dwp ? 1 : 0;
        pbase += (unsigned)T * gru_persist_count_per_step(H);
        if (l == 0) TRY0(resident.mark());
        else resident.note();
      }
      if (persist_b) {
        role = HPSGD_ROLE_GEMM_REC_BWD;
        HIP_TRY(launch_gru_bwd_persist_bf16(wtb, s_wtb, bfreg(c->dghx), 2 * (long)c->dghx.stride, s_dgb, D, s_D, d_zero,
                                            above, s_dx, sv, s_sv, hs, s_hs, dgxb, bfreg(c->dgxT), bfreg(c->dghT), TBp, s_T, dbp, B,
                                            H, T, groups, psync, pbase, c->spin_limit, c->device_scope, &ticket_launches, s));
        pbase += (unsigned)T * gru_persist_bf16_count_per_step(H);
        if (l == 0) TRY0(resident.mark());
        else resident.note();
      }
      for (int t = T - 1; t >= 0 && !persist && !persist_b; --t) {
        if (NC > 1 && next_chunk >= 1 && t < chunk_lo(next_chunk)) {
          // steps [chunk_lo, chunk_hi) are done: hand their weight gradients to the aux stream
          if (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess)
            return HPSGD_EHIP;
          const int rc = wgrad_rows(c->aux, chunk_lo(next_chunk), chunk_lo(next_chunk + 1),
                                    next_chunk == NC - 1 ? EPI_STORE : EPI_ACCUM);
          if (rc != HPSGD_OK) return rc;
          --next_chunk;
        }
        const float* above_t = above ? above + (size_t)t * B * H : nullptr;
        if (fused_b) {
          role = HPSGD_ROLE_GEMM_REC_BWD;
          HIP_TRY(launch_gru_bwd_step_bf16(wtb, s_wtb, t + 1 < T ? dghb + (size_t)(t + 1) * B * 3 * H : nullptr,
                                           dghb + (size_t)t * B * 3 * H, s_dgb, D, s_D, above_t, s_dx,
                                           sv + (size_t)t * B * 4 * H, s_sv, hs + (size_t)t * B * H, s_hs,
                                           dgx + (size_t)t * B * 3 * H, dgh + (size_t)t * B * 3 * H, s_gx,
                                           dgxb ? dgxb + (size_t)t * B * 3 * H : nullptr,
                                           dgxb ? bfreg(c->dgxT) + (size_t)t * B : nullptr,
                                           dgxb ? bfreg(c->dghT) + (size_t)t * B : nullptr, TBp, s_T, B, H,
                                           groups, s));
          continue;
        }
        if (fused) {
          role = HPSGD_ROLE_GEMM_REC_BWD;
          HIP_TRY(launch_gru_bwd_step(wt, s_wt, t + 1 < T ? dgh + (size_t)(t + 1) * B * 3 * H : nullptr, s_gx,
                                      D, s_D, above_t, s_dx, sv + (size_t)t * B * 4 * H, s_sv,
                                      hs + (size_t)t * B * H, s_hs, dgx + (size_t)t * B * 3 * H,
                                      dgh + (size_t)t * B * 3 * H, B, H, groups, s));
          continue;
        }
        role = HPSGD_ROLE_CELL_BWD;
        HIP_TRY(launch_gru_cell_bwd(D, s_D, above_t, s_dx, sv + (size_t)t * B * 4 * H, s_sv,
                                    hs + (size_t)t * B * H, s_hs, dgx + (size_t)t * B * 3 * H,
                                    dgh + (size_t)t * B * 3 * H, s_gx, B, H, groups, s));
        role = HPSGD_ROLE_GEMM_REC_BWD;
        if (t > 0)
          TRY(gemm(s, groups, bf, B, H, 3 * H, dgh + (size_t)t * B * 3 * H, 3 * H, s_gx, 0, Whh, H, sRi, 0, D,
                   H, s_D, EPI_ACCUM, nullptr, 0));
      }
      c->timer_nested = false;
      }
      const float* Wih = rin + c->eoff(c->lidx[l].wih);
      const bool need_dx = l > 0 || lm;
      NtView v_dgxT, v_dghT, v_xT, v_hsT, v_wihT;
      if (ntc && win % 8 == 0) {
        role = HPSGD_ROLE_OTHER;
        if (!stepT) {
          HIP_TRY(launch_cvt_bf16(dgx, 3 * H, s_gx, bfreg(c->dgxT), TBp, 2 * (long)c->dgxT.stride, TB, 3 * H,
                                  true, groups, s));
          HIP_TRY(launch_cvt_bf16(dgh, 3 * H, s_gx, bfreg(c->dghT), TBp, 2 * (long)c->dghT.stride, TB, 3 * H,
                                  true, groups, s));
        }
        v_dgxT = NtView{bfreg(c->dgxT), 1, TBp, 2 * (long)c->dgxT.stride};
        v_dghT = NtView{bfreg(c->dghT), 1, TBp, 2 * (long)c->dghT.stride};
        v_hsT = NtView{bfreg(c->hsT[l]), 1, TB1p, 2 * (long)c->hsT[l].stride};
        if (l > 0) {
          v_xT = NtView{bfreg(c->hsT[l - 1]) + B, 1, TB1p, 2 * (long)c->hsT[l - 1].stride};
        } else {
          if (!xT_ready)
            HIP_TRY(launch_cvt_bf16(layer_in, win, s_layer_in, bfreg(c->xT), TBp, 2 * (long)c->xT.stride, TB,
                                    win, true, groups, s));
          v_xT = NtView{bfreg(c->xT), 1, TBp, 2 * (long)c->xT.stride};
        }
        if (need_dx && wihT_ready[l]) {
          v_wihT = NtView{bfreg(c->wihTl[l]), 1, 3 * H, wstride(c->wihTl[l])};
        } else if (need_dx) {
          HIP_TRY(launch_cvt_bf16(Wih, win, sRi, bfreg(c->wihT), 3 * H, 2 * (long)c->wihT.stride, 3 * H, win, true,
                                  groups, s));
          v_wihT = NtView{bfreg(c->wihT), 1, 3 * H, 2 * (long)c->wihT.stride};
        }
      }
      role = HPSGD_ROLE_GEMM_DX;
      // bf16 operands: the input gradient reads only bf16 copies (not the weights the gradient
      // GEMMs below update in place) and has fewer tiles than the chip has CUs: with an auxiliary
      // stream it runs beside the layer's weight-gradient GEMMs (its launch is then not timed)
      bool dx_beside = false, swap = false;
      if (need_dx) {  // reads W_ih: before its update
        const NtView v_dgx = stepT ? NtView{dgxb, 1, 3 * H, s_dgb} : NtView{dgx, 0, 3 * H, s_gx};
        dx_beside = persist_b && stepT && v_wihT.bf16 && c->aux && c->ev_fork && c->ev_join && NC == 1;
        // Above the first layer the input gradient is the product with the long tiles (a contraction
        // over 3H, fewer tiles than CUs): it goes first, on this stream, and the first weight
        // gradient beside it on the auxiliary one, whose many short tiles fill in around it (issued
        // the other way round, the weight gradient's first wave of tiles held every CU and the
        // long tiles started a tile late).  The first layer's input gradient is short and has the
        // embedding gradient behind it: it stays on the auxiliary stream.
        swap = dx_beside && l > 0;
        if (swap) {
          if (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess)
            return HPSGD_EHIP;
          TRY(gemm2(s, groups, bf, TB, win, 3 * H, dgx, 3 * H, s_gx, 0, Wih, win, sRi, 0, dx, win, s_dx, EPI_STORE,
                    nullptr, 0, v_dgx, v_wihT, 0.f, persist_b));
        } else if (dx_beside) {
          if (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess)
            return HPSGD_EHIP;
          TRY0(gemm2(c->aux, groups, bf, TB, win, 3 * H, dgx, 3 * H, s_gx, 0, Wih, win, sRi, 0, dx, win, s_dx,
                     EPI_STORE, nullptr, 0, v_dgx, v_wihT, 0.f, persist_b));
          // the embedding rows need this product and nothing of the weight gradients beside it
          if (l == 0 && lm) {
            TRY0(embed_grad(c->aux));
            embed_done = true;
          }
          if (hipEventRecord(c->ev_join, c->aux) != hipSuccess) return HPSGD_EHIP;
        } else {
          TRY(gemm2(s, groups, bf, TB, win, 3 * H, dgx, 3 * H, s_gx, 0, Wih, win, sRi, 0, dx, win, s_dx, EPI_STORE,
                    nullptr, 0, v_dgx, v_wihT, 0.f, persist_b));
        }
        above = dx;
      }
      role = HPSGD_ROLE_GEMM_WGRAD;
      if (NC > 1) {
        // join, then the first chunk's share on top of what the aux stream accumulated
        if (hipEventRecord(c->ev_join, c->aux) != hipSuccess || hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess)
          return HPSGD_EHIP;
        TRY(wgrad_rows(s, 0, chunk_lo(1), EPI_ACCUM));
      } else {
        const WgradTarget wi = wgrad_target(c->lidx[l].wih);
        bool hh_first = false;
        // fp32, a narrow layer-0 input: the GEMM has few tiles and a long contraction (T*B), so the
        // contraction is cut into kWihSplits parts that run side by side; their sums are added
        // in order by the kernel that also applies the update
        const size_t n_wih = (size_t)3 * H * win;
        const bool split_wih = !bf && l == 0 && win <= 256 && win >= 4 && (3 * H) % 4 == 0 &&
                               TB % (4 * kWihSplits) == 0 &&
                               c->dwip.stride == (size_t)kWihSplits * n_wih && (n_wih & 3) == 0 &&
                               ((uintptr_t)dgx & 15) == 0 && ((uintptr_t)layer_in & 15) == 0 && (s_gx & 3) == 0 &&
                               (s_layer_in & 3) == 0 && (win & 3) == 0 && ((uintptr_t)wi.C & 15) == 0 &&
                               (wi.sC & 3) == 0 && (!wi.aux || (((uintptr_t)wi.aux & 15) == 0 && (sRi & 3) == 0));
        if (split_wih) {
          float* parts = reg(c->dwip);
          TRY(gemm(s, groups, 0, 3 * H, win, TB / kWihSplits, dgx, 3 * H, s_gx, 1, layer_in, win, s_layer_in, 0,
                   parts, win, (long)n_wih, EPI_STORE, nullptr, 0, 0, 0.f, kWihSplits));
          TRY0(queue_reduce(parts, kWihSplits, n_wih, wi.aux, (size_t)sRi, wi.C, (size_t)wi.sC, wi.epi == EPI_COMMIT));
        } else {
          // the first layer beside its input gradient: the recurrent weight gradient (the longer
          // tiles) before the input one, whose short tiles fill in at the end
          hh_first = dx_beside && !swap && !dwp;
          bool paired = false;
          if (hh_first) {
            const WgradTarget wh = wgrad_target(c->lidx[l].whh);
            // ... and both in one launch when both are updates in place: neither needs the other,
            // and on one stream the second would wait for the first one's last, partial round
            if (wh.epi == EPI_COMMIT && wi.epi == EPI_COMMIT && v_dghT.bf16 && v_hsT.bf16 && v_dgxT.bf16 && v_xT.bf16) {
              const GemmBf16Args ph{v_dghT.p, v_dghT.ld, v_dghT.stride, v_hsT.p, v_hsT.ld, v_hsT.stride, wh.C, H, wh.sC,
                                    wh.aux, sRi, lr, 3 * H, H, TB, groups};
              const GemmBf16Args pi{v_dgxT.p, v_dgxT.ld, v_dgxT.stride, v_xT.p, v_xT.ld, v_xT.stride, wi.C, win, wi.sC,
                                    wi.aux, sRi, lr, 3 * H, win, TB, groups};
              if (gemm_bf16_update_pair_supported(ph, pi)) {
                HIP_TRY(launch_gemm_bf16_update_pair(ph, pi, s));
                paired = true;
              }
            }
            if (!paired)
              TRY(gemm2(s, groups, bf, 3 * H, H, TB, dgh, 3 * H, s_gx, 1, hs, H, s_hs, 0, wh.C, H, wh.sC, wh.epi,
                        wh.aux, sRi, v_dghT, v_hsT, lr, persist_b));
          }
          if (paired) {
            // issued above
          } else if (swap) {
            // (both streams become runnable at the same event; a few microseconds' head start keeps the
            // long tiles in front also when this stream has marker packets - a timer's events - to
            // get through first)
            if (launch_delay(kAuxHeadStartUs, c->aux) != hipSuccess) return HPSGD_EHIP;
            TRY0(gemm2(c->aux, groups, bf, 3 * H, win, TB, dgx, 3 * H, s_gx, 1, layer_in, win, s_layer_in, 0, wi.C, win,
                       wi.sC, wi.epi, wi.aux, sRi, v_dgxT, v_xT, lr, persist_b));
            if (hipEventRecord(c->ev_join, c->aux) != hipSuccess) return HPSGD_EHIP;
          } else {
            TRY(gemm2(s, groups, bf, 3 * H, win, TB, dgx, 3 * H, s_gx, 1, layer_in, win, s_layer_in, 0, wi.C, win,
                      wi.sC, wi.epi, wi.aux, sRi, v_dgxT, v_xT, lr, persist_b));
          }
        }
        if (hh_first) {
          // issued above
        } else if (dwp) {
          const WgradTarget wh = wgrad_target(c->lidx[l].whh);
          TRY0(queue_reduce(dwp, (B + 31) / 32, (size_t)3 * H * H, wh.aux, (size_t)sRi, wh.C, (size_t)wh.sC,
                           wh.epi == EPI_COMMIT));
        } else {
          const WgradTarget wh = wgrad_target(c->lidx[l].whh);
          TRY(gemm2(s, groups, bf, 3 * H, H, TB, dgh, 3 * H, s_gx, 1, hs, H, s_hs, 0, wh.C, H, wh.sC, wh.epi,
                    wh.aux, sRi, v_dghT, v_hsT, lr, persist_b));
        }
      }
      role = HPSGD_ROLE_GEMM_WGRAD;
      if (dbp) {
        // the kernel that adds the partial sums applies the update too, when it can write the
        // replica with 16-byte accesses and the gradients are not accumulated as well
        const size_t ob_ih = c->eoff(c->lidx[l].bih);
        if (!acc && ((sR | sRi) & 3) == 0 && ((uintptr_t)(rin + ob_ih) & 15) == 0 && ((uintptr_t)(rout + ob_ih) & 15) == 0) {
          fused_commit[c->lidx[l].bih] = 1;
          fused_commit[c->lidx[l].bhh] = 1;
          TRY0(queue_reduce(dbp, (B + 31) / 32, (size_t)6 * H, rin + ob_ih, (size_t)sRi, rout + ob_ih, (size_t)sR, 1));
        } else {
          TRY0(queue_reduce(dbp, (B + 31) / 32, (size_t)6 * H, nullptr, 0, grad + ob_ih, (size_t)sG, 0));
        }
      } else {
        HIP_TRY(launch_colsum(dgx, 3 * H, s_gx, grad + c->eoff(c->lidx[l].bih), sG, TB, 3 * H, groups, s));
        HIP_TRY(launch_colsum(dgh, 3 * H, s_gx, grad + c->eoff(c->lidx[l].bhh), sG, TB, 3 * H, groups, s));
      }
      // the layer's sums of partial results (weight gradients of the resident-weight launch and
      // of the split contraction, bias gradients), with their updates: one launch
      HIP_TRY(launch_reduce_pack(rp, groups, s));
      if (dx_beside && hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess) return HPSGD_EHIP;
      role = HPSGD_ROLE_OTHER;
      d_zero = true;  // below the top layer nothing but `above` feeds a layer's gradient
    }
    if (lm && !embed_done) {
      role = HPSGD_ROLE_EMBED;
      TRY(embed_grad(s));
    }
  }
  // ---- commit (Alg. 2 "update replica")
  // the parameters not updated by a GEMM epilogue: one launch per contiguous run of them
  role = HPSGD_ROLE_COMMIT;
  c->last_commit_params = 0;
  for (size_t e = 0; e < c->entries.size();) {
    if (fused_commit[e]) {
      ++e;
      continue;
    }
    const size_t lo = c->entries[e].offset;
    while (e < c->entries.size() && !fused_commit[e]) ++e;
    const size_t hi = e < c->entries.size() ? c->entries[e].offset : c->P;
    if (acc)
      HIP_TRY(launch_commit_acc(rin + lo, (size_t)sRi, rout + lo, rstride, grad + lo, (size_t)sG, acc + lo, acc_stride, lr,
                                groups, hi - lo, s));
    else
      HIP_TRY(launch_commit(rin + lo, (size_t)sRi, rout + lo, rstride, grad + lo, (size_t)sG, lr, groups, hi - lo, s));
    c->last_commit_params += hi - lo;
  }
  if (abort_word) HIP_TRY(launch_poison_on_abort(abort_word, loss_out, groups, rout, sR, groups, s));
  return HPSGD_OK;
}

// ---- the workspace of hpsgd_local_step_all_static: a fixed array in device memory, one copy per
// device (every device that loads the library holds it until the process ends).  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address kernels and copies use is
// the one that call returns, looked up once per device with that device current.
static __device__ __align__(256) unsigned char g_static_workspace[HPSGD_STATIC_WORKSPACE_BYTES];
std::mutex g_static_mu;
void* g_static_workspace_ptr[kMaxDevices] = {nullptr};

int static_workspace(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HPSGD_EHIP;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_workspace_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_workspace)) != hipSuccess || !p) return HPSGD_EHIP;
    g_static_workspace_ptr[dev] = p;
  }
  *out = g_static_workspace_ptr[dev];
  return HPSGD_OK;
}

int check_step_args(const hpsgd_ctx* c, const float* rin, float* rout, size_t rstride, int groups,
                    const void* x, const int32_t* y, const void* ws) {
  if (!c || !rin || !rout || !x || !y) return HPSGD_EINVAL;
  if (!ws) return HPSGD_EWORKSPACE;
  if (((uintptr_t)ws & 255) != 0) return HPSGD_EWORKSPACE;
  if (!aligned16(rin) || !aligned16(rout) || ((uintptr_t)x & 3) != 0 || ((uintptr_t)y & 3) != 0)
    return HPSGD_EALIGN;
  if (groups > 1 && (rstride < c->P || (rstride & 3) != 0)) return HPSGD_EALIGN;
  const size_t span = ((size_t)(groups - 1) * rstride + c->P) * sizeof(float);
  if (rin != rout && overlaps(rin, span, rout, span)) return HPSGD_EALIAS;
  const size_t ws_bytes = c->ws_floats * sizeof(float);
  if (overlaps(ws, ws_bytes, rin, span) || overlaps(ws, ws_bytes, rout, span)) return HPSGD_EALIAS;
  return HPSGD_OK;
}

}  // namespace

namespace hpsgd {
static_assert((int)KID_COUNT == (int)HPSGD_KERNEL_COUNT, "kernel ids of kernels.h and hpsgd.h differ");

KernelTimer::KernelTimer(int kid, double work, hipStream_t s) : ctx_(nullptr), idx_(-1), s_(s) {
  hpsgd_ctx* c = t_step_ctx;
  if (!c || kid <= 0 || kid >= KID_COUNT || !(c->kernel_mask & (1u << kid))) return;
  hipEvent_t a = TimerScope::get(c), b = TimerScope::get(c);
  if (!a || !b) return;
  c->kstamps.push_back({kid, work, a, b});
  ctx_ = c;
  idx_ = (int)c->kstamps.size() - 1;
  (void)hipEventRecord(a, s);
}
KernelTimer::~KernelTimer() {
  if (!ctx_) return;
  hpsgd_ctx* c = static_cast<hpsgd_ctx*>(ctx_);
  (void)hipEventRecord(c->kstamps[idx_].b, s_);
}
}  // namespace hpsgd

extern "C" {

int hpsgd_create(const hpsgd_model_desc* desc, int K, hpsgd_ctx** out) {
  if (!desc || !out) return HPSGD_EINVAL;
  *out = nullptr;
  if (K < 1 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (desc->prec != HPSGD_FP32 && desc->prec != HPSGD_BF16_MFMA) return HPSGD_EINVAL;
  hpsgd_ctx* c = new (std::nothrow) hpsgd_ctx();
  if (!c) return HPSGD_EINVAL;
  c->d = *desc;
  c->K = K;
  const int rc = build_layout(c);
  if (rc != HPSGD_OK) {
    delete c;
    return rc;
  }
  *out = c;
  return HPSGD_OK;
}

int hpsgd_destroy(hpsgd_ctx* ctx) {
  if (ctx) {
    for (auto& st : ctx->stamps) {
      (void)hipEventDestroy(st.a);
      (void)hipEventDestroy(st.b);
    }
    for (auto& st : ctx->kstamps) {
      (void)hipEventDestroy(st.a);
      (void)hipEventDestroy(st.b);
    }
    for (auto e : ctx->free_events) (void)hipEventDestroy(e);
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  }
  delete ctx;
  return HPSGD_OK;
}

size_t hpsgd_param_count(const hpsgd_ctx* ctx) { return ctx ? ctx->P : 0; }
int hpsgd_param_entries(const hpsgd_ctx* ctx) { return ctx ? (int)ctx->entries.size() : 0; }

int hpsgd_param_entry(const hpsgd_ctx* ctx, int i, const char** name, size_t* offset, int* rows,
                      int* cols) {
  if (!ctx || i < 0 || i >= (int)ctx->entries.size()) return HPSGD_EINVAL;
  const Entry& e = ctx->entries[i];
  if (name) *name = e.name.c_str();
  if (offset) *offset = e.offset;
  if (rows) *rows = e.rows;
  if (cols) *cols = e.cols;
  return HPSGD_OK;
}

size_t hpsgd_workspace_bytes(const hpsgd_ctx* ctx) { return ctx ? ctx->ws_floats * sizeof(float) : 0; }

int hpsgd_local_step_all(hpsgd_ctx* ctx, const float* replicas_in, float* replicas_out,
                         size_t replica_stride, const void* x, const int32_t* y, float lr,
                         float* loss_out, void* workspace, void* hip_stream) {
  if (!ctx) return HPSGD_EINVAL;
  TRY0(check_step_args(ctx, replicas_in, replicas_out, replica_stride, ctx->K, x, y, workspace));
  return run_step(ctx, 0, ctx->K, replicas_in, replicas_out, replica_stride, x, y, lr, loss_out,
                  (float*)workspace, (hipStream_t)hip_stream);
}

int hpsgd_local_step_all_cloned(hpsgd_ctx* ctx, const float* source, float* replicas_out, size_t replica_stride,
                                const void* x, const int32_t* y, float lr, float* loss_out, void* workspace,
                                void* hip_stream) {
  if (!ctx) return HPSGD_EINVAL;
  // the output replicas alone are checked like those of a step in place, the source like a model
  TRY0(check_step_args(ctx, replicas_out, replicas_out, replica_stride, ctx->K, x, y, workspace));
  if (!source) return HPSGD_EINVAL;
  if (!aligned16(source)) return HPSGD_EALIGN;
  const size_t span = ((size_t)(ctx->K - 1) * replica_stride + ctx->P) * sizeof(float);
  const size_t pbytes = ctx->P * sizeof(float);
  if (overlaps(source, pbytes, replicas_out, span) ||
      overlaps(source, pbytes, workspace, ctx->ws_floats * sizeof(float)))
    return HPSGD_EALIAS;
  return run_step(ctx, 0, ctx->K, source, replicas_out, replica_stride, x, y, lr, loss_out, (float*)workspace,
                  (hipStream_t)hip_stream, nullptr, 0, true);
}

int hpsgd_local_step_all_static(hpsgd_ctx* ctx, const float* replicas_in, float* replicas_out,
                                size_t replica_stride, const void* x, const int32_t* y, float lr,
                                float* loss_out, void* hip_stream) {
  if (!ctx) return HPSGD_EINVAL;
  // the size check comes first and needs no device
  if (ctx->ws_floats * sizeof(float) > (size_t)HPSGD_STATIC_WORKSPACE_BYTES) return HPSGD_EWORKSPACE;
  if (!replicas_in || !replicas_out || !x || !y) return HPSGD_EINVAL;
  void* ws = nullptr;
  TRY0(static_workspace(&ws));
  TRY0(check_step_args(ctx, replicas_in, replicas_out, replica_stride, ctx->K, x, y, ws));
  return run_step(ctx, 0, ctx->K, replicas_in, replicas_out, replica_stride, x, y, lr, loss_out, (float*)ws,
                  (hipStream_t)hip_stream);
}

int hpsgd_prepare_replicas(hpsgd_ctx* ctx, const float* replicas, size_t replica_stride, void* workspace,
                           void* hip_stream) {
  if (!ctx || !replicas) return HPSGD_EINVAL;
  if (!workspace || ((uintptr_t)workspace & 255) != 0) return HPSGD_EWORKSPACE;
  if (!aligned16(replicas) || (ctx->K > 1 && (replica_stride < ctx->P || (replica_stride & 3) != 0)))
    return HPSGD_EALIGN;
  const size_t span = ((size_t)(ctx->K - 1) * replica_stride + ctx->P) * sizeof(float);
  if (overlaps(workspace, ctx->ws_floats * sizeof(float), replicas, span)) return HPSGD_EALIAS;
  ctx->drop_mark((const float*)workspace);
  if (ctx->d.prec != HPSGD_BF16_MFMA || ctx->d.kind == HPSGD_MLP) return HPSGD_OK;  // nothing to prepare
  WeightCopies wc;
  const int rc = weight_copies(ctx, replicas, (long)replica_stride, 0, ctx->K, (float*)workspace,
                               (hipStream_t)hip_stream, true, true, wc);
  if (rc != HPSGD_OK) return rc;
  ctx->set_mark(hpsgd_ctx::Mark{replicas, (const float*)workspace, replica_stride, nullptr, false});
  return HPSGD_OK;
}

int hpsgd_prepare_clones(hpsgd_ctx* ctx, const float* global, const float* replicas, size_t replica_stride,
                         void* workspace, int with_head, void* hip_stream) {
  if (!ctx || !global || !replicas) return HPSGD_EINVAL;
  if (!workspace || ((uintptr_t)workspace & 255) != 0) return HPSGD_EWORKSPACE;
  if (!aligned16(global) || !aligned16(replicas) ||
      (ctx->K > 1 && (replica_stride < ctx->P || (replica_stride & 3) != 0)))
    return HPSGD_EALIGN;
  const size_t span = ((size_t)(ctx->K - 1) * replica_stride + ctx->P) * sizeof(float);
  const size_t ws_bytes = ctx->ws_floats * sizeof(float);
  if (overlaps(workspace, ws_bytes, replicas, span) || overlaps(workspace, ws_bytes, global, ctx->P * sizeof(float)))
    return HPSGD_EALIAS;
  ctx->drop_mark((const float*)workspace);
  if (ctx->d.prec != HPSGD_BF16_MFMA || ctx->d.kind == HPSGD_MLP) return HPSGD_OK;  // nothing to prepare
  WeightCopies wc;
  // one set of copies, in worker 0's slice, which the step hands to every worker (the replicas are
  // clones: their copies would be the same bits).  The GRU layers' always; the head's when asked
  // for, else they are left to the step, which makes them from `global` right before the logits
  // GEMM (a training stream that makes them here, at a round's start, would share the memory
  // system with whatever the synchronising side is doing then)
  // (the step decides from the replicas' addresses which copies it has; made from another address
  // the set must come out the same, else the step makes its own)
  const bool head = with_head != 0;
  WeightCopies want;
  int rc = weight_copies(ctx, replicas, (long)replica_stride, 0, ctx->K, (float*)workspace, nullptr, false, head, want);
  if (rc == HPSGD_OK) rc = weight_copies(ctx, global, 0, 0, 1, (float*)workspace, nullptr, false, head, wc);
  if (rc != HPSGD_OK) return rc;
  if (std::memcmp(&want, &wc, sizeof(WeightCopies)) != 0) return HPSGD_OK;
  rc = weight_copies(ctx, global, 0, 0, 1, (float*)workspace, (hipStream_t)hip_stream, true, head, wc);
  if (rc != HPSGD_OK) return rc;
  ctx->set_mark(hpsgd_ctx::Mark{replicas, (const float*)workspace, replica_stride, global, head && wc.head});
  return HPSGD_OK;
}

int hpsgd_local_step_all_acc(hpsgd_ctx* ctx, const float* replicas_in, float* replicas_out,
                             size_t replica_stride, const void* x, const int32_t* y, float lr,
                             float* loss_out, float* grad_acc, size_t acc_stride, void* workspace,
                             void* hip_stream) {
  if (!ctx) return HPSGD_EINVAL;
  TRY0(check_step_args(ctx, replicas_in, replicas_out, replica_stride, ctx->K, x, y, workspace));
  if (!grad_acc) return HPSGD_EINVAL;
  if (((uintptr_t)grad_acc & 15) != 0 || (ctx->K > 1 && (acc_stride < ctx->P || (acc_stride & 3) != 0)))
    return HPSGD_EALIGN;
  const size_t span = ((size_t)(ctx->K - 1) * acc_stride + ctx->P) * sizeof(float);
  const size_t rspan = ((size_t)(ctx->K - 1) * replica_stride + ctx->P) * sizeof(float);
  if (overlaps(grad_acc, span, replicas_in, rspan) || overlaps(grad_acc, span, replicas_out, rspan))
    return HPSGD_EALIAS;
  return run_step(ctx, 0, ctx->K, replicas_in, replicas_out, replica_stride, x, y, lr, loss_out,
                  (float*)workspace, (hipStream_t)hip_stream, grad_acc, acc_stride);
}

int hpsgd_local_step(hpsgd_ctx* ctx, int worker, const float* replica_in, float* replica_out,
                     const void* x, const int32_t* y, float lr, float* loss_out, void* workspace,
                     void* hip_stream) {
  if (!ctx || worker < 0 || worker >= ctx->K) return HPSGD_EINVAL;
  TRY0(check_step_args(ctx, replica_in, replica_out, ctx->P, 1, x, y, workspace));
  return run_step(ctx, worker, 1, replica_in, replica_out, round_up(ctx->P, 4), x, y, lr, loss_out,
                  (float*)workspace, (hipStream_t)hip_stream);
}

int hpsgd_gather_batch(const void* shard, const int32_t* idx, int n_idx, size_t row_bytes,
                       int n_chunks, size_t chunk_bytes, void* out, void* hip_stream) {
  if (n_idx < 0 || n_chunks < 0) return HPSGD_EINVAL;
  if (n_idx == 0 || n_chunks == 0 || chunk_bytes == 0) return HPSGD_OK;
  if (!shard || !idx || !out) return HPSGD_EINVAL;
  if ((row_bytes & 3) || (chunk_bytes & 3) || ((uintptr_t)shard & 3) || ((uintptr_t)out & 3) ||
      ((uintptr_t)idx & 3))
    return HPSGD_EALIGN;
  if ((size_t)n_chunks * chunk_bytes > row_bytes || n_chunks > 65535) return HPSGD_ESHAPE;
  return launch_gather(shard, idx, n_idx, row_bytes, n_chunks, chunk_bytes, out,
                       (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK : HPSGD_EHIP;
}

int hpsgd_gather_batch_all(const void* const* shards, const int32_t* const* idx, int K, int n_idx,
                           size_t row_bytes, int n_chunks, size_t chunk_bytes, void* const* outs,
                           void* hip_stream) {
  if (K < 0 || K > HPSGD_MAX_WORKERS || n_idx < 0 || n_chunks < 0) return HPSGD_EINVAL;
  if (K == 0 || n_idx == 0 || n_chunks == 0 || chunk_bytes == 0) return HPSGD_OK;
  if (!shards || !idx || !outs) return HPSGD_EINVAL;
  if ((row_bytes & 3) || (chunk_bytes & 3)) return HPSGD_EALIGN;
  if ((size_t)n_chunks * chunk_bytes > row_bytes || n_chunks > 65535) return HPSGD_ESHAPE;
  for (int k = 0; k < K; ++k) {
    if (!shards[k] || !idx[k] || !outs[k]) return HPSGD_EINVAL;
    if (((uintptr_t)shards[k] & 3) || ((uintptr_t)outs[k] & 3) || ((uintptr_t)idx[k] & 3)) return HPSGD_EALIGN;
  }
  return launch_gather_all(shards, idx, K, n_idx, row_bytes, n_chunks, chunk_bytes, outs,
                           (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK : HPSGD_EHIP;
}

int hpsgd_merge(float* global, const float* const* replicas, const float* snapshot, int K, size_t P,
                void* hip_stream) {
  if (K < 1 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (P == 0) return HPSGD_OK;
  if (!global || !replicas || !snapshot) return HPSGD_EINVAL;
  if (!aligned16(global) || !aligned16(snapshot)) return HPSGD_EALIGN;
  PtrPack pk;
  for (int k = 0; k < K; ++k) {
    if (!replicas[k]) return HPSGD_EINVAL;
    if (!aligned16(replicas[k])) return HPSGD_EALIGN;
    if (overlaps(global, P * sizeof(float), replicas[k], P * sizeof(float))) return HPSGD_EALIAS;
    pk.p[k] = const_cast<float*>(replicas[k]);
  }
  if (snapshot != global && overlaps(global, P * sizeof(float), snapshot, P * sizeof(float)))
    return HPSGD_EALIAS;
  return launch_merge(global, pk, snapshot, K, P, (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK
                                                                                          : HPSGD_EHIP;
}

int hpsgd_merge_sync(float* global, float* const* replicas, float* snapshot, int K, size_t P, void* hip_stream) {
  if (K < 1 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (P == 0) return HPSGD_OK;
  if (!global || !replicas || !snapshot) return HPSGD_EINVAL;
  if (!aligned16(global) || !aligned16(snapshot)) return HPSGD_EALIGN;
  const size_t bytes = P * sizeof(float);
  PtrPack pk;
  for (int k = 0; k < K; ++k) {
    if (!replicas[k]) return HPSGD_EINVAL;
    if (!aligned16(replicas[k])) return HPSGD_EALIGN;
    // every buffer is written here: no two may overlap
    if (overlaps(global, bytes, replicas[k], bytes) || overlaps(snapshot, bytes, replicas[k], bytes)) return HPSGD_EALIAS;
    for (int j = 0; j < k; ++j)
      if (overlaps(replicas[j], bytes, replicas[k], bytes)) return HPSGD_EALIAS;
    pk.p[k] = replicas[k];
  }
  if (overlaps(global, bytes, snapshot, bytes)) return HPSGD_EALIAS;
  return launch_merge_sync(global, pk, snapshot, K, P, (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK : HPSGD_EHIP;
}

int hpsgd_merge_snapshot(float* global, const float* const* replicas, float* snapshot, int K, size_t P,
                         void* hip_stream) {
  if (K < 1 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (P == 0) return HPSGD_OK;
  if (!global || !replicas || !snapshot) return HPSGD_EINVAL;
  if (!aligned16(global) || !aligned16(snapshot)) return HPSGD_EALIGN;
  const size_t bytes = P * sizeof(float);
  PtrPack pk;
  for (int k = 0; k < K; ++k) {
    if (!replicas[k]) return HPSGD_EINVAL;
    if (!aligned16(replicas[k])) return HPSGD_EALIGN;
    // the replicas are read while the two models are written
    if (overlaps(global, bytes, replicas[k], bytes) || overlaps(snapshot, bytes, replicas[k], bytes)) return HPSGD_EALIAS;
    pk.p[k] = const_cast<float*>(replicas[k]);
  }
  if (overlaps(global, bytes, snapshot, bytes)) return HPSGD_EALIAS;
  return launch_merge_sync(global, pk, snapshot, K, P, (hipStream_t)hip_stream, false) == hipSuccess ? HPSGD_OK
                                                                                                      : HPSGD_EHIP;
}

int hpsgd_merge_grad(float* global, const float* const* grad_accs, float lr, int K, size_t P,
                     void* hip_stream) {
  if (K < 1 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (P == 0) return HPSGD_OK;
  if (!global || !grad_accs) return HPSGD_EINVAL;
  if (!aligned16(global)) return HPSGD_EALIGN;
  PtrPack pk;
  for (int k = 0; k < K; ++k) {
    if (!grad_accs[k]) return HPSGD_EINVAL;
    if (!aligned16(grad_accs[k])) return HPSGD_EALIGN;
    if (overlaps(global, P * sizeof(float), grad_accs[k], P * sizeof(float))) return HPSGD_EALIAS;
    pk.p[k] = const_cast<float*>(grad_accs[k]);
  }
  return launch_merge_grad(global, pk, lr, K, P, (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK
                                                                                        : HPSGD_EHIP;
}

int hpsgd_sync_all(const float* global, float* const* replicas, int K, float* snapshot, size_t P,
                   void* hip_stream) {
  if (K < 0 || K > HPSGD_MAX_WORKERS) return HPSGD_EINVAL;
  if (P == 0) return HPSGD_OK;
  if (!global || (K > 0 && !replicas)) return HPSGD_EINVAL;
  if (!aligned16(global) || (snapshot && !aligned16(snapshot))) return HPSGD_EALIGN;
  PtrPack pk;
  for (int k = 0; k < K; ++k) {
    if (!replicas[k]) return HPSGD_EINVAL;
    if (!aligned16(replicas[k])) return HPSGD_EALIGN;
    if (overlaps(global, P * sizeof(float), replicas[k], P * sizeof(float))) return HPSGD_EALIAS;
    pk.p[k] = replicas[k];
  }
  if (snapshot && overlaps(global, P * sizeof(float), snapshot, P * sizeof(float))) return HPSGD_EALIAS;
  if (K == 0 && !snapshot) return HPSGD_OK;
  return launch_sync_all(global, pk, K, snapshot, P, (hipStream_t)hip_stream) == hipSuccess
             ? HPSGD_OK
             : HPSGD_EHIP;
}

int hpsgd_sync_replica(const float* global, float* replica, size_t P, void* hip_stream) {
  float* one[1] = {replica};
  if (!replica) return P == 0 ? HPSGD_OK : HPSGD_EINVAL;
  return hpsgd_sync_all(global, one, 1, nullptr, P, hip_stream);
}

int hpsgd_set_aux_stream(hpsgd_ctx* ctx, void* hip_stream) {
  if (!ctx) return HPSGD_EINVAL;
  if (hip_stream && !ctx->ev_fork) {
    if (hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming) != hipSuccess)
      return HPSGD_EHIP;
  }
  ctx->aux = (hipStream_t)hip_stream;
  return HPSGD_OK;
}

int hpsgd_set_recurrence(hpsgd_ctx* ctx, int resident, unsigned spin_limit) {
  if (!ctx) return HPSGD_EINVAL;
  ctx->resident = resident != 0;
  ctx->device_scope = resident == 2;
  ctx->spin_limit = spin_limit;
  return HPSGD_OK;
}

int hpsgd_recurrence_gave_up(const hpsgd_ctx* ctx, const void* workspace, void* hip_stream, int* gave_up) {
  if (!ctx || !gave_up) return HPSGD_EINVAL;
  if (!workspace) return HPSGD_EWORKSPACE;
  *gave_up = 0;
  if (ctx->psync.stride == 0) return HPSGD_OK;  // no such kernels for this model
  // the abort word is the first word of a worker's slice (of the first worker's for a grouped step)
  std::vector<unsigned> host(ctx->psync.stride * (size_t)ctx->K);
  hipStream_t s = (hipStream_t)hip_stream;
  if (hipMemcpyAsync(host.data(), (const float*)workspace + ctx->psync.offset, host.size() * sizeof(unsigned),
                     hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return HPSGD_EHIP;
  for (int k = 0; k < ctx->K; ++k)
    if (host[(size_t)k * ctx->psync.stride] == 1u) *gave_up = 1;
  return HPSGD_OK;
}

int hpsgd_timer_enable(hpsgd_ctx* ctx, unsigned role_mask) {
  if (!ctx) return HPSGD_EINVAL;
  ctx->timer_mask = role_mask & ((1u << HPSGD_ROLE_COUNT) - 1u);
  return HPSGD_OK;
}

int hpsgd_timer_read(hpsgd_ctx* ctx, int role, long* launches, double* total_ms) {
  if (!ctx || role < 0 || role >= HPSGD_ROLE_COUNT) return HPSGD_EINVAL;
  // fold every recorded pair into the per-role totals, then hand back and clear this role's
  for (auto& st : ctx->stamps) {
    if (hipEventSynchronize(st.b) != hipSuccess) return HPSGD_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, st.a, st.b) != hipSuccess) return HPSGD_EHIP;
    ctx->role_ms[st.role] += ms;
    ctx->role_launches[st.role] += st.launches;
    ctx->free_events.push_back(st.a);
    ctx->free_events.push_back(st.b);
  }
  ctx->stamps.clear();
  if (launches) *launches = ctx->role_launches[role];
  if (total_ms) *total_ms = ctx->role_ms[role];
  ctx->role_launches[role] = 0;
  ctx->role_ms[role] = 0.0;
  return HPSGD_OK;
}

int hpsgd_kernel_timer_enable(hpsgd_ctx* ctx, unsigned kernel_mask) {
  if (!ctx) return HPSGD_EINVAL;
  ctx->kernel_mask = kernel_mask & ((1u << HPSGD_KERNEL_COUNT) - 1u) & ~1u;
  return HPSGD_OK;
}

int hpsgd_kernel_timer_read(hpsgd_ctx* ctx, int kernel, long* launches, double* total_ms, double* work) {
  if (!ctx || kernel <= 0 || kernel >= HPSGD_KERNEL_COUNT) return HPSGD_EINVAL;
  for (auto& st : ctx->kstamps) {
    if (hipEventSynchronize(st.b) != hipSuccess) return HPSGD_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, st.a, st.b) != hipSuccess) return HPSGD_EHIP;
    ctx->kernel_ms[st.kid] += ms;
    ctx->kernel_work[st.kid] += st.work;
    ctx->kernel_launches[st.kid] += 1;
    ctx->free_events.push_back(st.a);
    ctx->free_events.push_back(st.b);
  }
  ctx->kstamps.clear();
  if (launches) *launches = ctx->kernel_launches[kernel];
  if (total_ms) *total_ms = ctx->kernel_ms[kernel];
  if (work) *work = ctx->kernel_work[kernel];
  ctx->kernel_launches[kernel] = 0;
  ctx->kernel_ms[kernel] = 0.0;
  ctx->kernel_work[kernel] = 0.0;
  return HPSGD_OK;
}

const char* hpsgd_kernel_name(int kernel) {
  switch (kernel) {
    case HPSGD_KERNEL_GRU_FWD_PERSIST: return "gru_fwd_persist_kernel";
    case HPSGD_KERNEL_GRU_BWD_PERSIST: return "gru_bwd_persist_kernel";
    case HPSGD_KERNEL_GRU_FWD_PERSIST_BF16: return "gru_fwd_persist_bf16_kernel";
    case HPSGD_KERNEL_GRU_BWD_PERSIST_BF16: return "gru_bwd_persist_bf16_kernel";
    case HPSGD_KERNEL_GEMM_BF16_DL: return "gemm_bf16_dl_kernel<false>";
    case HPSGD_KERNEL_GEMM_BF16_DL_COMMIT: return "gemm_bf16_dl_kernel<true>";
    case HPSGD_KERNEL_GEMM_BF16_DLX128: return "gemm_bf16_dlx_kernel<false, 2, 4, 2, 2, 3>";
    case HPSGD_KERNEL_GEMM_BF16_DLX128_COMMIT: return "gemm_bf16_dlx_kernel<true, 2, 4, 2, 2, 3>";
    case HPSGD_KERNEL_GEMM_BF16_DLX192: return "gemm_bf16_dlx_kernel<false, 2, 4, 3, 2, 2>";
    case HPSGD_KERNEL_GEMM_BF16_DLX192_COMMIT: return "gemm_bf16_dlx_kernel<true, 2, 4, 3, 2, 2>";
    case HPSGD_KERNEL_GEMM_BF16_DLX256: return "gemm_bf16_dlx_kernel<false, 2, 4, 4, 2, 2>";
    case HPSGD_KERNEL_GEMM_BF16_DLX256_COMMIT: return "gemm_bf16_dlx_kernel<true, 2, 4, 4, 2, 2>";
    case HPSGD_KERNEL_GEMM_BF16_NT: return "gemm_bf16_nt_kernel";
    case HPSGD_KERNEL_GEMM_F32_FAST: return "gemm_f32_fast_kernel";
    case HPSGD_KERNEL_GEMM_F32: return "gemm_f32_kernel";
    case HPSGD_KERNEL_CVT2: return "cvt2_kernel";
    case HPSGD_KERNEL_SOFTMAX_CE_BF16: return "softmax_ce_bf16_rows_kernel";
    case HPSGD_KERNEL_GRU_STEP: return "gru_step_kernel";
    case HPSGD_KERNEL_COMMIT_ACC: return "commit_acc4_kernel";
    case HPSGD_KERNEL_COMMIT: return "commit_kernel";
    case HPSGD_KERNEL_CVT2_PACK: return "cvt2_pack_kernel";
    default: return nullptr;
  }
}

int hpsgd_delay_us(unsigned microseconds, void* hip_stream) {
  if (microseconds > 1000000u) return HPSGD_EINVAL;
  return launch_delay(microseconds, (hipStream_t)hip_stream) == hipSuccess ? HPSGD_OK : HPSGD_EHIP;
}

size_t hpsgd_commit_kernel_params(const hpsgd_ctx* ctx) { return ctx ? ctx->last_commit_params : 0; }

int hpsgd_recurrence_info(const hpsgd_ctx* ctx, int* resident_layers, int* xproj_layers, int* dw_layers) {
  if (!ctx) return HPSGD_EINVAL;
  if (resident_layers) *resident_layers = ctx->last_resident;
  if (xproj_layers) *xproj_layers = ctx->last_xproj;
  if (dw_layers) *dw_layers = ctx->last_dw;
  return HPSGD_OK;
}

int hpsgd_gemm_bf16_nt(const void* A, long lda, long strideA, const void* B, long ldb, long strideB, float* C,
                       long ldc, long strideC, const float* win, long strideWin, float lr, int M, int N, int Kd,
                       int groups, int form, void* hip_stream) {
  if (!A || !B || !C || M < 1 || N < 1 || Kd < 8 || Kd % 8 != 0 || groups < 1 || form < 0 || form > 4)
    return HPSGD_EINVAL;
  if (lda < Kd || ldb < Kd || ldc < N) return HPSGD_EINVAL;
  if (!gemm_bf16_nt_supported(A, 1, lda, strideA, Kd) || !gemm_bf16_nt_supported(B, 1, ldb, strideB, Kd))
    return HPSGD_EALIGN;
  return launch_gemm_bf16_nt(A, 1, lda, strideA, B, 1, ldb, strideB, C, ldc, strideC, nullptr, 0, win, strideWin, lr,
                             M, N, Kd, groups, (hipStream_t)hip_stream, form) == hipSuccess
             ? HPSGD_OK
             : HPSGD_EHIP;
}

int hpsgd_probe_mfma_rate(int precision, const void* operands, int iterations, double* result, float* sink,
                          void* hip_stream) {
  if (!operands || !result || !sink || iterations < 1) return HPSGD_EINVAL;
  if (precision != HPSGD_FP32 && precision != HPSGD_BF16_MFMA) return HPSGD_EINVAL;
  if (((uintptr_t)operands & 15) != 0) return HPSGD_EALIGN;
  return launch_mfma_probe(precision == HPSGD_BF16_MFMA, operands, iterations, result, sink,
                           (hipStream_t)hip_stream) == hipSuccess
             ? HPSGD_OK
             : HPSGD_EHIP;
}

const char* hpsgd_role_name(int role) {
  switch (role) {
    case HPSGD_ROLE_OTHER: return "other";
    case HPSGD_ROLE_GEMM_INPUT: return "gemm_input_projection";
    case HPSGD_ROLE_GEMM_REC_FWD: return "gemm_recurrent_fwd";
    case HPSGD_ROLE_GEMM_REC_BWD: return "gemm_recurrent_bwd";
    case HPSGD_ROLE_GEMM_WGRAD: return "gemm_weight_grad";
    case HPSGD_ROLE_GEMM_DX: return "gemm_input_grad";
    case HPSGD_ROLE_GEMM_HEAD: return "gemm_head";
    case HPSGD_ROLE_CELL_FWD: return "gru_cell_fwd";
    case HPSGD_ROLE_CELL_BWD: return "gru_cell_bwd";
    case HPSGD_ROLE_LOSS: return "softmax_ce";
    case HPSGD_ROLE_EMBED: return "embedding";
    case HPSGD_ROLE_COMMIT: return "commit";
    case HPSGD_ROLE_MLP_FWD: return "mlp_fwd";
    case HPSGD_ROLE_MLP_BWD: return "mlp_bwd";
    default: return nullptr;
  }
}

const char* hpsgd_strerror(int status) {
  switch (status) {
    case HPSGD_OK: return "ok";
    case HPSGD_EINVAL: return "invalid argument";
    case HPSGD_ESHAPE: return "unsupported or inconsistent shape";
    case HPSGD_EALIGN: return "pointer or stride not aligned";
    case HPSGD_EALIAS: return "buffers overlap";
    case HPSGD_EWORKSPACE: return "workspace null or misaligned";
    case HPSGD_EUNSUPPORTED: return "not supported";
    case HPSGD_EHIP: return "HIP call failed";
    default: return "unknown status";
  }
}

}  // extern "C"
