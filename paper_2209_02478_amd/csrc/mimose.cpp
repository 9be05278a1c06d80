// libmimose: context, budget-enforcing activation stack, step executor and the C ABI.
//
// Device memory is one caller-provided arena.  The bottom holds parameters and fp32
// gradients (the fixed bytes F); above it a LIFO stack holds the step's activations.
// Every layer allocates its output first and its internal tensors above it, so dropping a
// layer (paper Section 5: checkpointing keeps only the boundary tensor) is a pop to just
// above the output, and rebuilding it in backward pushes the same tensors again and replays
// the same kernel launches.  The stack's high-water mark is the step's true peak.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cmath>
#include <cstring>
#include <memory>
#include <string>
#include <utility>
#include <vector>

#include "../../include/mimose.h"
#include "kernels.h"
#include "planner.h"

namespace {

struct OomError { uint64_t want, top, cap; };
struct StepError { int code; std::string msg; };

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

class Arena {
 public:
  void init(char* base, uint64_t cap) { base_ = base; cap_ = cap; top_ = high_ = section_high_ = 0; }
  void* alloc(uint64_t bytes) {
    const uint64_t sz = align_up(bytes);
    if (top_ + sz > cap_) throw OomError{sz, top_, cap_};
    void* p = base_ ? base_ + top_ : nullptr;
    top_ += sz;
    high_ = std::max(high_, top_);
    section_high_ = std::max(section_high_, top_);
    return p;
  }
  uint64_t top() const { return top_; }
  uint64_t high() const { return high_; }
  void pop_to(uint64_t mark) { top_ = mark; }
  void reset_high() { high_ = top_; }
  void begin_section() { section_high_ = top_; }
  uint64_t section_high() const { return section_high_; }
  uint64_t cap() const { return cap_; }
 private:
  char* base_ = nullptr;
  uint64_t cap_ = 0, top_ = 0, high_ = 0, section_high_ = 0;
};

struct Param {
  std::string name;
  int64_t shape[4] = {0, 0, 0, 0};
  int ndim = 0;
  int64_t n = 0;
  void* w = nullptr;    // storage dtype
  float* g = nullptr;   // fp32 gradient
  // optimizer state (after mimose_optimizer_init): moments, and an fp32 master copy when the
  // storage type is narrower than fp32 (for fp32 storage the parameter itself is the master)
  float* m = nullptr;
  float* v = nullptr;
  float* master = nullptr;
};

struct LayerIdx { int wqkv, bqkv, wo, bo, ln1g, ln1b, w1, b1, w2, b2, ln2g, ln2b; };

struct LayerActs {       // device tensors of one layer, in allocation order
  bool has_out = false;  // the boundary tensor is allocated (survives a drop)
  uint64_t mark = 0;     // stack top before the layer
  uint64_t after_out = 0;
  bool dropped = false;
  const void* x = nullptr;                       // layer input (previous boundary)
  void *out = nullptr, *n1 = nullptr, *qkv = nullptr, *ctx = nullptr, *s1 = nullptr, *u = nullptr,
       *pre = nullptr, *act = nullptr, *s2 = nullptr;
  float* lse = nullptr;
};

}  // namespace

struct mimose_ctx {
  mimose_model_cfg cfg;
  uint64_t budget = 0;
  bool has_device = false;
  hipStream_t stream = nullptr;
  // weight-gradient products run on a second stream, beside the data-gradient chain that
  // needs the same incoming gradient (fork / join with events; default priority)
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  // the last weight-gradient product of a layer is waited for one layer later: ev_early marks
  // the side stream just before it, ev_late just after it
  hipEvent_t ev_early = nullptr, ev_late = nullptr;
  // end of a layer's first weight-gradient product, which reads the incoming gradient where the
  // layer's last data-gradient product writes when the carriers have the storage type
  hipEvent_t ev_w2 = nullptr;
  std::vector<hipEvent_t> ev_layer;   // begin / end of each layer's forward in a collecting step
  Arena arena;
  uint64_t fixed_top = 0;
  std::vector<Param> params;
  std::vector<LayerIdx> lidx;
  int i_tok = -1, i_pos = -1, i_eg = -1, i_eb = -1, i_fg = -1, i_fb = -1, i_wt = -1, i_bt = -1, i_hg = -1,
      i_hb = -1, i_bdec = -1;
  std::unique_ptr<mimose::Planner> planner;
  int64_t forced_plan = -1;
  int plan_mode = MIMOSE_PLAN_INPUT_AWARE;
  int collector = MIMOSE_COLLECTOR_MARKS;
  // dropout: probability of the hidden sites, seed, number of the next iteration
  float p_hidden = 0.f, p_attn = 0.f;
  uint64_t drop_seed = 0, drop_step = 0;
  // parameter update (Section 2.1: the iteration ends with it; its state is part of the
  // input-independent memory of Section 3.1)
  bool opt_on = false;
  mimose_adamw_cfg opt;
  uint64_t opt_t = 0;
  mk::AdamTensor* opt_tensors = nullptr;   // device tables
  mk::AdamChunk* opt_chunks = nullptr;
  int opt_n_chunks = 0;
  mimose_stats stats;
  std::string err;
  // pinned host staging for ids / labels / sort order / segments and the loss
  // (two of them, taken in turn: a step that returns before the device has finished leaves copies
  // out of its buffer pending, marked by that buffer's event)
  int32_t* stage_buf[2] = {nullptr, nullptr};
  size_t stage_buf_ints[2] = {0, 0};
  hipEvent_t ev_stage[2] = {nullptr, nullptr};
  bool stage_busy[2] = {false, false};
  int stage_turn = 0;
  int32_t* stage = nullptr;              // the buffer of the step being issued
  float* loss_host = nullptr;
  bool loss_pending = false;             // a step was issued whose loss has not been waited for
  bool dry = false;
  std::vector<LayerActs> acts;
  std::vector<int32_t> sort_count;       // reused scratch of the per-step counting sort
  // memory components measured in the last completed step
  uint64_t last_e = 0, last_g = 0;
  std::vector<uint64_t> last_a, last_b, last_w, last_t;
  // optional per-kernel-class timing with events on the work stream
  bool prof_on = false;
  struct ProfPending { int cls; double work; hipEvent_t a, b; };
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  std::vector<ProfPending> prof_pending;
  struct ProfClass { uint64_t launches = 0; double ms = 0, work = 0; } prof[MIMOSE_K_COUNT];
  hipEvent_t prof_event() {
    if (ev_used == ev_pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      ev_pool.push_back(e);
    }
    return ev_pool[ev_used++];
  }

  int elt() const { return cfg.dtype == mk::BF16 ? 2 : 4; }
  int64_t ldv() const { return (cfg.vocab + 63) / 64 * 64; }
};

static thread_local std::string g_init_error;

// the message mimose_last_error(NULL) returns on this thread, for entry points without a context
void mimose_set_thread_error(const char* msg) { g_init_error = msg ? msg : ""; }

namespace {

int fail(mimose_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_init_error = msg;
  return code;
}

#define HIPCHK(c, call)                                                                     \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess) throw StepError{MIMOSE_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)}; \
  } while (0)

int add_param(mimose_ctx* c, const std::string& name, std::initializer_list<int64_t> shape) {
  Param p;
  p.name = name;
  p.n = 1;
  for (int64_t s : shape) { p.shape[p.ndim++] = s; p.n *= s; }
  c->params.push_back(p);
  return (int)c->params.size() - 1;
}

// width of layer l's feed-forward block
inline int ffn_of(const mimose_model_cfg& f, int l) { return f.ffn_by_layer[l] > 0 ? f.ffn_by_layer[l] : f.ffn; }

void build_params(mimose_ctx* c) {
  const auto& f = c->cfg;
  const int64_t H = f.hidden, V = f.vocab;
  c->i_tok = add_param(c, "tok_emb", {V, H});
  c->i_pos = add_param(c, "pos_emb", {f.max_seq, H});
  if (!f.pre_ln) { c->i_eg = add_param(c, "emb_ln_g", {H}); c->i_eb = add_param(c, "emb_ln_b", {H}); }
  for (int l = 0; l < f.n_layers; ++l) {
    const std::string p = "layer" + std::to_string(l) + ".";
    const int64_t F = ffn_of(f, l);
    LayerIdx x;
    x.wqkv = add_param(c, p + "wqkv", {3 * H, H}); x.bqkv = add_param(c, p + "bqkv", {3 * H});
    x.wo = add_param(c, p + "wo", {H, H});         x.bo = add_param(c, p + "bo", {H});
    x.ln1g = add_param(c, p + "ln1_g", {H});       x.ln1b = add_param(c, p + "ln1_b", {H});
    x.w1 = add_param(c, p + "w1", {F, H});         x.b1 = add_param(c, p + "b1", {F});
    x.w2 = add_param(c, p + "w2", {H, F});         x.b2 = add_param(c, p + "b2", {H});
    x.ln2g = add_param(c, p + "ln2_g", {H});       x.ln2b = add_param(c, p + "ln2_b", {H});
    c->lidx.push_back(x);
  }
  if (f.pre_ln) { c->i_fg = add_param(c, "final_ln_g", {H}); c->i_fb = add_param(c, "final_ln_b", {H}); }
  if (f.head) {
    c->i_wt = add_param(c, "head.wt", {H, H});   c->i_bt = add_param(c, "head.bt", {H});
    c->i_hg = add_param(c, "head.ln_g", {H});    c->i_hb = add_param(c, "head.ln_b", {H});
    c->i_bdec = add_param(c, "head.bdec", {V});
  }
}

// ------------------------------------------------------------------ step executor
class Step {
 public:
  Step(mimose_ctx* c, int B, int L, uint64_t plan, bool collect)
      : c_(c), f_(c->cfg), B_(B), L_(L), T_(B * L), plan_(plan), collect_(collect), dry_(c->dry),
        st_(c->stream), dt_(c->cfg.dtype), es_(c->elt()) {}

  void run(const int32_t* tokens, const int32_t* labels, float* loss_out, bool wait);
  const int32_t* lens_host = nullptr;   // padded batch: real tokens per sample ([B], host), else null

  // collected bytes (valid after run)
  uint64_t e_bytes = 0, g_bytes = 0;
  std::vector<uint64_t> a_bytes, b_bytes, w_bytes;

 private:
  mimose_ctx* c_;
  const mimose_model_cfg& f_;
  int B_, L_, T_;
  uint64_t plan_;
  bool collect_, dry_;
  hipStream_t st_;
  int dt_, es_;
  // embedding-stage tensors
  int32_t *ids_ = nullptr, *labels_ = nullptr, *order_ = nullptr, *seg_ = nullptr, *lens_ = nullptr;
  // Gradient of the residual stream.  Post-LN blocks in bf16 carry it in fp32 (gA_, gB_) and
  // keep the bf16 copies the products consume in oA_, oB_; otherwise the carriers have the
  // storage type and oA_/oB_ alias them (LayerNorm backward then works in place).
  void *gA_ = nullptr, *gB_ = nullptr, *oA_ = nullptr, *oB_ = nullptr, *emb_sum_ = nullptr, *h0_ = nullptr;
  bool wide_ = false;   // fp32 residual sums and gradient carriers
  int stage_turn_ = 0;  // which pinned staging buffer this step uses
  int n_seg_ = 0, n_valid_ = 0;

  // times everything enqueued during its lifetime as one launch of kernel class `cls`
  struct Timed {
    mimose_ctx* c; hipEvent_t b = nullptr;
    Timed(Step* s, int cls, double work) : c(s->c_) {
      if (!c->prof_on || s->dry_) { c = nullptr; return; }
      hipEvent_t a = c->prof_event();
      b = c->prof_event();
      if (!a || !b) { c = nullptr; return; }
      (void)hipEventRecord(a, s->st_);
      c->prof_pending.push_back({cls, work, a, b});
    }
    ~Timed() { if (c) (void)hipEventRecord(b, c->stream); }
  };
  double es_d() const { return (double)es_; }

  void* w(int i) const { return c_->params[i].w; }
  float* g(int i) const { return c_->params[i].g; }
  void* talloc(int64_t elems) { return c_->arena.alloc((uint64_t)elems * es_); }
  void* walloc(int64_t elems) { return c_->arena.alloc((uint64_t)elems * (wide_ ? 4 : es_)); }

  void gemm(const mk::GemmArgs& a) {
    if (dry_) return;
    forked_ = false;                      // the main stream moves on: later side work needs a new fork
    mk::GemmArgs b = a;
    if (c_->prof_on) {                    // timed by the kernel's own start and end, not by markers around the launch
      b.time_start = c_->prof_event();
      b.time_stop = c_->prof_event();
      if (b.time_start && b.time_stop) c_->prof_pending.push_back({MIMOSE_K_GEMM, 2.0 * a.M * a.N * a.K, b.time_start, b.time_stop});
      else b.time_start = b.time_stop = nullptr;
    }
    if (!mk::gemm(dt_, b, st_)) throw StepError{MIMOSE_ERR_INVALID_ARG, "gemm: unsupported alignment"};
  }
  // Y[T,out] = X[T,in] W[out,in]^T + bias (+ resid) (GELU: Y = pre-activation, act = GELU(Y))
  void linear(const void* X, int in, int wi, int bi, void* Y, int out, int64_t ldy, const void* resid = nullptr,
              void* act = nullptr, int gelu = 0, bool out_f32 = false) {
    mk::GemmArgs a{X, in, true, w(wi), in, true, Y, ldy, out_f32, T_, out, in};
    a.bias = bi >= 0 ? w(bi) : nullptr;
    a.resid = resid; a.ldr = out;
    a.gelu_out = act; a.gelu = gelu;
    gemm(a);
  }
  // Dropout sites: 0 the embedding output; layer l: 4(l+1)+1 the attention block's output
  // projection, 4(l+1)+2 the feed-forward block's output (4(l+1) is kept for the attention
  // probabilities).
  bool drop_on() const { return c_->p_hidden > 0.f; }
  mk::DropDesc drop_desc(uint32_t site, bool attn = false) const {
    mk::DropDesc d;
    const double p = (double)(attn ? c_->p_attn : c_->p_hidden);
    if (p <= 0.0) return d;
    d.thr = (uint32_t)std::min(std::floor(p * 4294967296.0 + 0.5), 4294967295.0);
    d.scale = (float)(1.0 / (1.0 - p));
    d.k0 = (uint32_t)c_->drop_seed; d.k1 = (uint32_t)(c_->drop_seed >> 32);
    d.site = site; d.step = (uint32_t)c_->drop_step;
    return d;
  }
  // io (storage type, or fp32 when io_f32) = resid + dropout(src); src may be io
  void dropout(void* dst, const void* src, bool io_f32, const void* resid, uint32_t site) {
    if (!dry_) mk::dropout_apply(dt_, dst, src, io_f32, resid, (int64_t)T_ * f_.hidden, drop_desc(site), st_);
  }
  // dX[T,in] = dY[T,out] W[out,in] (+ resid)
  void dgrad(const void* dY, int64_t ldy, int out, int wi, void* dX, int in, const void* resid = nullptr,
             bool out_f32 = false) {
    mk::GemmArgs a{dY, ldy, true, w(wi), in, false, dX, in, out_f32, T_, in, out};
    a.resid = resid; a.ldr = in;
    gemm(a);
  }
  // dW[out,in] = dY^T X, db[out] = column sums of dY
  void wgrad(const void* dY, int64_t ldy, int out, const void* X, int in, int wi, int bi, bool late = false) {
    mk::GemmArgs a{dY, ldy, false, X, in, false, g(wi), in, true, out, in, T_};
    a.a_rowsum = bi >= 0 ? g(bi) : nullptr;
    with_workspace(a, late);
  }
  // Weight-gradient products may cut their reduction in parts; the scratch for that is taken
  // once per layer backward / head (a size fixed by the weight shapes), so that every
  // component of the step's memory stays a polynomial of the input size.
  void* ws_ = nullptr;
  size_t ws_bytes_ = 0;
  void reserve_workspace(std::initializer_list<std::pair<int, int>> shapes) {
    size_t need = 0;
    if (dt_ == mk::BF16)
      for (auto& s : shapes) need = std::max(need, mk::gemm_workspace_bytes(s.first, s.second));
    ws_ = need ? c_->arena.alloc(need) : nullptr;
    ws_bytes_ = need;
  }
  // late: the product reads and writes nothing that the layer's pop frees (its operand and its
  // scratch live in the step-long slot), so the layer's end need not wait for it
  void with_workspace(mk::GemmArgs& a, bool late = false) {
    a.workspace = late ? late_ws_ : ws_;
    a.workspace_bytes = late ? late_ws_bytes_ : ws_bytes_;
    if (dry_) return;
    // per-kernel timing brackets work on the main stream only, so it keeps everything there
    if (!c_->side || c_->prof_on) { gemm(a); return; }
    if (!forked_) fork();
    if (late && hipEventRecord(c_->ev_early, c_->side) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "marking the weight-gradient stream failed"};
    if (!mk::gemm(dt_, a, c_->side)) throw StepError{MIMOSE_ERR_INVALID_ARG, "gemm: unsupported alignment"};
    if (late) {
      if (hipEventRecord(c_->ev_late, c_->side) != hipSuccess)
        throw StepError{MIMOSE_ERR_HIP, "marking the weight-gradient stream failed"};
      late_pending_ = early_marked_ = true;
    }
    side_busy_ = true;
  }
  // Step-long slot for the gradient of the fused QKV projection and the scratch of its
  // weight-gradient product (post-LN stacks; see layer_backward).
  void* late_dqkv_ = nullptr;
  void* late_ws_ = nullptr;
  size_t late_ws_bytes_ = 0;
  bool late_pending_ = false, early_marked_ = false;
  bool late_ok() const { return !f_.pre_ln; }
  // before the slot is written again: the product that still reads it must be done
  void wait_late() {
    if (!late_pending_) return;
    if (hipStreamWaitEvent(st_, c_->ev_late, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "waiting for the weight-gradient stream failed"};
    late_pending_ = false;
  }
  // the main stream waits for the weight-gradient products issued before the late one
  void join_early() {
    if (!early_marked_) { join(); return; }
    if (hipStreamWaitEvent(st_, c_->ev_early, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "join of the weight-gradient stream failed"};
    early_marked_ = false;
  }
  // the main stream waits for every weight-gradient product issued so far (before their inputs
  // or scratch are reused, and before anything reads the gradients)
  bool side_busy_ = false;
  void join() {
    if (!side_busy_) return;
    if (hipEventRecord(c_->ev_join, c_->side) != hipSuccess || hipStreamWaitEvent(st_, c_->ev_join, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "join of the weight-gradient stream failed"};
    side_busy_ = late_pending_ = early_marked_ = false;
  }
  void ln_fwd(const void* x, int gi, int bi, void* y, bool x_f32 = false) {
    Timed t(this, MIMOSE_K_LN_FWD, (x_f32 ? 6.0 : 2.0 * es_d()) * T_ * f_.hidden);
    if (!dry_) mk::layernorm_fwd(dt_, x, x_f32, w(gi), w(bi), y, T_, f_.hidden, f_.ln_eps, st_);
  }
  void ln_bwd(const void* dy, const void* x, int gi, int bi, void* dx, const void* add, bool dy_f32 = false,
              bool x_f32 = false) {
    const uint64_t m = c_->arena.top();
    float* partial = (float*)c_->arena.alloc((uint64_t)mk::partial_rows(T_) * 2 * f_.hidden * 4);
    const double bytes = (dy_f32 ? 4.0 : es_d()) + (x_f32 ? 4.0 : es_d()) + es_d() * (add ? 2.0 : 1.0);
    Timed t(this, MIMOSE_K_LN_BWD, bytes * T_ * f_.hidden);
    if (!dry_)
      mk::layernorm_bwd(dt_, dy, dy_f32, x, x_f32, w(gi), dx, add, g(gi), g(bi), partial, T_, f_.hidden, f_.ln_eps, st_);
    c_->arena.pop_to(m);
  }

  // The same in two halves, for the layers' backward: the row pass on the main stream (its
  // partial sums stay allocated until the layer's end), the small reduction to dgamma, dbeta on
  // the weight-gradient stream after the next fork, off the chain of data gradients.
  float* ln_bwd_rows(const void* dy, const void* x, int gi, void* dx, const void* add, bool dy_f32 = false,
                     bool x_f32 = false) {
    float* partial = (float*)c_->arena.alloc((uint64_t)mk::partial_rows(T_) * 2 * f_.hidden * 4);
    const double bytes = (dy_f32 ? 4.0 : es_d()) + (x_f32 ? 4.0 : es_d()) + es_d() * (add ? 2.0 : 1.0);
    Timed t(this, MIMOSE_K_LN_BWD, bytes * T_ * f_.hidden);
    if (!dry_) mk::layernorm_bwd_rows(dt_, dy, dy_f32, x, x_f32, w(gi), dx, add, partial, T_, f_.hidden, f_.ln_eps, st_);
    return partial;
  }
  void ln_bwd_reduce(const float* partial, int gi, int bi) {
    if (dry_) return;
    const bool aside = c_->side && !c_->prof_on;
    mk::layernorm_bwd_reduce(partial, g(gi), g(bi), T_, f_.hidden, aside ? c_->side : st_);
    if (aside) side_busy_ = true;
  }
  // One fork serves everything issued on the weight-gradient stream until the main stream
  // launches its next product (every group of side work here is followed by one).
  bool forked_ = false;
  void fork() {
    if (dry_ || !c_->side || c_->prof_on) return;
    if (hipEventRecord(c_->ev_fork, st_) != hipSuccess || hipStreamWaitEvent(c_->side, c_->ev_fork, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "fork to the weight-gradient stream failed"};
    forked_ = true;
  }

  void embed_stage(const int32_t* tokens, const int32_t* labels);
  void embed_sort(const int32_t* tokens);
  void alloc_layer(int l, LayerActs& A);
  void layer_forward(int l, LayerActs& A, bool rebuild = false);
  void layer_forward_rows(int l, LayerActs& A, int b0, int nb, hipStream_t s);
  bool split_forward() const;
  void cross_sync();
  void layer_backward(int l, LayerActs& A);
  void head(float* loss_dev);
  void embed_backward();
};

void Step::embed_stage(const int32_t* tokens, const int32_t* labels) {
  const int H = f_.hidden;
  // ids, labels, sort order, run boundaries, per-sample lengths (the last B only read for padded batches)
  int32_t* ints = (int32_t*)c_->arena.alloc((uint64_t)(4 * (int64_t)T_ + 1 + B_) * 4);
  ids_ = ints; labels_ = ints ? ints + T_ : nullptr; order_ = ints ? ints + 2 * (int64_t)T_ : nullptr;
  seg_ = ints ? ints + 3 * (int64_t)T_ : nullptr;
  lens_ = ints && lens_host ? ints + 4 * (int64_t)T_ + 1 : nullptr;
  wide_ = !f_.pre_ln && dt_ == mk::BF16;
  gA_ = walloc((int64_t)T_ * H);
  gB_ = walloc((int64_t)T_ * H);
  oA_ = wide_ ? talloc((int64_t)T_ * H) : gA_;
  oB_ = wide_ ? talloc((int64_t)T_ * H) : gB_;
  if (!f_.pre_ln) emb_sum_ = talloc((int64_t)T_ * H);
  h0_ = talloc((int64_t)T_ * H);
  if (late_ok()) {
    late_dqkv_ = talloc(3 * (int64_t)T_ * H);
    late_ws_bytes_ = dt_ == mk::BF16 ? mk::gemm_workspace_bytes(3 * H, H) : 0;
    late_ws_ = late_ws_bytes_ ? c_->arena.alloc(late_ws_bytes_) : nullptr;
  }
  if (dry_) return;

  // host side: stable sort of positions by token id, run boundaries of equal ids
  const size_t need = 4 * (size_t)T_ + 1 + (size_t)B_;
  const int turn = c_->stage_turn;
  c_->stage_turn ^= 1;
  if (c_->stage_busy[turn]) {               // copies of the step before last out of this buffer: long done
    HIPCHK(c_, hipEventSynchronize(c_->ev_stage[turn]));
    c_->stage_busy[turn] = false;
  }
  if (c_->stage_buf_ints[turn] < need) {
    if (c_->stage_buf[turn]) HIPCHK(c_, hipHostFree(c_->stage_buf[turn]));
    c_->stage_buf[turn] = nullptr; c_->stage_buf_ints[turn] = 0;
    HIPCHK(c_, hipHostMalloc((void**)&c_->stage_buf[turn], need * 4 + 1024, hipHostMallocDefault));
    c_->stage_buf_ints[turn] = need;
  }
  c_->stage = c_->stage_buf[turn];
  stage_turn_ = turn;
  int32_t* s = c_->stage;
  std::memcpy(s, tokens, (size_t)T_ * 4);
  std::memcpy(s + T_, labels, (size_t)T_ * 4);
  if (lens_host) {                        // padded positions are never scored
    for (int b = 0; b < B_; ++b)
      for (int p = lens_host[b]; p < L_; ++p) s[T_ + (size_t)b * L_ + p] = -1;
    std::memcpy(s + 4 * (size_t)T_ + 1, lens_host, (size_t)B_ * 4);
    HIPCHK(c_, hipMemcpyAsync(lens_, s + 4 * (size_t)T_ + 1, (size_t)B_ * 4, hipMemcpyHostToDevice, st_));
  }
  HIPCHK(c_, hipMemcpyAsync(ints, s, 2 * (size_t)T_ * 4, hipMemcpyHostToDevice, st_));
  Timed t(this, MIMOSE_K_EMBED_FWD, (f_.pre_ln ? 3.0 : 4.0) * T_ * H * es_d());
  mk::embed_fwd(dt_, ids_, w(c_->i_tok), w(c_->i_pos), f_.pre_ln ? nullptr : w(c_->i_eg),
                f_.pre_ln ? nullptr : w(c_->i_eb), emb_sum_, h0_, B_, L_, H, f_.ln_eps, !f_.pre_ln, st_);
  if (drop_on()) dropout(h0_, h0_, false, nullptr, 0);
}

void Step::alloc_layer(int l, LayerActs& A) {
  const int64_t TH = (int64_t)T_ * f_.hidden, TF = (int64_t)T_ * ffn_of(f_, l);
  if (!A.has_out) {                   // first pass: the boundary tensor goes first
    A.mark = c_->arena.top();
    A.out = talloc(TH);
    A.after_out = c_->arena.top();
    A.has_out = true;                 // (not the pointer: a host-only context hands out null)
  }
  if (f_.pre_ln) A.n1 = talloc(TH);   // LN1(x)
  A.qkv = talloc(3 * TH);
  A.lse = (float*)c_->arena.alloc((uint64_t)B_ * f_.n_heads * L_ * 4);
  A.ctx = talloc(TH);
  A.s1 = walloc(TH);                  // post-LN: x + proj (LN1 input, fp32 when wide); pre-LN: u = x + proj
  A.u = talloc(TH);                   // post-LN: LN1(s1); pre-LN: LN2(u)
  A.pre = talloc(TF);
  A.act = talloc(TF);
  if (!f_.pre_ln) A.s2 = walloc(TH);  // post-LN: u + ffn (LN2 input, fp32 when wide)
}

// The forward of samples [b0, b0 + nb) of the batch on stream s: the same kernels on a range of
// rows.  Nothing in a layer's forward couples two samples, and every product uses the same tile
// shape and reduction order wherever its rows sit, so the values are those of layer_forward
// bit for bit.  Two such halves on two streams let one half's kernels fill the compute units
// that the other's leave idle in their last round of tiles.
void Step::layer_forward_rows(int l, LayerActs& A, int b0, int nb, hipStream_t s) {
  const LayerIdx& p = c_->lidx[l];
  const int H = f_.hidden, F = ffn_of(f_, l), nh = f_.n_heads, d = H / nh;
  const int gelu = f_.gelu_tanh ? mk::GELU_TANH : mk::GELU_ERF;
  const int64_t r0 = (int64_t)b0 * L_;
  const int rows = nb * L_;
  auto at = [&](const void* base, int64_t width, bool f32 = false) -> void* {
    return (char*)const_cast<void*>(base) + r0 * width * (f32 ? 4 : (int64_t)es_);
  };
  auto lin = [&](const void* X, int in, int wi, int bi, void* Y, int out, const void* resid, void* act, int ge,
                 bool out_f32) {
    mk::GemmArgs a{X, in, true, w(wi), in, true, Y, out, out_f32, rows, out, in};
    a.bias = w(bi);
    a.resid = resid; a.ldr = out;
    a.gelu_out = act; a.gelu = ge;
    if (!mk::gemm(dt_, a, s)) throw StepError{MIMOSE_ERR_INVALID_ARG, "gemm: unsupported alignment"};
  };
  auto ln = [&](const void* x, int gi, int bi, void* y, bool x_f32) {
    mk::layernorm_fwd(dt_, x, x_f32, w(gi), w(bi), y, rows, H, f_.ln_eps, s);
  };
  const void* x = at(A.x, H);
  const void* a = x;
  if (f_.pre_ln) { ln(x, p.ln1g, p.ln1b, at(A.n1, H), false); a = at(A.n1, H); }
  lin(a, H, p.wqkv, p.bqkv, at(A.qkv, 3 * H), 3 * H, nullptr, nullptr, 0, false);
  mk::attention_fwd(dt_, at(A.qkv, 3 * H), at(A.ctx, H), A.lse + (int64_t)b0 * nh * L_, lens_ ? lens_ + b0 : nullptr, nb, L_,
                    nh, d, f_.causal, mk::DropDesc(), s);
  lin(at(A.ctx, H), H, p.wo, p.bo, at(A.s1, H, wide_), H, x, nullptr, 0, wide_);
  if (f_.pre_ln) {
    ln(at(A.s1, H), p.ln2g, p.ln2b, at(A.u, H), false);
    lin(at(A.u, H), H, p.w1, p.b1, at(A.pre, F), F, nullptr, at(A.act, F), gelu, false);
    lin(at(A.act, F), F, p.w2, p.b2, at(A.out, H), H, at(A.s1, H), nullptr, 0, false);
  } else {
    ln(at(A.s1, H, wide_), p.ln1g, p.ln1b, at(A.u, H), wide_);
    lin(at(A.u, H), H, p.w1, p.b1, at(A.pre, F), F, nullptr, at(A.act, F), gelu, false);
    lin(at(A.act, F), F, p.w2, p.b2, at(A.s2, H, wide_), H, at(A.u, H), nullptr, 0, wide_);
    ln(at(A.s2, H, wide_), p.ln2g, p.ln2b, at(A.out, H), wide_);
  }
}

// Both halves on their own stream: only a real step, without dropout (whose masks count elements
// from the tensor's start), without per-kernel or per-layer timing, with two samples at least.
bool Step::split_forward() const {
  return !dry_ && c_->side && !c_->prof_on && !collect_ && !drop_on() && c_->p_attn <= 0.f && B_ >= 2;
}

// each stream waits for what the other has been given so far
void Step::cross_sync() {
  if (hipEventRecord(c_->ev_fork, st_) != hipSuccess || hipStreamWaitEvent(c_->side, c_->ev_fork, 0) != hipSuccess ||
      hipEventRecord(c_->ev_join, c_->side) != hipSuccess || hipStreamWaitEvent(st_, c_->ev_join, 0) != hipSuccess)
    throw StepError{MIMOSE_ERR_HIP, "synchronising the two forward streams failed"};
}

// rebuild: the forward of a checkpointed layer run again before its backward.  Its output is
// still in place (it is the layer's boundary tensor), so a post-LN layer leaves out the final
// LayerNorm, which produces nothing else; later layers' pending products may still read it.
void Step::layer_forward(int l, LayerActs& A, bool rebuild) {
  const LayerIdx& p = c_->lidx[l];
  const int H = f_.hidden, F = ffn_of(f_, l), nh = f_.n_heads, d = H / nh;
  const int gelu = f_.gelu_tanh ? mk::GELU_TANH : mk::GELU_ERF;
  const void* a = A.x;
  if (f_.pre_ln) { ln_fwd(A.x, p.ln1g, p.ln1b, A.n1); a = A.n1; }
  linear(a, H, p.wqkv, p.bqkv, A.qkv, 3 * H, 3 * H);
  {
    Timed t(this, MIMOSE_K_ATTN_FWD, 4.0 * T_ * L_ * H * (f_.causal ? 0.5 : 1.0));
    if (!dry_)
      mk::attention_fwd(dt_, A.qkv, A.ctx, A.lse, lens_, B_, L_, nh, d, f_.causal, drop_desc(4 * (uint32_t)(l + 1), true), st_);
  }
  // with dropout the product lands in the sum's buffer and an element-wise pass makes
  // sum = residual + dropout(product) in place; without it the residual rides in the epilogue
  const bool drop = drop_on();
  const uint32_t site_o = 4 * (uint32_t)(l + 1) + 1, site_f = site_o + 1;
  linear(A.ctx, H, p.wo, p.bo, A.s1, H, H, drop ? nullptr : A.x, nullptr, 0, wide_);
  if (drop) dropout(A.s1, A.s1, wide_, A.x, site_o);
  if (f_.pre_ln) {
    ln_fwd(A.s1, p.ln2g, p.ln2b, A.u);
    linear(A.u, H, p.w1, p.b1, A.pre, F, F, nullptr, A.act, gelu);
    linear(A.act, F, p.w2, p.b2, A.out, H, H, drop ? nullptr : A.s1);
    if (drop) dropout(A.out, A.out, false, A.s1, site_f);
  } else {
    ln_fwd(A.s1, p.ln1g, p.ln1b, A.u, wide_);
    linear(A.u, H, p.w1, p.b1, A.pre, F, F, nullptr, A.act, gelu);
    linear(A.act, F, p.w2, p.b2, A.s2, H, H, drop ? nullptr : A.u, nullptr, 0, wide_);
    if (drop) dropout(A.s2, A.s2, wide_, A.u, site_f);
    if (!rebuild) ln_fwd(A.s2, p.ln2g, p.ln2b, A.out, wide_);
  }
}

// Gradient of the layer output arrives in gA_; the gradient of its input leaves in gA_.
void Step::layer_backward(int l, LayerActs& A) {
  const LayerIdx& p = c_->lidx[l];
  const int H = f_.hidden, F = ffn_of(f_, l), nh = f_.n_heads, d = H / nh;
  const int64_t TH = (int64_t)T_ * H, TF = (int64_t)T_ * F;
  Arena& ar = c_->arena;
  if (late_ok()) reserve_workspace({{H, F}, {F, H}, {H, H}});
  else reserve_workspace({{H, F}, {F, H}, {H, H}, {3 * H, H}});
  const uint64_t m0 = ar.top();
  // post-LN: oA = d s2 (LayerNorm 2 backward of the incoming gradient); pre-LN: the incoming
  // gradient is d s2 itself (oA aliases gA)
  float* part2 = f_.pre_ln ? nullptr : ln_bwd_rows(gA_, A.s2, p.ln2g, oA_, nullptr, wide_, wide_);
  // with dropout the branch sees the masked gradient (a copy: the residual path keeps the whole one)
  const bool drop = drop_on();
  const uint32_t site_o = 4 * (uint32_t)(l + 1) + 1, site_f = site_o + 1;
  const void* dffn = oA_;
  if (drop) { void* m = talloc(TH); dropout(m, oA_, false, nullptr, site_f); dffn = m; }
  fork();
  if (part2) ln_bwd_reduce(part2, p.ln2g, p.ln2b);
  wgrad(dffn, H, H, A.act, F, p.w2, p.b2);
  // Carriers of the storage type: that product reads gA_ (dffn is oA_, which is gA_), and the
  // layer's last data gradient writes gA_ before the streams join, so it is ordered by an event.
  const bool guard_gA = !dry_ && side_busy_ && dffn == gA_;
  if (guard_gA && hipEventRecord(c_->ev_w2, c_->side) != hipSuccess)
    throw StepError{MIMOSE_ERR_HIP, "marking the weight-gradient stream failed"};
  void* dact = talloc(TF);
  dgrad(dffn, H, H, p.w2, dact, F);
  {
    Timed t(this, MIMOSE_K_GELU_BWD, 3.0 * TF * es_d());
    if (!dry_) mk::gelu_bwd(dt_, dact, A.pre, TF, f_.gelu_tanh, st_);        // dact = d pre
  }
  wgrad(dact, F, F, A.u, H, p.w1, p.b1);
  // dact stays allocated until the end of the layer: the weight-gradient stream may still read
  // it, and waiting for that stream here would idle the chip for the length of the hand-over
  float* part1;
  if (f_.pre_ln) {
    dgrad(dact, F, F, p.w1, gB_, H);                                          // gB = d LN2(u)
    part1 = ln_bwd_rows(gB_, A.s1, p.ln2g, gB_, gA_);                         // gB = d u
  } else {
    dgrad(dact, F, F, p.w1, gB_, H, oA_, wide_);                              // gB = d u = d s2 + FFN path
    part1 = ln_bwd_rows(gB_, A.s1, p.ln1g, oB_, nullptr, wide_, wide_);       // oB = d s1
  }
  const void* dproj = oB_;
  if (drop) { void* m = talloc(TH); dropout(m, oB_, false, nullptr, site_o); dproj = m; }
  fork();
  if (f_.pre_ln) ln_bwd_reduce(part1, p.ln2g, p.ln2b);
  else ln_bwd_reduce(part1, p.ln1g, p.ln1b);
  wgrad(dproj, H, H, A.ctx, H, p.wo, p.bo);
  void* dctx = talloc(TH);
  dgrad(dproj, H, H, p.wo, dctx, H);
  // Post-LN: the QKV weight gradient is the last product of the layer, issued when the main
  // stream has one product left; waiting for it at the layer's end idles the chip.  Its operands
  // (this gradient, in a step-long slot, and the layer's input, which the pop does not free) and
  // its scratch outlive the layer, so only the earlier products are waited for here and this one
  // before the slot is written again, a layer later.
  void* dqkv = late_ok() ? late_dqkv_ : talloc(3 * TH);
  float* delta = (float*)ar.alloc((uint64_t)B_ * nh * L_ * 4);
  if (late_ok() && !dry_) wait_late();
  {
    Timed t(this, MIMOSE_K_ATTN_BWD, 8.0 * T_ * L_ * H * (f_.causal ? 0.5 : 1.0));
    if (!dry_)
      mk::attention_bwd(dt_, A.qkv, A.ctx, dctx, A.lse, delta, dqkv, lens_, B_, L_, nh, d, f_.causal,
                        drop_desc(4 * (uint32_t)(l + 1), true), st_);
  }
  const void* a = f_.pre_ln ? A.n1 : A.x;
  wgrad(dqkv, 3 * H, 3 * H, a, H, p.wqkv, p.bqkv, late_ok());
  if (guard_gA && hipStreamWaitEvent(st_, c_->ev_w2, 0) != hipSuccess)
    throw StepError{MIMOSE_ERR_HIP, "waiting for the weight-gradient stream failed"};
  if (f_.pre_ln) {
    dgrad(dqkv, 3 * H, 3 * H, p.wqkv, gA_, H);                                // gA = d LN1(x)
    join();
    ar.pop_to(m0);
    ln_bwd(gA_, A.x, p.ln1g, p.ln1b, gA_, gB_);                               // gA = d x
  } else {
    dgrad(dqkv, 3 * H, 3 * H, p.wqkv, gA_, H, oB_, wide_);                    // gA = d x = d s1 + attention path
    if (dry_) {} else join_early();
    ar.pop_to(m0);
  }
}

// Head forward, loss, head backward.  Leaves the gradient of the last layer's output in gA_.
void Step::head(float* loss_dev) {
  const int H = f_.hidden, V = f_.vocab;
  const int64_t TH = (int64_t)T_ * H, ldv = c_->ldv();
  const int gelu = f_.gelu_tanh ? mk::GELU_TANH : mk::GELU_ERF;
  const void* hlast = f_.n_layers ? c_->acts[f_.n_layers - 1].out : h0_;
  reserve_workspace({{V, H}, {H, H}});
  const void* hs = hlast;
  void* hs_buf = nullptr;
  if (f_.pre_ln) { hs_buf = talloc(TH); ln_fwd(hlast, c_->i_fg, c_->i_fb, hs_buf); hs = hs_buf; }
  void *z = nullptr, *gz = nullptr, *t = nullptr;
  const void* dec_in = hs;
  if (f_.head) {
    z = talloc(TH); gz = talloc(TH); t = talloc(TH);
    linear(hs, H, c_->i_wt, c_->i_bt, z, H, H, nullptr, gz, gelu);
    ln_fwd(gz, c_->i_hg, c_->i_hb, t);
    dec_in = t;
  }
  void* logits = talloc((int64_t)T_ * ldv);
  float* row_loss = (float*)c_->arena.alloc((uint64_t)T_ * 4);
  {
    mk::GemmArgs a{dec_in, H, true, w(c_->i_tok), H, true, logits, ldv, false, T_, V, H};
    a.bias = f_.head ? w(c_->i_bdec) : nullptr;
    gemm(a);
  }
  {
    Timed t(this, MIMOSE_K_XENT, 2.0 * T_ * ldv * es_d());
    if (!dry_) mk::softmax_xent(dt_, logits, ldv, labels_, row_loss, loss_dev, T_, V, n_valid_, st_);
  }
  // tied decoder: its weight gradient overwrites the embedding gradient, the embedding
  // backward adds onto it later
  {
    mk::GemmArgs a{logits, ldv, false, dec_in, H, false, g(c_->i_tok), H, true, V, H, T_};
    a.a_rowsum = f_.head ? g(c_->i_bdec) : nullptr;
    with_workspace(a);
  }
  void* dhs = f_.pre_ln ? talloc(TH) : gA_;            // post-LN: straight into the (possibly fp32) carrier
  // scratch of the vocabulary-long data gradient (its own: the decoder's weight gradient uses the
  // other one at the same time on the second stream); a constant of the model
  const size_t long_ws_bytes = dt_ == mk::BF16 && V >= 8192 ? mk::gemm_long_k_workspace_bytes(H) : 0;
  void* long_ws = long_ws_bytes ? c_->arena.alloc(long_ws_bytes) : nullptr;
  // the loss kernel left zeros in the padding columns [V, ldv) of the logits' gradient
  auto vocab_dgrad = [&](void* out, bool out_f32) {
    mk::GemmArgs a{logits, ldv, true, w(c_->i_tok), H, false, out, H, out_f32, T_, H, V};
    a.a_tail_zero = true;
    a.workspace = long_ws; a.workspace_bytes = long_ws_bytes;
    gemm(a);
  };
  if (f_.head) {
    void* dt = talloc(TH);
    vocab_dgrad(dt, false);
    ln_bwd(dt, gz, c_->i_hg, c_->i_hb, dt, nullptr);                          // dt = d gz
    if (!dry_) mk::gelu_bwd(dt_, dt, z, TH, f_.gelu_tanh, st_);               // dt = d z
    wgrad(dt, H, H, hs, H, c_->i_wt, c_->i_bt);
    dgrad(dt, H, H, c_->i_wt, dhs, H, nullptr, wide_);
  } else {
    vocab_dgrad(dhs, wide_);
  }
  if (f_.pre_ln) ln_bwd(dhs, hlast, c_->i_fg, c_->i_fb, gA_, nullptr);
  join();
}

// Host side of the embedding backward: stable sort of positions by token id and the run
// boundaries of equal ids.  Only the last kernels of the step read them, so this runs after the
// forward launches are queued, while the device is busy (second half of the pinned staging
// buffer; the first half is still being read by the copy of the ids).
void Step::embed_sort(const int32_t* tokens) {
  if (dry_) return;
  int32_t* s = c_->stage;
  std::vector<int32_t>& count = c_->sort_count;
  count.assign((size_t)f_.vocab + 1, 0);
  for (int t = 0; t < T_; ++t) ++count[(size_t)tokens[t] + 1];
  n_seg_ = 0;
  int32_t* seg = s + 3 * (size_t)T_;
  for (int v = 0; v < f_.vocab; ++v) {
    if (count[v + 1]) seg[n_seg_++] = count[v];
    count[v + 1] += count[v];
  }
  seg[n_seg_] = T_;
  int32_t* order = s + 2 * (size_t)T_;
  for (int t = 0; t < T_; ++t) order[count[tokens[t]]++] = t;
  HIPCHK(c_, hipMemcpyAsync(order_, order, (2 * (size_t)T_ + 1) * 4, hipMemcpyHostToDevice, st_));
  HIPCHK(c_, hipEventRecord(c_->ev_stage[stage_turn_], st_));     // the last copy out of this staging buffer
  c_->stage_busy[stage_turn_] = true;
}

void Step::embed_backward() {
  const int H = f_.hidden;
  if (drop_on()) dropout(gA_, gA_, wide_, nullptr, 0);
  if (!f_.pre_ln) ln_bwd(gA_, emb_sum_, c_->i_eg, c_->i_eb, oA_, nullptr, wide_, false);
  if (!dry_)
    mk::embed_bwd(dt_, oA_, ids_, order_, seg_, n_seg_, g(c_->i_tok), g(c_->i_pos), B_, L_, H, f_.max_seq, st_);
}

void Step::run(const int32_t* tokens, const int32_t* labels, float* loss_out, bool wait) {
  Arena& ar = c_->arena;
  const int N = f_.n_layers;
  a_bytes.assign(N, 0); b_bytes.assign(N, 0); w_bytes.assign(N, 0);
  ar.pop_to(c_->fixed_top);
  ar.reset_high();
  if (!dry_) {
    n_valid_ = 0;
    for (int b = 0; b < B_; ++b) {
      const int n = lens_host ? lens_host[b] : L_;
      for (int p = 0; p < n; ++p) n_valid_ += labels[(size_t)b * L_ + p] >= 0;
    }
  }
  const uint64_t base = ar.top();
  float* loss_dev = (float*)ar.alloc(4);
  embed_stage(tokens, labels);
  e_bytes = ar.top() - base;

  c_->acts.assign(N, LayerActs());
  const void* x = h0_;
  // the two halves of the batch run through the layers on two streams, meeting only where a
  // dropped layer's memory is handed to the next layer and at the end
  const bool split = split_forward() && N > 0;
  const int nb0 = B_ / 2;
  if (split) {
    if (hipEventRecord(c_->ev_fork, st_) != hipSuccess || hipStreamWaitEvent(c_->side, c_->ev_fork, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "fork of the forward streams failed"};
  }
  for (int l = 0; l < N; ++l) {
    LayerActs& A = c_->acts[l];
    A.x = x;
    alloc_layer(l, A);
    const bool timed = collect_ && !dry_ && (int)c_->ev_layer.size() == 2 * N;
    if (timed) HIPCHK(c_, hipEventRecord(c_->ev_layer[2 * l], st_));
    if (split) {
      layer_forward_rows(l, A, 0, nb0, st_);
      layer_forward_rows(l, A, nb0, B_ - nb0, c_->side);
    } else {
      layer_forward(l, A);
    }
    if (timed) HIPCHK(c_, hipEventRecord(c_->ev_layer[2 * l + 1], st_));
    a_bytes[l] = ar.top() - A.mark;
    b_bytes[l] = A.after_out - A.mark;
    if (collect_ && c_->collector == MIMOSE_COLLECTOR_TWO_FORWARDS) {
      // Section 4.2 to the letter: the first forward was the measuring one, its tensors, the output
      // included, are discarded; the second one keeps the output alone (the pop below), which is
      // what the next block's measurement starts from.  Same launches, same addresses, same values
      // (dropout masks are a function of the element, not of a generator state).
      ar.pop_to(A.mark);
      A.has_out = false;
      alloc_layer(l, A);
      layer_forward(l, A);
      b_bytes[l] = A.after_out - A.mark;
    }
    if ((plan_ >> l) & 1) {
      ar.pop_to(A.after_out); A.dropped = true;
      if (split && l + 1 < N) cross_sync();   // the next layer writes where this one's tensors are still read
    }
    x = A.out;
  }
  if (split) {
    if (hipEventRecord(c_->ev_join, c_->side) != hipSuccess || hipStreamWaitEvent(st_, c_->ev_join, 0) != hipSuccess)
      throw StepError{MIMOSE_ERR_HIP, "join of the forward streams failed"};
  }

  embed_sort(tokens);                     // host work hidden behind the queued forward
  const uint64_t m_head = ar.top();
  ar.begin_section();
  head(loss_dev);
  g_bytes = ar.section_high() - m_head;
  ar.pop_to(m_head);

  for (int l = N - 1; l >= 0; --l) {
    LayerActs& A = c_->acts[l];
    if (A.dropped) {                      // rebuild: same tensors, same values
      alloc_layer(l, A);
      layer_forward(l, A, true);
    }
    const uint64_t m = ar.top();
    ar.begin_section();
    layer_backward(l, A);
    w_bytes[l] = ar.section_high() - m;
    ar.pop_to(A.mark);
  }
  join();
  embed_backward();
  if (!dry_) {
    HIPCHK(c_, hipMemcpyAsync(c_->loss_host, loss_dev, 4, hipMemcpyDeviceToHost, st_));
    c_->loss_pending = true;
    // the caller does not want the loss now: the step stays queued and the host runs ahead
    // (collecting steps read their layer timers, profiled steps their events: they wait)
    if (!wait && !collect_ && !c_->prof_on) return;
    HIPCHK(c_, hipStreamSynchronize(st_));
    HIPCHK(c_, hipGetLastError());
    c_->loss_pending = false;
    *loss_out = *c_->loss_host;
    for (auto& p : c_->prof_pending) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
        auto& k = c_->prof[p.cls];
        k.launches++; k.ms += ms; k.work += p.work;
      }
    }
    c_->prof_pending.clear();
    c_->ev_used = 0;
  }
}

void flops(const mimose_model_cfg& f, int B, int L, uint64_t plan, double* useful, double* re) {
  const double T = (double)B * L, H = f.hidden, V = f.vocab;
  const double attn = 4.0 * L * H * (f.causal ? 0.5 : 1.0);
  const double head = 2.0 * H * V + (f.head ? 2.0 * H * H : 0.0);
  double layers = 0.0;
  *re = 0.0;
  for (int l = 0; l < f.n_layers; ++l) {
    const double layer = 8.0 * H * H + 4.0 * H * ffn_of(f, l) + attn;
    layers += layer;
    if ((plan >> l) & 1) *re += T * layer;
  }
  *useful = 3.0 * T * (layers + head);
}

int do_step(mimose_ctx* c, const int32_t* tokens, const int32_t* labels, const int32_t* lengths, int32_t B, int32_t L,
            bool dry, float* loss, uint64_t* peak, uint64_t* plan_id) {
  const auto& f = c->cfg;
  if (B < 1 || L < 1 || L > f.max_seq) return fail(c, MIMOSE_ERR_INVALID_ARG, "B >= 1 and 1 <= L <= max_seq required");
  if ((int64_t)B * L > (int64_t)1 << 28) return fail(c, MIMOSE_ERR_INVALID_ARG, "B*L too large");
  if (!dry) {
    if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context: no device arena");
    if (!tokens || !labels) return fail(c, MIMOSE_ERR_INVALID_ARG, "tokens and labels must be given");
    const int64_t T = (int64_t)B * L;
    for (int64_t t = 0; t < T; ++t) {
      if (tokens[t] < 0 || tokens[t] >= f.vocab) return fail(c, MIMOSE_ERR_INVALID_ARG, "token id out of range");
      if (labels[t] < -1 || labels[t] >= f.vocab) return fail(c, MIMOSE_ERR_INVALID_ARG, "label out of range");
    }
    if (lengths)
      for (int b = 0; b < B; ++b)
        if (lengths[b] < 1 || lengths[b] > L) return fail(c, MIMOSE_ERR_INVALID_ARG, "sample length outside [1, L]");
  }
  const int64_t x = (int64_t)B * L;
  const uint64_t all = f.n_layers >= 64 ? ~(uint64_t)0 : (((uint64_t)1 << f.n_layers) - 1);
  // ---- plan (host only, on the critical path of every iteration)
  const auto t0 = std::chrono::steady_clock::now();
  uint64_t plan = 0;
  bool collect = false, generated = false, planned = false;
  int64_t predicted = 0, xq_planned = 0;
  if (c->forced_plan >= 0) {
    plan = (uint64_t)c->forced_plan & all;
  } else if (c->plan_mode == MIMOSE_PLAN_ALL) {
    plan = all;
  } else if (c->plan_mode == MIMOSE_PLAN_NONE) {
    plan = 0;
  } else if (c->planner->sheltered()) {
    plan = all;
    collect = true;
  } else {
    // a static planner sizes its one plan for the largest input it may meet (Section 3.2)
    const int64_t xq = c->plan_mode == MIMOSE_PLAN_STATIC_MAX ? (int64_t)B * f.max_seq : x;
    mimose::PlanOut po;
    bool hit = false;
    const int rc = c->planner->query(xq, &po, &hit);
    if (rc == -1) return fail(c, MIMOSE_ERR_NOT_READY, "estimator could not be fitted");
    predicted = po.predicted_peak;
    generated = !hit;
    if (rc == -2) {
      c->stats.predicted_peak_last = (uint64_t)predicted;
      return fail(c, MIMOSE_ERR_BUDGET_INFEASIBLE, "predicted peak exceeds the budget even with every layer checkpointed");
    }
    plan = po.plan;
    planned = true;
    xq_planned = xq;
  }
  const uint64_t ns = (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                          std::chrono::steady_clock::now() - t0).count();
  // ---- run
  c->dry = dry;
  Step s(c, B, L, plan, collect);
  s.lens_host = dry ? nullptr : lengths;
  float lv = 0.f;
  try {
    s.run(tokens, labels, &lv, dry || loss != nullptr);
  } catch (const OomError& e) {
    c->prof_pending.clear(); c->ev_used = 0;
    c->arena.pop_to(c->fixed_top);
    if (!dry && c->has_device) { if (c->side) (void)hipStreamSynchronize(c->side); (void)hipStreamSynchronize(c->stream); }
    // A plan of the planner's own that does not fit means the estimator under-predicted (the paper
    // keeps 0.5-1 GB free for that, Section 6.4).  The cached plan would fail again on every batch
    // of this size, so it is dropped and the key planned anew against what was missing; the
    // iteration is then issued again, as long as that yields a plan with more layers.
    if (planned && plan != all) {
      mimose::PlanOut po;
      if (c->planner->replan(xq_planned, (int64_t)(e.top + e.want - e.cap), plan, &po)) {
        c->stats.replans++;
        return do_step(c, tokens, labels, lengths, B, L, dry, loss, peak, plan_id);
      }
    }
    char buf[160];
    snprintf(buf, sizeof buf, "allocation of %llu bytes at %llu exceeds the budget of %llu bytes",
             (unsigned long long)e.want, (unsigned long long)e.top, (unsigned long long)e.cap);
    return fail(c, MIMOSE_ERR_OOM_BUDGET, buf);
  } catch (const StepError& e) {
    c->prof_pending.clear(); c->ev_used = 0;
    c->arena.pop_to(c->fixed_top);
    if (!dry && c->has_device) { if (c->side) (void)hipStreamSynchronize(c->side); (void)hipStreamSynchronize(c->stream); }
    return fail(c, e.code, e.msg);
  }
  const uint64_t pk = c->arena.high();
  c->arena.pop_to(c->fixed_top);
  c->last_e = s.e_bytes; c->last_g = s.g_bytes;
  c->last_a = s.a_bytes; c->last_b = s.b_bytes; c->last_w = s.w_bytes;
  if (collect) {
    auto& pl = *c->planner;
    for (int l = 0; l < f.n_layers; ++l) {
      pl.feed(x, MIMOSE_Q_LAYER_KEPT, l, s.a_bytes[l]);
      pl.feed(x, MIMOSE_Q_LAYER_BOUNDARY, l, s.b_bytes[l]);
      pl.feed(x, MIMOSE_Q_LAYER_BWD, l, s.w_bytes[l]);
    }
    pl.feed(x, MIMOSE_Q_EMBED, -1, s.e_bytes);
    pl.feed(x, MIMOSE_Q_HEAD, -1, s.g_bytes);
    pl.feed(x, MIMOSE_Q_FIXED, -1, c->fixed_top);
    if (!dry && (int)c->ev_layer.size() == 2 * f.n_layers)      // forward time of each layer, Section 4.1
      for (int l = 0; l < f.n_layers; ++l) {
        float ms = 0.f;
        c->last_t.resize(f.n_layers, 0);
        if (hipEventElapsedTime(&ms, c->ev_layer[2 * l], c->ev_layer[2 * l + 1]) == hipSuccess)
          c->last_t[l] = (uint64_t)std::llround((double)ms * 1e6);
        pl.feed(x, MIMOSE_Q_LAYER_TIME, l, c->last_t[l]);
      }
    pl.end_step(x);
  }
  // ---- bookkeeping
  auto& S = c->stats;
  const int n_re = __builtin_popcountll(plan);
  double uf, rf;
  flops(f, B, L, plan, &uf, &rf);
  S.steps++;
  if (!dry) c->drop_step++;                 // the next iteration draws other masks
  S.sheltered_steps = c->planner->sheltered_steps_seen();
  S.cache_hits = c->planner->hits; S.cache_misses = c->planner->misses;
  S.cache_entries = c->planner->cache_entries();
  S.planner_ns_last = ns; S.planner_ns_total += ns;
  if (generated) {                          // estimator + scheduler ran (Section 6.4's overhead accounting)
    S.plan_gen_ns_min = S.plan_gen_count ? std::min(S.plan_gen_ns_min, ns) : ns;
    S.plan_gen_ns_max = std::max(S.plan_gen_ns_max, ns);
    S.plan_gen_ns_total += ns;
    S.plan_gen_count++;
  }
  S.recomputed_layers_last = n_re; S.recomputed_layers_total += n_re;
  S.useful_flops_last = uf; S.recompute_flops_last = rf;
  S.useful_flops_total += uf; S.recompute_flops_total += rf;
  S.peak_bytes_last = pk; S.peak_bytes_max = std::max(S.peak_bytes_max, pk);
  S.predicted_peak_last = (uint64_t)predicted;
  if (loss) *loss = lv;
  if (peak) *peak = pk;
  if (plan_id) *plan_id = plan;
  return MIMOSE_OK;
}

}  // namespace

// ====================================================================== C ABI
extern "C" {

int mimose_init(const mimose_model_cfg* cfg, uint64_t mem_budget_bytes, void* arena_dev, uint64_t arena_bytes,
                void* hip_stream, mimose_ctx** out) {
  if (!cfg || !out) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "cfg and out must be given");
  *out = nullptr;
  mimose_model_cfg f = *cfg;
  if (f.n_layers < 0 || f.n_layers > 64 || f.hidden < 1 || f.n_heads < 1 || f.ffn < 1 || f.vocab < 1 || f.max_seq < 1)
    return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "bad model dimensions");
  if (f.hidden % f.n_heads) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "hidden must be a multiple of n_heads");
  const int d = f.hidden / f.n_heads;
  if (d != 32 && d != 64) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "head size must be 32 or 64");
  if (f.hidden > mk::kMaxRowWidth) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "hidden larger than 1024 is not supported");
  if (f.dtype != 0 && f.dtype != 1) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "dtype must be 0 (fp32) or 1 (bf16)");
  if (f.dtype == 1 && (f.hidden % 8 || f.ffn % 8)) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "bf16 needs hidden and ffn multiples of 8");
  for (int l = 0; l < f.n_layers; ++l)
    if (f.ffn_by_layer[l] < 0 || (f.dtype == 1 && f.ffn_by_layer[l] % 8))
      return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "ffn_by_layer: entries must be >= 0 (multiples of 8 for bf16)");
  if (f.ln_eps <= 0.f) f.ln_eps = 1e-5f;
  if (f.sheltered_steps <= 0) f.sheltered_steps = 10;
  if (f.bucket_tol_permille <= 0) f.bucket_tol_permille = 100;
  if (f.poly_order <= 0) f.poly_order = 2;
  if (f.size_quantum <= 0) f.size_quantum = 1;
  if (f.guard_bytes == 0) f.guard_bytes = 4096;
  if (arena_dev && mem_budget_bytes && arena_bytes < mem_budget_bytes)
    return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "arena smaller than the budget");
  if (arena_dev && (((uintptr_t)arena_dev) & 255)) return fail(nullptr, MIMOSE_ERR_INVALID_ARG, "arena must be 256-byte aligned");

  std::unique_ptr<mimose_ctx> c(new mimose_ctx());
  c->cfg = f;
  c->budget = mem_budget_bytes;
  c->has_device = arena_dev != nullptr;
  c->stream = (hipStream_t)hip_stream;
  std::memset(&c->stats, 0, sizeof c->stats);
  const uint64_t cap = mem_budget_bytes ? mem_budget_bytes : (arena_dev ? arena_bytes : ~(uint64_t)0 >> 1);
  c->arena.init((char*)arena_dev, cap);
  build_params(c.get());
  try {
    for (auto& p : c->params) p.w = c->arena.alloc((uint64_t)p.n * c->elt());
    for (auto& p : c->params) p.g = (float*)c->arena.alloc((uint64_t)p.n * 4);
  } catch (const OomError&) {
    return fail(nullptr, MIMOSE_ERR_OOM_BUDGET, "parameters and gradients do not fit in the budget");
  }
  c->fixed_top = c->arena.top();
  c->stats.fixed_bytes = c->fixed_top;
  c->stats.budget_bytes = mem_budget_bytes;
  c->planner.reset(new mimose::Planner(f.n_layers, mem_budget_bytes, f.sheltered_steps, f.bucket_tol_permille,
                                       f.poly_order, f.size_quantum, f.reserve_bytes, f.guard_bytes,
                                       f.cost_aware != 0));
  if (c->has_device) {
    c->ev_layer.resize(2 * (size_t)f.n_layers, nullptr);
    for (auto& e : c->ev_layer)
      if (hipEventCreate(&e) != hipSuccess) return fail(nullptr, MIMOSE_ERR_HIP, "hipEventCreate failed");
    if (hipHostMalloc((void**)&c->loss_host, 256, hipHostMallocDefault) != hipSuccess)
      return fail(nullptr, MIMOSE_ERR_HIP, "hipHostMalloc failed");
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_early, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_late, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_w2, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_stage[0], hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_stage[1], hipEventDisableTiming) != hipSuccess)
      return fail(nullptr, MIMOSE_ERR_HIP, "creating the weight-gradient stream failed");
    // gradients start at zero so that a read before the first step is defined
    mk::fill_zero(c->params.front().g, (int64_t)((char*)c->arena.alloc(0) - (char*)c->params.front().g), c->stream);
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(nullptr, MIMOSE_ERR_HIP, "device initialisation failed");
  }
  *out = c.release();
  return MIMOSE_OK;
}

int mimose_param_count(mimose_ctx* c, int32_t* n) {
  if (!c || !n) return MIMOSE_ERR_INVALID_ARG;
  *n = (int32_t)c->params.size();
  return MIMOSE_OK;
}

int mimose_param_info(mimose_ctx* c, int32_t i, const char** name, int64_t shape[4], int32_t* ndim) {
  if (!c || i < 0 || i >= (int)c->params.size()) return fail(c, MIMOSE_ERR_INVALID_ARG, "parameter index out of range");
  const Param& p = c->params[i];
  if (name) *name = p.name.c_str();
  if (shape) for (int k = 0; k < 4; ++k) shape[k] = p.shape[k];
  if (ndim) *ndim = p.ndim;
  return MIMOSE_OK;
}

int mimose_load_param(mimose_ctx* c, int32_t i, const float* host, uint64_t n) {
  if (!c || i < 0 || i >= (int)c->params.size() || !host) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad parameter index or pointer");
  if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context");
  Param& p = c->params[i];
  if ((int64_t)n != p.n) return fail(c, MIMOSE_ERR_INVALID_ARG, "element count does not match " + p.name);
  // stage through the gradient buffer of the same parameter (fp32, same element count)
  if (hipMemcpyAsync(p.g, host, n * 4, hipMemcpyHostToDevice, c->stream) != hipSuccess)
    return fail(c, MIMOSE_ERR_HIP, "copy of " + p.name + " failed");
  mk::convert_from_f32(c->cfg.dtype, p.g, p.w, p.n, c->stream);
  if (c->opt_on && p.master != (float*)p.w) mk::convert_to_f32(c->cfg.dtype, p.w, p.master, p.n, c->stream);
  mk::fill_zero(p.g, p.n * 4, c->stream);
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, MIMOSE_ERR_HIP, "load of " + p.name + " failed");
  return MIMOSE_OK;
}

int mimose_train_step(mimose_ctx* c, const int32_t* tokens, const int32_t* labels, int32_t B, int32_t L,
                      float* loss, uint64_t* peak, uint64_t* plan_id) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  return do_step(c, tokens, labels, nullptr, B, L, false, loss, peak, plan_id);
}

int mimose_train_step_padded(mimose_ctx* c, const int32_t* tokens, const int32_t* labels, const int32_t* lengths,
                             int32_t B, int32_t L, float* loss, uint64_t* peak, uint64_t* plan_id) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  if (!lengths) return fail(c, MIMOSE_ERR_INVALID_ARG, "lengths must be given");
  return do_step(c, tokens, labels, lengths, B, L, false, loss, peak, plan_id);
}

int mimose_sync_loss(mimose_ctx* c, float* loss) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context");
  if (c->stats.steps == 0) return fail(c, MIMOSE_ERR_NOT_READY, "no step has been issued yet");
  if (hipStreamSynchronize(c->stream) != hipSuccess || hipGetLastError() != hipSuccess)
    return fail(c, MIMOSE_ERR_HIP, "a queued step failed on the device");
  c->loss_pending = false;
  if (loss) *loss = *c->loss_host;
  return MIMOSE_OK;
}

int mimose_set_dropout(mimose_ctx* c, float p_hidden, float p_attn, uint64_t seed, uint64_t first_step) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  if (!(p_hidden >= 0.f) || !(p_hidden < 1.f) || !(p_attn >= 0.f) || !(p_attn < 1.f))
    return fail(c, MIMOSE_ERR_INVALID_ARG, "dropout probabilities must lie in [0, 1)");
  c->p_hidden = p_hidden;
  c->p_attn = p_attn;
  c->drop_seed = seed;
  c->drop_step = first_step;
  return MIMOSE_OK;
}

int mimose_dry_step(mimose_ctx* c, int32_t B, int32_t L, uint64_t* peak, uint64_t* plan_id) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  return do_step(c, nullptr, nullptr, nullptr, B, L, true, nullptr, peak, plan_id);
}

int mimose_get_grad(mimose_ctx* c, int32_t i, float* host, uint64_t n) {
  if (!c || i < 0 || i >= (int)c->params.size() || !host) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad parameter index or pointer");
  if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context");
  const Param& p = c->params[i];
  if ((int64_t)n != p.n) return fail(c, MIMOSE_ERR_INVALID_ARG, "element count does not match " + p.name);
  if (hipMemcpyAsync(host, p.g, n * 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess ||
      hipStreamSynchronize(c->stream) != hipSuccess)
    return fail(c, MIMOSE_ERR_HIP, "copy of gradient " + p.name + " failed");
  return MIMOSE_OK;
}

int mimose_get_param(mimose_ctx* c, int32_t i, float* host, uint64_t n) {
  if (!c || i < 0 || i >= (int)c->params.size() || !host) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad parameter index or pointer");
  if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context");
  const Param& p = c->params[i];
  if ((int64_t)n != p.n) return fail(c, MIMOSE_ERR_INVALID_ARG, "element count does not match " + p.name);
  // the values the kernels compute with: the storage-type parameter, widened
  if (c->cfg.dtype == mk::F32) {
    if (hipMemcpyAsync(host, p.w, n * 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess)
      return fail(c, MIMOSE_ERR_HIP, "copy of " + p.name + " failed");
  } else {
    // widen into scratch taken from the top of the stack, which is free between steps
    float* tmp = nullptr;
    try { tmp = (float*)c->arena.alloc(n * 4); } catch (const OomError&) {
      return fail(c, MIMOSE_ERR_OOM_BUDGET, "no room to stage " + p.name);
    }
    mk::convert_to_f32(c->cfg.dtype, p.w, tmp, p.n, c->stream);
    const hipError_t e = hipMemcpyAsync(host, tmp, n * 4, hipMemcpyDeviceToHost, c->stream);
    const hipError_t e2 = hipStreamSynchronize(c->stream);
    c->arena.pop_to(c->fixed_top);
    if (e != hipSuccess || e2 != hipSuccess) return fail(c, MIMOSE_ERR_HIP, "copy of " + p.name + " failed");
    return MIMOSE_OK;
  }
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, MIMOSE_ERR_HIP, "copy of " + p.name + " failed");
  return MIMOSE_OK;
}

int mimose_optimizer_init(mimose_ctx* c, const mimose_adamw_cfg* o) {
  if (!c || !o) return fail(c, MIMOSE_ERR_INVALID_ARG, "ctx and cfg must be given");
  if (c->opt_on) return fail(c, MIMOSE_ERR_INVALID_ARG, "the optimizer is already initialised");
  if (c->stats.steps != 0) return fail(c, MIMOSE_ERR_NOT_READY, "initialise the optimizer before the first step");
  if (!(o->lr >= 0.f) || !(o->beta1 >= 0.f && o->beta1 < 1.f) || !(o->beta2 >= 0.f && o->beta2 < 1.f) || !(o->eps >= 0.f) ||
      !(o->weight_decay >= 0.f))
    return fail(c, MIMOSE_ERR_INVALID_ARG, "hyper-parameters out of range");
  const bool narrow = c->cfg.dtype != mk::F32;
  std::vector<mk::AdamTensor> tens;
  std::vector<mk::AdamChunk> chunks;
  const uint64_t mark = c->arena.top();
  try {
    for (auto& p : c->params) {
      p.m = (float*)c->arena.alloc((uint64_t)p.n * 4);
      p.v = (float*)c->arena.alloc((uint64_t)p.n * 4);
      p.master = narrow ? (float*)c->arena.alloc((uint64_t)p.n * 4) : (float*)p.w;
    }
    for (size_t i = 0; i < c->params.size(); ++i) {
      const Param& p = c->params[i];
      mk::AdamTensor t;
      t.master = p.master; t.lowp = narrow ? p.w : nullptr; t.grad = p.g; t.m = p.m; t.v = p.v; t.n = p.n;
      t.decay = p.ndim >= 2 ? 1 : 0; t.pad = 0;
      tens.push_back(t);
      for (int64_t s0 = 0; s0 < p.n; s0 += mk::kAdamChunk) chunks.push_back(mk::AdamChunk{(int32_t)i, 0, s0});
    }
    c->opt_tensors = (mk::AdamTensor*)c->arena.alloc(tens.size() * sizeof(mk::AdamTensor));
    c->opt_chunks = (mk::AdamChunk*)c->arena.alloc(chunks.size() * sizeof(mk::AdamChunk));
  } catch (const OomError&) {
    c->arena.pop_to(mark);
    for (auto& p : c->params) p.m = p.v = p.master = nullptr;
    return fail(c, MIMOSE_ERR_OOM_BUDGET, "optimizer state does not fit in the budget");
  }
  c->opt_n_chunks = (int)chunks.size();
  if (c->has_device) {
    mk::fill_zero(c->params.front().m, (int64_t)((char*)c->opt_tensors - (char*)c->params.front().m), c->stream);
    if (narrow)
      for (auto& p : c->params) mk::convert_to_f32(c->cfg.dtype, p.w, p.master, p.n, c->stream);
    if (hipMemcpyAsync(c->opt_tensors, tens.data(), tens.size() * sizeof(mk::AdamTensor), hipMemcpyHostToDevice, c->stream) != hipSuccess ||
        hipMemcpyAsync(c->opt_chunks, chunks.data(), chunks.size() * sizeof(mk::AdamChunk), hipMemcpyHostToDevice, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess) {
      c->arena.pop_to(mark);
      for (auto& p : c->params) p.m = p.v = p.master = nullptr;
      return fail(c, MIMOSE_ERR_HIP, "optimizer initialisation failed");
    }
  }
  c->opt = *o;
  c->opt_t = 0;
  c->opt_on = true;
  c->fixed_top = c->arena.top();
  c->stats.fixed_bytes = c->fixed_top;
  return MIMOSE_OK;
}

int mimose_optimizer_step(mimose_ctx* c) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  if (!c->opt_on) return fail(c, MIMOSE_ERR_NOT_READY, "the optimizer is not initialised");
  if (!c->has_device) return fail(c, MIMOSE_ERR_NOT_READY, "host-only context");
  if (c->stats.steps == 0) return fail(c, MIMOSE_ERR_NOT_READY, "no gradients yet: run a training step first");
  c->opt_t += 1;
  mk::AdamHyper h;
  h.lr = c->opt.lr; h.beta1 = c->opt.beta1; h.beta2 = c->opt.beta2; h.eps = c->opt.eps; h.weight_decay = c->opt.weight_decay;
  h.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)c->opt.beta1, (double)c->opt_t)));
  h.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)c->opt.beta2, (double)c->opt_t)));
  mk::adamw_update(c->cfg.dtype, c->opt_tensors, c->opt_chunks, c->opt_n_chunks, h, c->stream);
  if (hipGetLastError() != hipSuccess) return fail(c, MIMOSE_ERR_HIP, "update launch failed");
  return MIMOSE_OK;
}

int mimose_force_plan(mimose_ctx* c, int64_t plan) {
  if (!c || plan < -1) return fail(c, MIMOSE_ERR_INVALID_ARG, "plan must be -1 or a bitmask");
  c->forced_plan = plan;
  return MIMOSE_OK;
}

int mimose_set_collector(mimose_ctx* c, int32_t mode) {
  if (!c || (mode != MIMOSE_COLLECTOR_MARKS && mode != MIMOSE_COLLECTOR_TWO_FORWARDS))
    return fail(c, MIMOSE_ERR_INVALID_ARG, "unknown collector mode");
  c->collector = mode;
  return MIMOSE_OK;
}

int mimose_set_plan_mode(mimose_ctx* c, int32_t mode) {
  if (!c || mode < MIMOSE_PLAN_INPUT_AWARE || mode > MIMOSE_PLAN_NONE)
    return fail(c, MIMOSE_ERR_INVALID_ARG, "unknown plan mode");
  c->plan_mode = mode;
  return MIMOSE_OK;
}

int mimose_planner_feed(mimose_ctx* c, int32_t B, int32_t L, int32_t quantity, int32_t layer, uint64_t bytes) {
  if (!c || B < 1 || L < 1 || quantity < 0 || quantity > MIMOSE_Q_LAYER_TIME) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad sample");
  if ((quantity <= 2 || quantity == MIMOSE_Q_LAYER_TIME) && (layer < 0 || layer >= c->cfg.n_layers))
    return fail(c, MIMOSE_ERR_INVALID_ARG, "layer out of range");
  c->planner->feed((int64_t)B * L, quantity, layer, bytes);
  return MIMOSE_OK;
}

int mimose_planner_end_step(mimose_ctx* c, int32_t B, int32_t L) {
  if (!c || B < 1 || L < 1) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad size");
  c->planner->end_step((int64_t)B * L);
  return MIMOSE_OK;
}

int mimose_planner_query(mimose_ctx* c, int32_t B, int32_t L, uint64_t* plan, uint64_t* predicted_peak) {
  if (!c || B < 1 || L < 1) return fail(c, MIMOSE_ERR_INVALID_ARG, "bad size");
  if (c->planner->sheltered()) return fail(c, MIMOSE_ERR_NOT_READY, "still in the sheltered phase");
  mimose::PlanOut po;
  const int rc = c->planner->query((int64_t)B * L, &po, nullptr);
  if (rc == -1) return fail(c, MIMOSE_ERR_NOT_READY, "estimator could not be fitted");
  if (plan) *plan = po.plan;
  if (predicted_peak) *predicted_peak = (uint64_t)po.predicted_peak;
  if (rc == -2) return fail(c, MIMOSE_ERR_BUDGET_INFEASIBLE, "no plan fits the budget");
  return MIMOSE_OK;
}

int mimose_profile_enable(mimose_ctx* c, int32_t on) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  c->prof_on = on != 0;
  for (auto& k : c->prof) k = mimose_ctx::ProfClass();
  return MIMOSE_OK;
}

int mimose_profile_read(mimose_ctx* c, int32_t kernel_class, uint64_t* launches, double* total_ms, double* total_work) {
  if (!c || kernel_class < 0 || kernel_class >= MIMOSE_K_COUNT) return fail(c, MIMOSE_ERR_INVALID_ARG, "kernel class out of range");
  if (launches) *launches = c->prof[kernel_class].launches;
  if (total_ms) *total_ms = c->prof[kernel_class].ms;
  if (total_work) *total_work = c->prof[kernel_class].work;
  return MIMOSE_OK;
}

int mimose_get_step_memory(mimose_ctx* c, uint64_t* fixed, uint64_t* embed, uint64_t* head, uint64_t* kept,
                           uint64_t* boundary, uint64_t* bwd) {
  if (!c) return MIMOSE_ERR_INVALID_ARG;
  if (c->last_a.size() != (size_t)c->cfg.n_layers) return fail(c, MIMOSE_ERR_NOT_READY, "no step has completed yet");
  if (fixed) *fixed = c->fixed_top;
  if (embed) *embed = c->last_e;
  if (head) *head = c->last_g;
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    if (kept) kept[l] = c->last_a[l];
    if (boundary) boundary[l] = c->last_b[l];
    if (bwd) bwd[l] = c->last_w[l];
  }
  return MIMOSE_OK;
}

int mimose_get_layer_times(mimose_ctx* c, uint64_t* ns) {
  if (!c || !ns) return MIMOSE_ERR_INVALID_ARG;
  if (c->last_t.size() != (size_t)c->cfg.n_layers) return fail(c, MIMOSE_ERR_NOT_READY, "no collecting step has completed yet");
  for (int l = 0; l < c->cfg.n_layers; ++l) ns[l] = c->last_t[l];
  return MIMOSE_OK;
}

int mimose_get_stats(mimose_ctx* c, mimose_stats* out) {
  if (!c || !out) return MIMOSE_ERR_INVALID_ARG;
  c->stats.cache_hits = c->planner->hits;
  c->stats.cache_misses = c->planner->misses;
  c->stats.cache_entries = c->planner->cache_entries();
  *out = c->stats;
  return MIMOSE_OK;
}

const char* mimose_last_error(mimose_ctx* c) { return c ? c->err.c_str() : g_init_error.c_str(); }

void mimose_destroy(mimose_ctx* c) {
  if (!c) return;
  if (c->has_device) {
    (void)hipStreamSynchronize(c->stream);
    if (c->side) (void)hipStreamSynchronize(c->side);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev_layer) if (e) (void)hipEventDestroy(e);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->ev_early) (void)hipEventDestroy(c->ev_early);
    if (c->ev_late) (void)hipEventDestroy(c->ev_late);
    if (c->ev_w2) (void)hipEventDestroy(c->ev_w2);
    if (c->side) (void)hipStreamDestroy(c->side);
    for (int k = 0; k < 2; ++k) {
      if (c->ev_stage[k]) (void)hipEventDestroy(c->ev_stage[k]);
      if (c->stage_buf[k]) (void)hipHostFree(c->stage_buf[k]);
    }
    if (c->loss_host) (void)hipHostFree(c->loss_host);
  }
  delete c;
}

}  // extern "C"
