/*
 * libmimose - input-aware activation checkpointing for transformer training on
 * one MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * The library runs the checkpointed training iteration of Mimose
 * (arXiv 2209.02478): forward keeping activations, loss, backward consuming
 * them (Section 2.1), with layer-granular checkpointing (Section 1, Section 5:
 * a dropped layer keeps only its boundary tensor and is replayed in backward),
 * driven by the paper's planner: sheltered / responsive phases (Section 4.1),
 * a per-layer quadratic memory estimator (Section 4.3), the greedy bucketed
 * scheduler (Section 4.4, Algorithm 1) and a plan cache keyed by input size
 * (Section 5).
 *
 * Conventions
 *   - every function returns MIMOSE_OK (0) or a negative MIMOSE_ERR_* code;
 *     mimose_last_error() gives a text for the last failure on that context;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory on the current device; the library never frees, resizes or
 *     retains caller memory beyond what is stated per function;
 *   - all device memory the library uses is carved out of the arena passed to
 *     mimose_init; all device work is enqueued on the stream passed there;
 *   - a failed call leaves the context usable.
 */
#ifndef MIMOSE_H
#define MIMOSE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIMOSE_OK 0
#define MIMOSE_ERR_INVALID_ARG (-1)
#define MIMOSE_ERR_OOM_BUDGET (-2)        /* an allocation would exceed the memory budget   */
#define MIMOSE_ERR_BUDGET_INFEASIBLE (-3) /* even the all-checkpointed plan exceeds budget  */
#define MIMOSE_ERR_HIP (-4)
#define MIMOSE_ERR_NOT_READY (-5)

typedef struct mimose_ctx mimose_ctx; /* opaque, owned by the library */

/* Plain data, caller-owned, copied by mimose_init. */
typedef struct {
  int32_t n_layers, hidden, n_heads, ffn, vocab, max_seq;
  int32_t dtype;     /* 0: fp32 storage and arithmetic; 1: bf16 storage, fp32 accumulation */
  int32_t causal;    /* 1: causal attention mask                                          */
  int32_t pre_ln;    /* 0: post-LN blocks (BERT-shaped); 1: pre-LN blocks + final LN       */
  int32_t gelu_tanh; /* 0: erf GELU; 1: tanh approximation                                 */
  int32_t head;      /* 1: dense+GELU+LN transform, tied decoder + bias; 0: tied decoder   */
  float ln_eps;
  /* planner; zero selects the paper's value given in brackets */
  int32_t sheltered_steps;     /* [10]  iterations of data collection, Section 6.4          */
  int32_t bucket_tol_permille; /* [100] bucket similarity, Section 4.4                       */
  int32_t poly_order;          /* [2]   estimator order, Section 6.5                         */
  int32_t size_quantum;        /* [1]   plan-cache key granularity, Section 5                */
  uint64_t reserve_bytes;      /* kept free below the budget (Section 6.4 keeps 0.5-1 GB)    */
  uint64_t guard_bytes;        /* added to every predicted component; 0 selects 4096         */
  /* stacks whose layers differ (the stages of Section 4.4): width of layer l's feed-forward
   * block; 0 = ffn.  Entries from n_layers on are ignored. */
  int32_t ffn_by_layer[64];
  /* 1: inside the bucket Algorithm 1 selects, take the earliest layer whose estimated forward
   * time (collected in the sheltered phase, Section 4.1) is within bucket_tol_permille of the
   * bucket's cheapest remaining layer, instead of simply the earliest.  Equal times, or no
   * collected times (host-only contexts that were fed none), give Algorithm 1. */
  int32_t cost_aware;
  int32_t reserved_;           /* keep zero */
} mimose_model_cfg;

typedef struct {
  uint64_t steps, sheltered_steps;
  uint64_t cache_hits, cache_misses, cache_entries;
  uint64_t planner_ns_last, planner_ns_total;
  uint64_t recomputed_layers_last, recomputed_layers_total;
  double useful_flops_last, recompute_flops_last;
  double useful_flops_total, recompute_flops_total;
  uint64_t peak_bytes_last, peak_bytes_max, predicted_peak_last;
  uint64_t fixed_bytes, budget_bytes;
  /* estimator + scheduler time of the iterations that had to generate a plan (cache misses),
   * for the overhead accounting of Section 6.4; min is 0 until the first miss */
  uint64_t plan_gen_count, plan_gen_ns_total, plan_gen_ns_min, plan_gen_ns_max;
  /* iterations whose cached plan did not fit (the estimator under-predicted): the plan was
   * dropped, the key planned again against the missing bytes, the iteration issued again */
  uint64_t replans;
} mimose_stats;

/* quantities of the collector's sample table (Section 4.2), see mimose_planner_feed */
#define MIMOSE_Q_LAYER_KEPT 0    /* a_l: bytes layer l holds from forward to backward       */
#define MIMOSE_Q_LAYER_BOUNDARY 1/* b_l: bytes it holds when checkpointed (its output)      */
#define MIMOSE_Q_LAYER_BWD 2     /* w_l: transient bytes of its backward                    */
#define MIMOSE_Q_EMBED 3         /* e: bytes of the embedding stage held all step           */
#define MIMOSE_Q_HEAD 4          /* g: transient bytes of head forward + backward           */
#define MIMOSE_Q_FIXED 5         /* F: parameters, gradients, persistent scratch            */
#define MIMOSE_Q_LAYER_TIME 6    /* t_l: forward time of layer l in ns (Section 4.1)        */

/*
 * Create a context (Section 4.1: the planner wraps the training iteration).
 *   cfg              model and planner configuration (host, copied)
 *   mem_budget_bytes memory budget M of Algorithm 1, covering everything the
 *                    library keeps on the device; 0 = unlimited (calibration)
 *   arena_dev        device buffer the library sub-allocates from; stays owned by
 *                    the caller and must outlive the context.  NULL creates a
 *                    host-only context: planner calls and mimose_dry_step work,
 *                    mimose_train_step returns MIMOSE_ERR_NOT_READY.
 *   arena_bytes      its size; must be >= mem_budget_bytes when both are non-zero
 *   hip_stream       hipStream_t (as void*) all work is enqueued on; NULL = default
 * Errors: INVALID_ARG (bad shapes, hidden % n_heads, head_dim not 32/64,
 * n_layers > 64), OOM_BUDGET (parameters and gradients do not fit).
 */
int mimose_init(const mimose_model_cfg* cfg, uint64_t mem_budget_bytes, void* arena_dev,
                uint64_t arena_bytes, void* hip_stream, mimose_ctx** out);

/* Named parameter tensors.  name stays valid for the context's life; shape has ndim entries. */
int mimose_param_count(mimose_ctx* ctx, int32_t* n);
int mimose_param_info(mimose_ctx* ctx, int32_t i, const char** name, int64_t shape[4], int32_t* ndim);
/* Copy parameter i from host fp32 (row-major); the library rounds to its storage type
 * (round to nearest even).  Synchronous. */
int mimose_load_param(mimose_ctx* ctx, int32_t i, const float* host_fp32, uint64_t n_elems);

/*
 * One training iteration on a mini-batch of B sequences of exactly L tokens
 * (Section 2.1; input size x = B*L, Section 3.1).  Chooses the plan (sheltered:
 * all layers; responsive: cache or Algorithm 1), runs forward / loss / backward
 * with recomputation of dropped layers, and waits for completion.
 *   tokens_host  [B,L] row-major ids in [0,vocab); borrowed for the call
 *   labels_host  [B,L], -1 = position not scored; borrowed for the call
 *   loss         mean cross-entropy over scored positions.  NULL: the iteration is only
 *                queued on the context's stream and the call returns without waiting (the
 *                planner is on the critical path of every iteration, Section 5; the device need
 *                not idle while the host plans and queues the next one); plan, peak and errors of
 *                allocation are known at once, the loss through mimose_sync_loss.  Iterations of
 *                the sheltered phase and profiled ones always wait.
 *   peak_bytes   true high-water mark of device memory in this step
 *   plan_id      bitmask, bit l set = layer l was dropped and recomputed
 * A planner-made plan that turns out not to fit (the estimator under-predicted) is dropped from
 * the cache, the size is planned again against the bytes that were missing and the iteration is
 * issued once more, as long as that selects more layers (stats.replans counts these).
 * Errors: INVALID_ARG, OOM_BUDGET (the step is abandoned, the arena is reset),
 * BUDGET_INFEASIBLE, HIP, NOT_READY (host-only context).
 */
int mimose_train_step(mimose_ctx* ctx, const int32_t* tokens_host, const int32_t* labels_host,
                      int32_t B, int32_t L, float* loss, uint64_t* peak_bytes, uint64_t* plan_id);

/* Waits for every iteration queued so far; loss (may be NULL) receives the loss of the last one.
 * Errors: NOT_READY before the first iteration or on a host-only context, HIP. */
int mimose_sync_loss(mimose_ctx* ctx, float* loss);

/*
 * The same iteration on a batch whose samples were padded to the longest one
 * (Section 3.1: the input tensor of a batch has the size of its longest
 * sample; the planner's x stays B*L, padding included).
 *   lengths_host [B] real tokens of each sample, 1 <= lengths[b] <= L; borrowed.
 * Positions from lengths[b] on are padding: no query gives them attention
 * weight, their labels are ignored, and no gradient reaches them; their token
 * ids must still lie in [0,vocab).  Memory use, plan and error behaviour are
 * those of mimose_train_step at the same B and L.
 * Errors: as mimose_train_step, plus INVALID_ARG for a length outside [1, L].
 */
int mimose_train_step_padded(mimose_ctx* ctx, const int32_t* tokens_host, const int32_t* labels_host,
                             const int32_t* lengths_host, int32_t B, int32_t L, float* loss,
                             uint64_t* peak_bytes, uint64_t* plan_id);

/*
 * Dropout, as the fine-tuning tasks of Section 6.1 train with it.  p_hidden acts on the
 * embedding output, on the attention block's output projection and on the feed-forward block's
 * output (each before its residual sum); kept elements are scaled by 1/(1-p).  The masks come
 * from a counter-based generator (Philox4x32, ten rounds): element i of the tensor at site s in
 * iteration t is kept when word i%4 of the block with counter (i/4 low, i/4 high, s, t) and key
 * (seed low, seed high) is >= round(p * 2^32).  Sites: 0 the embedding output; layer l:
 * 4(l+1)+1 the attention output projection, 4(l+1)+2 the feed-forward output.  A layer that is
 * checkpointed and run again before its backward therefore meets the masks of its first run
 * (Section 2.2: recomputation must reproduce the dropped tensors), and nothing is stored.
 * first_step numbers the next iteration; every completed mimose_train_step adds one.
 * p_attn acts on the attention probabilities of every layer (site 4(l+1); element number
 * ((b*heads + head)*L + query) * 4*ceil(L/4) + key, so that four neighbouring keys of a query
 * share a block): the softmax normaliser counts every probability, the dropped ones leave the
 * product with V.
 * Zero probabilities (the initial state) switch dropout off.  Errors: INVALID_ARG.
 */
int mimose_set_dropout(mimose_ctx* ctx, float p_hidden, float p_attn, uint64_t seed,
                       uint64_t first_step);

/* Same planning, allocation and bookkeeping as mimose_train_step but no device work:
 * reports the peak the step would reach.  Works on host-only contexts. */
int mimose_dry_step(mimose_ctx* ctx, int32_t B, int32_t L, uint64_t* peak_bytes, uint64_t* plan_id);

/* Gradient of parameter i from the last completed step, as fp32 to host. Synchronous. */
int mimose_get_grad(mimose_ctx* ctx, int32_t i, float* host_fp32, uint64_t n_elems);

/* Parameter i as the kernels use it (storage type widened to fp32), to host.  Synchronous. */
int mimose_get_param(mimose_ctx* ctx, int32_t i, float* host_fp32, uint64_t n_elems);

/* Parameter update that ends a training iteration (Section 2.1); its state counts towards the
 * input-independent memory of Section 3.1.  The paper names no optimizer: this is Adam with
 * decoupled weight decay, p -= lr * (m_hat / (sqrt(v_hat) + eps) + weight_decay * p), the decay
 * applied to tensors of two or more dimensions only.  State comes out of the arena's persistent
 * region: two fp32 moments per element, plus an fp32 master copy when dtype is bf16 (the bf16
 * parameter is then the master rounded to nearest-even after every update).
 * mimose_optimizer_init: once, before the first step (NOT_READY after), also on host-only
 * contexts (bookkeeping only); OOM_BUDGET if the state does not fit, the context stays usable.
 * mimose_optimizer_step: one update from the gradients of the last completed step, enqueued on
 * the context's stream (asynchronous); NOT_READY without a preceding step or on host-only
 * contexts.  Parameters loaded afterwards with mimose_load_param refresh the master copy. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
} mimose_adamw_cfg;
int mimose_optimizer_init(mimose_ctx* ctx, const mimose_adamw_cfg* cfg);
int mimose_optimizer_step(mimose_ctx* ctx);

/* Test hook: plan >= 0 forces that bitmask on every following step (0 = keep everything)
 * and suspends the phase logic; -1 returns control to the planner. */
int mimose_force_plan(mimose_ctx* ctx, int64_t plan_or_minus1);

/* Planning policy of the responsive phase.  The sheltered phase (Section 4.1) is the same for
 * modes 0 and 1; modes 2 and 3 never consult the planner and collect nothing.
 *   MIMOSE_PLAN_INPUT_AWARE  plan for the size of the batch at hand (Sections 4.1, 4.4): default
 *   MIMOSE_PLAN_STATIC_MAX   one plan, made for the largest admissible input (B * max_seq tokens
 *                            at the batch size of the step) and applied to every batch: what a
 *                            static planner does when input sizes vary (Section 3.2)
 *   MIMOSE_PLAN_ALL          every layer checkpointed: the lower memory limit of Section 6.2
 *   MIMOSE_PLAN_NONE         nothing checkpointed: the upper memory limit of Section 6.2
 * A plan forced with mimose_force_plan takes precedence over the mode.  Unknown mode: INVALID_ARG. */
#define MIMOSE_PLAN_INPUT_AWARE 0
#define MIMOSE_PLAN_STATIC_MAX 1
#define MIMOSE_PLAN_ALL 2
#define MIMOSE_PLAN_NONE 3
int mimose_set_plan_mode(mimose_ctx* ctx, int32_t mode);

/* How a sheltered iteration collects a block's memory (Section 4.2).
 *   MIMOSE_COLLECTOR_MARKS         one forward per block: the library owns the allocator, so it
 *                                  reads the stack's marks before and after the block drops its
 *                                  internals (default; same samples, no extra work)
 *   MIMOSE_COLLECTOR_TWO_FORWARDS  the paper's shuttling forward to the letter: every block's
 *                                  forward runs twice, first as normal (measured, then discarded
 *                                  with its output), then keeping only the output.  Same samples,
 *                                  same results bit for bit; costs one more forward pass per
 *                                  sheltered iteration (the collector column of the paper's
 *                                  overhead table).
 * Errors: INVALID_ARG for an unknown mode. */
#define MIMOSE_COLLECTOR_MARKS 0
#define MIMOSE_COLLECTOR_TWO_FORWARDS 1
int mimose_set_collector(mimose_ctx* ctx, int32_t mode);

/* Host-only planner access (Section 4.2-4.4): inject a collected sample / ask for a plan. */
int mimose_planner_feed(mimose_ctx* ctx, int32_t B, int32_t L, int32_t quantity, int32_t layer,
                        uint64_t bytes);
/* Marks the end of one sheltered iteration at this input size (phase accounting). */
int mimose_planner_end_step(mimose_ctx* ctx, int32_t B, int32_t L);
/* Plan for input size B*L from the fitted estimator (fits on first use); counts as a cache
 * lookup.  Returns NOT_READY while the planner is still in the sheltered phase and
 * BUDGET_INFEASIBLE (plan = all layers, predicted_peak filled) if no plan fits. */
int mimose_planner_query(mimose_ctx* ctx, int32_t B, int32_t L, uint64_t* plan,
                         uint64_t* predicted_peak);

/* Per-kernel-class timing with events on the work stream (measurement aid; adds two event
 * records per launch while enabled).  Enabling or disabling clears the totals.  work is
 * algorithmic: floating-point operations for GEMM and attention, bytes for the others. */
#define MIMOSE_K_GEMM 0
#define MIMOSE_K_ATTN_FWD 1
#define MIMOSE_K_ATTN_BWD 2
#define MIMOSE_K_LN_FWD 3
#define MIMOSE_K_LN_BWD 4
#define MIMOSE_K_GELU_BWD 5
#define MIMOSE_K_XENT 6
#define MIMOSE_K_EMBED_FWD 7
#define MIMOSE_K_COUNT 8
int mimose_profile_enable(mimose_ctx* ctx, int32_t on);
int mimose_profile_read(mimose_ctx* ctx, int32_t kernel_class, uint64_t* launches, double* total_ms,
                        double* total_work);

/* What the collector measured in the last completed step (Section 4.2), in bytes: fixed F,
 * embedding stage e, head transient g, and per layer (arrays of n_layers, may be NULL) the
 * bytes kept (a_l), kept when checkpointed (b_l) and the backward transient (w_l). */
int mimose_get_step_memory(mimose_ctx* ctx, uint64_t* fixed, uint64_t* embed, uint64_t* head,
                           uint64_t* kept, uint64_t* boundary, uint64_t* bwd);

/* Forward time of each layer in the last sheltered (collecting) step, in ns, as fed to the
 * estimator (Section 4.1).  ns: host array of n_layers.  NOT_READY before the first such step. */
int mimose_get_layer_times(mimose_ctx* ctx, uint64_t* ns);

int mimose_get_stats(mimose_ctx* ctx, mimose_stats* out);
const char* mimose_last_error(mimose_ctx* ctx); /* ctx may be NULL: last init error */
void mimose_destroy(mimose_ctx* ctx);

/* ------------------------------------------------------------------------
 * Kernel-level entry points (device pointers, current device, given stream).
 * These are the kernels the training step is made of, exposed for parity tests
 * and per-kernel measurement.  dtype as in mimose_model_cfg.  No allocation.
 * They have no counterpart in the paper, which runs stock library kernels under
 * its planner and describes none of its own: what each computes is the model's
 * standard operation named in its comment.
 * ---------------------------------------------------------------------- */

/* C[M,N] = sum_k A(m,k) B(n,k) (+ bias[n]) (+ resid[m,n]); optional GELU: C receives the
 * pre-activation, gelu_out the activation.  a_kmajor: A(m,k) = A[m*lda+k], else A[k*lda+m];
 * likewise B with ldb.  c_f32: C is fp32 regardless of dtype (weight gradients).
 * a_rowsum (optional, fp32[M]) receives sum_k A(m,k) (the bias gradient of a weight-gradient
 * product).  gelu: 0 none, 1 erf, 2 tanh.  bf16: lda, ldb must be multiples of 8 and A, B
 * 16-byte aligned, otherwise INVALID_ARG.  workspace: optional device scratch, see
 * mimose_op_gemm_workspace_bytes. */
int mimose_op_gemm(int32_t dtype, const void* A, int64_t lda, int32_t a_kmajor, const void* B,
                   int64_t ldb, int32_t b_kmajor, void* C, int64_t ldc, int32_t c_f32, int32_t M,
                   int32_t N, int32_t K, const void* bias, const void* resid, int64_t ldr,
                   void* gelu_out, int32_t gelu, float* a_rowsum, void* workspace,
                   uint64_t workspace_bytes, void* stream);
/* Scratch that lets a bf16 product with fp32 output and few output tiles cut its reduction
 * into parts that are summed in a fixed order (a function of M and N only; 0 = never needed).
 * Passing NULL workspace to mimose_op_gemm is always allowed. */
uint64_t mimose_op_gemm_workspace_bytes(int32_t M, int32_t N);
/* Scratch for the products with a very long reduction (K >= 8192) behind a k-major A and an
 * m-major B, no epilogue, few output tiles (the head's data gradient, reduced over the
 * vocabulary): with it they cut their reduction in parts on the large tiles.  A function of N
 * alone.  Passing less, or NULL, to mimose_op_gemm is always allowed. */
uint64_t mimose_op_gemm_long_k_workspace_bytes(int32_t N);
/* y = LayerNorm(x) * gamma + beta over rows of length H <= 1024.  x_f32: with dtype bf16 the
 * input rows are fp32 (an unrounded residual sum); ignored for dtype fp32. */
int mimose_op_layernorm_fwd(int32_t dtype, const void* x, int32_t x_f32, const void* gamma,
                            const void* beta, void* y, int32_t T, int32_t H, float eps, void* stream);
/* dx = LayerNorm backward of dy at x (+ add[T,H] when not NULL); dgamma, dbeta fp32[H]; partial:
 * fp32 scratch of mimose_op_partial_rows(T)*2*H elements.  dy_f32 / x_f32: with dtype bf16 those
 * inputs are fp32.  dx may alias dy when both have the storage type. */
int mimose_op_layernorm_bwd(int32_t dtype, const void* dy, int32_t dy_f32, const void* x,
                            int32_t x_f32, const void* gamma, void* dx, const void* add,
                            float* dgamma, float* dbeta, float* partial, int32_t T, int32_t H,
                            float eps, void* stream);
int32_t mimose_op_partial_rows(int32_t T);
/* mimose_op_layernorm_bwd for callers that cannot allocate or bring a workspace (code under HIP
 * graph capture, serving loops, harnesses that forbid hipMalloc): same kernels, same results, the
 * partial sums live in a fixed device array inside the library (8 MiB per device, held until the
 * process ends).  It allocates nothing and calls no allocating routine.  Sizes with
 * mimose_op_partial_rows(T) * 2 * H > mimose_op_layernorm_bwd_noalloc_max_floats() are refused
 * with INVALID_ARG (mimose_last_error(NULL) says by how much); HIP if the array's address
 * cannot be obtained on the current device.  Nothing in the array needs clearing between calls
 * (every partial row read is written first), but all calls on one device share it: two calls
 * that overlap on the same device (different streams, no ordering between them) race. */
int mimose_op_layernorm_bwd_noalloc(int32_t dtype, const void* dy, int32_t dy_f32, const void* x,
                                    int32_t x_f32, const void* gamma, void* dx, const void* add,
                                    float* dgamma, float* dbeta, int32_t T, int32_t H, float eps,
                                    void* stream);
uint64_t mimose_op_layernorm_bwd_noalloc_max_floats(void);
/* d[n] (in place) *= gelu'(pre[n]). */
int mimose_op_gelu_bwd(int32_t dtype, void* d, const void* pre, int64_t n, int32_t tanh_form,
                       void* stream);
/* qkv [B*L, 3*H] (q | k | v, heads contiguous inside each) -> ctx [B*L, H], lse fp32 [B, h, L].
 * head_dim must be 32 or 64.  lengths: NULL, or device int32 [B] with 1 <= lengths[b] <= L (not
 * checked: the caller guarantees it): keys of sample b from lengths[b] on are padding and get
 * no weight.  p_drop > 0: dropout of the probabilities with the masks mimose_set_dropout
 * describes for (seed, site, step). */
int mimose_op_attention_fwd(int32_t dtype, const void* qkv, void* ctx, float* lse,
                            const int32_t* lengths, int32_t B, int32_t L, int32_t n_heads,
                            int32_t head_dim, int32_t causal, float p_drop, uint64_t seed,
                            uint32_t site, uint32_t step, void* stream);
/* dqkv from qkv, ctx, dctx, lse; delta: fp32 scratch [B, h, L]; lengths and dropout as in the
 * forward (dK, dV of padded keys are written as zeros). */
int mimose_op_attention_bwd(int32_t dtype, const void* qkv, const void* ctx, const void* dctx,
                            const float* lse, float* delta, void* dqkv, const int32_t* lengths,
                            int32_t B, int32_t L, int32_t n_heads, int32_t head_dim,
                            int32_t causal, float p_drop, uint64_t seed, uint32_t site,
                            uint32_t step, void* stream);
/* dst[n] = (resid ? resid[n] : 0) + mask * src[n] / (1-p) with the mask mimose_set_dropout
 * describes for (seed, site, step).  dst, src: storage type, or fp32 when io_f32; resid: storage
 * type or NULL; dst may be src. */
int mimose_op_dropout(int32_t dtype, void* dst, const void* src, int32_t io_f32, const void* resid,
                      int64_t n, float p, uint64_t seed, uint32_t site, uint32_t step,
                      void* stream);
/* logits [T, ld] (first V columns valid) -> in place d loss / d logits (columns >= V zeroed);
 * row_loss fp32[T]; loss: device fp32 scalar = sum(row_loss)/n_valid. */
int mimose_op_softmax_xent(int32_t dtype, void* logits, int64_t ld, const int32_t* labels,
                           float* row_loss, float* loss, int32_t T, int32_t V, int32_t n_valid,
                           void* stream);
/* sum_out (may be NULL when has_ln = 0) = tok_emb[id] + pos_emb[pos]; y = LN(sum) or sum. */
int mimose_op_embed_fwd(int32_t dtype, const int32_t* ids, const void* tok_emb, const void* pos_emb,
                        const void* gamma, const void* beta, void* sum_out, void* y, int32_t B,
                        int32_t L, int32_t H, float eps, int32_t has_ln, void* stream);
/* Deterministic scatter-add of d[T,H] into dtok (fp32 [V,H], accumulated onto) and dpos
 * (fp32 [max_seq,H], overwritten; rows >= L cleared).  order: token positions sorted by id
 * (ties by position); seg: start offsets of each distinct id's run in order (n_seg+1 entries). */
int mimose_op_embed_bwd(int32_t dtype, const void* d, const int32_t* ids, const int32_t* order,
                        const int32_t* seg, int32_t n_seg, float* dtok, float* dpos, int32_t B,
                        int32_t L, int32_t H, int32_t max_seq, void* stream);

#ifdef __cplusplus
}
#endif
#endif
