// Launchers of the gfx950 kernels the training step is made of.
// All pointers are device pointers; every launcher only enqueues work on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mk {

enum DType : int { F32 = 0, BF16 = 1 };
enum Gelu : int { GELU_NONE = 0, GELU_ERF = 1, GELU_TANH = 2 };

constexpr int kMaxRowWidth = 1024;  // widest row the row-wise kernels accept (hidden size)

inline size_t elt_size(int dtype) { return dtype == BF16 ? 2 : 4; }

// Dropout mask descriptor, passed by value to kernels.  thr == 0: dropout off.
struct DropDesc {
  uint32_t thr = 0;      // an element is kept when its 32-bit word >= thr (thr = round(p * 2^32))
  float scale = 1.f;     // 1 / (1 - p), applied to kept elements
  uint32_t k0 = 0, k1 = 0;  // seed, low and high half
  uint32_t site = 0;     // which tensor of the model (embedding, layer l's projections ...)
  uint32_t step = 0;     // iteration number
};

struct GemmArgs {
  const void* A; int64_t lda; bool a_kmajor;
  const void* B; int64_t ldb; bool b_kmajor;
  void* C; int64_t ldc; bool c_f32;
  int M, N, K;
  const void* bias = nullptr;      // [N], storage dtype
  const void* resid = nullptr;     // [M, ldr], storage dtype
  int64_t ldr = 0;
  void* gelu_out = nullptr;        // [M, ldc], storage dtype
  int gelu = GELU_NONE;
  float* a_rowsum = nullptr;       // [M] fp32: sum_k A(m,k) (bias gradient of a weight-gradient product)
  // A k-major with K not a multiple of 8: its columns [K, K rounded up to 8) exist (lda covers
  // them) and hold zeros, so a kernel that moves whole 16-byte chunks may read them
  bool a_tail_zero = false;
  void* workspace = nullptr;       // optional scratch of gemm_workspace_bytes(M, N) for split reductions
  size_t workspace_bytes = 0;
  // optional, both or neither: recorded by the product kernel's own start and end (not by markers
  // around the launch), for per-kernel timing; a split product ends with its reduction kernel
  hipEvent_t time_start = nullptr, time_stop = nullptr;
};

// scratch that lets a bf16 product with fp32 output cut its reduction in parts (0: never splits);
// a function of the output shape alone
size_t gemm_workspace_bytes(int M, int N);
// scratch that lets a data-gradient product with a very long reduction and few output tiles (the
// vocabulary-long one of the head: A k-major, B m-major, no epilogue) cut its reduction in parts:
// a function of the column count alone, so that it is a constant of the model
size_t gemm_long_k_workspace_bytes(int N);

// returns false when the arguments violate the kernel's alignment assumptions
bool gemm(int dtype, const GemmArgs& g, hipStream_t st);

// x_f32: in a bf16 configuration the input rows are fp32 (an unrounded residual sum)
void layernorm_fwd(int dtype, const void* x, bool x_f32, const void* gamma, const void* beta,
                   void* y, int T, int H, float eps, hipStream_t st);
// partial: fp32 scratch of partial_rows(T) * 2 * H elements
// dx = LayerNorm backward (+ add when given); dx may alias dy when they have the same type;
// dy_f32 / x_f32: in a bf16 configuration those inputs are fp32
void layernorm_bwd(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32,
                   const void* gamma, void* dx, const void* add, float* dgamma, float* dbeta,
                   float* partial, int T, int H, float eps, hipStream_t st);
// the two halves of layernorm_bwd: dx and the per-chunk partial sums; then dgamma, dbeta from them
void layernorm_bwd_rows(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32, const void* gamma, void* dx,
                        const void* add, float* partial, int T, int H, float eps, hipStream_t st);
void layernorm_bwd_reduce(const float* partial, float* dgamma, float* dbeta, int T, int H, hipStream_t st);
int partial_rows(int T);
// layernorm_bwd with the partial sums in a fixed device array of the library (no allocation, no
// workspace argument).  Returns 0, -1 when partial_rows(T) * 2 * H exceeds
// kStaticPartialFloats, -2 when the array's address cannot be obtained.  One array per device,
// shared by every call on that device.
constexpr size_t kStaticPartialFloats = (size_t)2 << 20;   // 8 MiB
int layernorm_bwd_static(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32, const void* gamma,
                         void* dx, const void* add, float* dgamma, float* dbeta, int T, int H, float eps,
                         hipStream_t st);
void gelu_bwd(int dtype, void* d, const void* pre, int64_t n, int tanh_form, hipStream_t st);
// lens (optional, device, [B]): real tokens per sample of a padded batch; keys from lens[b] on get
// no weight.  nullptr: every sample fills its row.  drop: dropout of the probabilities (the
// softmax normaliser counts all of them; ctx = (mask * scale * P) V).
void attention_fwd(int dtype, const void* qkv, void* ctx, float* lse, const int32_t* lens, int B, int L, int nh, int d,
                   int causal, const DropDesc& drop, hipStream_t st);
void attention_bwd(int dtype, const void* qkv, const void* ctx, const void* dctx, const float* lse,
                   float* delta, void* dqkv, const int32_t* lens, int B, int L, int nh, int d, int causal,
                   const DropDesc& drop, hipStream_t st);
void softmax_xent(int dtype, void* logits, int64_t ld, const int32_t* labels, float* row_loss,
                  float* loss, int T, int V, int n_valid, hipStream_t st);
void embed_fwd(int dtype, const int32_t* ids, const void* tok, const void* pos, const void* gamma,
               const void* beta, void* sum_out, void* y, int B, int L, int H, float eps, int has_ln,
               hipStream_t st);
void embed_bwd(int dtype, const void* d, const int32_t* ids, const int32_t* order,
               const int32_t* seg, int n_seg, float* dtok, float* dpos, int B, int L, int H,
               int max_seq, hipStream_t st);
// dst (storage dtype) = round(src fp32)
void convert_from_f32(int dtype, const float* src, void* dst, int64_t n, hipStream_t st);
void fill_zero(void* p, int64_t bytes, hipStream_t st);

// AdamW over a list of tensors in one launch.  Device-resident tables, one entry per tensor
// (master fp32 values, optional low-precision copy, gradient, first and second moment, element
// count, whether weight decay applies) and one per chunk of kAdamChunk elements (tensor, start).
constexpr int kAdamChunk = 16384;
struct AdamTensor {
  float* master; void* lowp; const float* grad; float* m; float* v; int64_t n; int32_t decay; int32_t pad;
};
struct AdamChunk { int32_t tensor; int32_t pad; int64_t start; };
struct AdamHyper { float lr, beta1, beta2, eps, weight_decay, inv_c1, inv_c2; };   // inv_c = 1 / (1 - beta^t)
void adamw_update(int lowp_dtype, const AdamTensor* tensors, const AdamChunk* chunks, int n_chunks, AdamHyper h,
                  hipStream_t st);
// dst[n] = (resid ? resid[n] : 0) + mask * d.scale * src[n] with the mask of d (element i: word i % 4
// of block i / 4).  dst and src have the storage type, or fp32 when io_f32; resid has the storage
// type; dst may be src.
void dropout_apply(int dtype, void* dst, const void* src, bool io_f32, const void* resid, int64_t n, const DropDesc& d,
                   hipStream_t st);
// dst fp32 = src (storage dtype)
void convert_to_f32(int dtype, const void* src, float* dst, int64_t n, hipStream_t st);

}  // namespace mk
