// C ABI of the kernel-level entry points: argument checks, then the launcher.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "../../include/mimose.h"
#include "kernels.h"

// sets what mimose_last_error(NULL) returns on this thread (mimose.cpp)
void mimose_set_thread_error(const char* msg);

namespace {
inline bool bad_dtype(int d) { return d != 0 && d != 1; }
inline int done() { return hipGetLastError() == hipSuccess ? MIMOSE_OK : MIMOSE_ERR_HIP; }
inline bool bad_head(int d) { return d != 32 && d != 64; }
}  // namespace

extern "C" {

int mimose_op_gemm(int32_t dtype, const void* A, int64_t lda, int32_t a_kmajor, const void* B, int64_t ldb,
                   int32_t b_kmajor, void* C, int64_t ldc, int32_t c_f32, int32_t M, int32_t N, int32_t K,
                   const void* bias, const void* resid, int64_t ldr, void* gelu_out, int32_t gelu,
                   float* a_rowsum, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (bad_dtype(dtype) || !A || !B || !C || M < 0 || N < 0 || K < 0 || gelu < 0 || gelu > 2) return MIMOSE_ERR_INVALID_ARG;
  if (lda < (a_kmajor ? K : M) || ldb < (b_kmajor ? K : N) || ldc < N || (resid && ldr < N)) return MIMOSE_ERR_INVALID_ARG;
  mk::GemmArgs g{A, lda, a_kmajor != 0, B, ldb, b_kmajor != 0, C, ldc, c_f32 != 0, M, N, K};
  g.bias = bias; g.resid = resid; g.ldr = ldr; g.gelu_out = gelu_out; g.gelu = gelu; g.a_rowsum = a_rowsum;
  g.workspace = workspace; g.workspace_bytes = workspace_bytes;
  if (!mk::gemm(dtype, g, (hipStream_t)stream)) return MIMOSE_ERR_INVALID_ARG;
  return done();
}

uint64_t mimose_op_gemm_workspace_bytes(int32_t M, int32_t N) {
  return M > 0 && N > 0 ? mk::gemm_workspace_bytes(M, N) : 0;
}

uint64_t mimose_op_gemm_long_k_workspace_bytes(int32_t N) { return N > 0 ? mk::gemm_long_k_workspace_bytes(N) : 0; }

int mimose_op_layernorm_fwd(int32_t dtype, const void* x, int32_t x_f32, const void* gamma, const void* beta, void* y,
                            int32_t T, int32_t H, float eps, void* stream) {
  if (bad_dtype(dtype) || !x || !gamma || !beta || !y || T < 0 || H < 1 || H > mk::kMaxRowWidth) return MIMOSE_ERR_INVALID_ARG;
  mk::layernorm_fwd(dtype, x, x_f32 != 0, gamma, beta, y, T, H, eps, (hipStream_t)stream);
  return done();
}

int mimose_op_layernorm_bwd(int32_t dtype, const void* dy, int32_t dy_f32, const void* x, int32_t x_f32,
                            const void* gamma, void* dx, const void* add, float* dgamma, float* dbeta, float* partial,
                            int32_t T, int32_t H, float eps, void* stream) {
  if (bad_dtype(dtype) || !dy || !x || !gamma || !dx || !dgamma || !dbeta || !partial || T < 0 || H < 1 ||
      H > mk::kMaxRowWidth || add == dx || (dx == dy && dtype == 1 && dy_f32))
    return MIMOSE_ERR_INVALID_ARG;
  mk::layernorm_bwd(dtype, dy, dy_f32 != 0, x, x_f32 != 0, gamma, dx, add, dgamma, dbeta, partial, T, H, eps,
                    (hipStream_t)stream);
  return done();
}

int32_t mimose_op_partial_rows(int32_t T) { return mk::partial_rows(T); }

int mimose_op_layernorm_bwd_noalloc(int32_t dtype, const void* dy, int32_t dy_f32, const void* x, int32_t x_f32,
                                    const void* gamma, void* dx, const void* add, float* dgamma, float* dbeta,
                                    int32_t T, int32_t H, float eps, void* stream) {
  if (bad_dtype(dtype) || !dy || !x || !gamma || !dx || !dgamma || !dbeta || T < 0 || H < 1 || H > mk::kMaxRowWidth ||
      add == dx || (dx == dy && dtype == 1 && dy_f32)) {
    mimose_set_thread_error("mimose_op_layernorm_bwd_noalloc: bad argument");
    return MIMOSE_ERR_INVALID_ARG;
  }
  const int rc = mk::layernorm_bwd_static(dtype, dy, dy_f32 != 0, x, x_f32 != 0, gamma, dx, add, dgamma, dbeta, T, H, eps,
                                          (hipStream_t)stream);
  if (rc == -1) {
    char buf[200];
    snprintf(buf, sizeof buf,
             "mimose_op_layernorm_bwd_noalloc: %d rows of %d need %lld scratch floats, the fixed array holds %llu",
             T, H, (long long)mk::partial_rows(T) * 2 * H, (unsigned long long)mk::kStaticPartialFloats);
    mimose_set_thread_error(buf);
    return MIMOSE_ERR_INVALID_ARG;
  }
  if (rc != 0) {
    mimose_set_thread_error("mimose_op_layernorm_bwd_noalloc: address of the scratch array not available");
    return MIMOSE_ERR_HIP;
  }
  return done();
}

uint64_t mimose_op_layernorm_bwd_noalloc_max_floats(void) { return mk::kStaticPartialFloats; }

int mimose_op_gelu_bwd(int32_t dtype, void* d, const void* pre, int64_t n, int32_t tanh_form, void* stream) {
  if (bad_dtype(dtype) || !d || !pre || n < 0) return MIMOSE_ERR_INVALID_ARG;
  mk::gelu_bwd(dtype, d, pre, n, tanh_form, (hipStream_t)stream);
  return done();
}

static bool bad_p(float p) { return !(p >= 0.f) || !(p < 1.f); }
static mk::DropDesc make_desc(float p, uint64_t seed, uint32_t site, uint32_t step) {
  mk::DropDesc d;
  if (p <= 0.f) return d;
  d.thr = (uint32_t)std::min(std::floor((double)p * 4294967296.0 + 0.5), 4294967295.0);
  d.scale = (float)(1.0 / (1.0 - (double)p));
  d.k0 = (uint32_t)seed; d.k1 = (uint32_t)(seed >> 32);
  d.site = site; d.step = step;
  return d;
}

int mimose_op_attention_fwd(int32_t dtype, const void* qkv, void* ctx, float* lse, const int32_t* lengths, int32_t B,
                            int32_t L, int32_t nh, int32_t d, int32_t causal, float p_drop, uint64_t seed,
                            uint32_t site, uint32_t step, void* stream) {
  if (bad_dtype(dtype) || !qkv || !ctx || !lse || B < 0 || L < 0 || nh < 1 || bad_head(d) || bad_p(p_drop))
    return MIMOSE_ERR_INVALID_ARG;
  mk::attention_fwd(dtype, qkv, ctx, lse, lengths, B, L, nh, d, causal, make_desc(p_drop, seed, site, step),
                    (hipStream_t)stream);
  return done();
}

int mimose_op_attention_bwd(int32_t dtype, const void* qkv, const void* ctx, const void* dctx, const float* lse,
                            float* delta, void* dqkv, const int32_t* lengths, int32_t B, int32_t L, int32_t nh,
                            int32_t d, int32_t causal, float p_drop, uint64_t seed, uint32_t site, uint32_t step,
                            void* stream) {
  if (bad_dtype(dtype) || !qkv || !ctx || !dctx || !lse || !delta || !dqkv || B < 0 || L < 0 || nh < 1 || bad_head(d) ||
      bad_p(p_drop))
    return MIMOSE_ERR_INVALID_ARG;
  mk::attention_bwd(dtype, qkv, ctx, dctx, lse, delta, dqkv, lengths, B, L, nh, d, causal,
                    make_desc(p_drop, seed, site, step), (hipStream_t)stream);
  return done();
}

int mimose_op_dropout(int32_t dtype, void* dst, const void* src, int32_t io_f32, const void* resid, int64_t n, float p,
                      uint64_t seed, uint32_t site, uint32_t step, void* stream) {
  if (bad_dtype(dtype) || !dst || !src || n < 0 || bad_p(p)) return MIMOSE_ERR_INVALID_ARG;
  mk::dropout_apply(dtype, dst, src, io_f32 != 0, resid, n, make_desc(p, seed, site, step), (hipStream_t)stream);
  return done();
}

int mimose_op_softmax_xent(int32_t dtype, void* logits, int64_t ld, const int32_t* labels, float* row_loss,
                           float* loss, int32_t T, int32_t V, int32_t n_valid, void* stream) {
  if (bad_dtype(dtype) || !logits || !labels || !row_loss || !loss || T < 0 || V < 1 || ld < V) return MIMOSE_ERR_INVALID_ARG;
  mk::softmax_xent(dtype, logits, ld, labels, row_loss, loss, T, V, n_valid, (hipStream_t)stream);
  return done();
}

int mimose_op_embed_fwd(int32_t dtype, const int32_t* ids, const void* tok, const void* pos, const void* gamma,
                        const void* beta, void* sum_out, void* y, int32_t B, int32_t L, int32_t H, float eps,
                        int32_t has_ln, void* stream) {
  if (bad_dtype(dtype) || !ids || !tok || !pos || !y || B < 0 || L < 0 || H < 1 || H > mk::kMaxRowWidth) return MIMOSE_ERR_INVALID_ARG;
  if (has_ln && (!gamma || !beta)) return MIMOSE_ERR_INVALID_ARG;
  mk::embed_fwd(dtype, ids, tok, pos, gamma, beta, sum_out, y, B, L, H, eps, has_ln, (hipStream_t)stream);
  return done();
}

int mimose_op_embed_bwd(int32_t dtype, const void* d, const int32_t* ids, const int32_t* order, const int32_t* seg,
                        int32_t n_seg, float* dtok, float* dpos, int32_t B, int32_t L, int32_t H, int32_t max_seq,
                        void* stream) {
  if (bad_dtype(dtype) || !d || !ids || !order || !seg || !dtok || !dpos || B < 0 || L < 0 || H < 1 || n_seg < 0 || max_seq < L)
    return MIMOSE_ERR_INVALID_ARG;
  mk::embed_bwd(dtype, d, ids, order, seg, n_seg, dtok, dpos, B, L, H, max_seq, (hipStream_t)stream);
  return done();
}

}  // extern "C"
