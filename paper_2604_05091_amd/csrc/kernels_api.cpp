// C ABI wrappers around the individual kernels (declared in include/megatrain_kernels.h):
// argument checks and marshalling only.
#include <hip/hip_runtime.h>
#include <math.h>

#include "../../include/megatrain.h"
#include "../../include/megatrain_kernels.h"
#include "common.h"
#include "host_ops.h"

using namespace mt;

namespace {
inline int32_t to_status(hipError_t e) {
    if (e == hipSuccess) return MT_OK;
    (void)hipGetLastError();
    return e == hipErrorInvalidValue ? MT_ERR_INVALID_ARG : MT_ERR_HIP;
}
inline hipStream_t S(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }
}  // namespace

extern "C" {

int32_t mt_k_gemm_nt(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, void *C, int64_t ldc,
                     const uint16_t *R, int64_t ldr, int32_t M, int32_t N, int32_t K, int32_t out_fp32,
                     int32_t accumulate, void *stream) {
    if (!A || !B || !C) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = R; g.ldr = ldr;
    g.M = M; g.N = N; g.K = K; g.out_fp32 = out_fp32 != 0; g.accumulate = accumulate != 0;
    return to_status(gemm_nt(g, S(stream)));
}

int32_t mt_k_gemm_nt_bias(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *C, int64_t ldc,
                          const uint16_t *bias, int32_t M, int32_t N, int32_t K, void *stream) {
    if (!A || !B || !C || !bias) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = N; g.K = K; g.out_fp32 = 0; g.accumulate = 0; g.bias = bias;
    return to_status(gemm_nt(g, S(stream)));
}

int32_t mt_k_gemm_nt_rope(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *C, int64_t ldc,
                          const uint16_t *bias, const float *cos_tab, const float *sin_tab, int32_t T,
                          int32_t rope_cols, int32_t M, int32_t N, int32_t K, void *stream) {
    if (!A || !B || !C || !cos_tab || !sin_tab || T <= 0 || rope_cols < 0) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = N; g.K = K; g.out_fp32 = 0; g.accumulate = 0; g.bias = bias;
    g.rope_cos = cos_tab; g.rope_sin = sin_tab; g.rope_T = T; g.rope_cols = rope_cols;
    const hipError_t e = gemm_nt(g, S(stream));
    if (e == hipErrorNotSupported) return MT_ERR_UNSUPPORTED;
    return to_status(e);
}

int32_t mt_k_gemm_nt_swiglu(const uint16_t *A, int64_t lda, const uint16_t *W, int64_t ldw, uint16_t *gu, int64_t ldgu,
                            uint16_t *s, int64_t lds, int32_t M, int32_t F, int32_t K, void *stream) {
    if (!A || !W || !s || F <= 0) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = W; g.ldb = ldw; g.C = gu; g.ldc = ldgu; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = 2 * F; g.K = K; g.out_fp32 = 0; g.accumulate = 0;
    g.glu_F = F; g.glu_out = s; g.ld_glu = lds;
    const hipError_t e = gemm_nt(g, S(stream));
    if (e == hipErrorNotSupported) return MT_ERR_UNSUPPORTED;
    return to_status(e);
}

int32_t mt_k_gemm_nt_swiglu_bwd(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *dgu, int64_t lddgu,
                                const uint16_t *gu, int64_t ldgu, int32_t M, int32_t F, int32_t K, void *stream) {
    if (!A || !B || !dgu || !gu || F <= 0) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = dgu; g.ldc = lddgu; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = F; g.K = K; g.out_fp32 = 0; g.accumulate = 0;
    g.glu_bwd_gu = gu; g.ld_glu_bwd = ldgu;
    const hipError_t e = gemm_nt(g, S(stream));
    if (e == hipErrorNotSupported) return MT_ERR_UNSUPPORTED;
    return to_status(e);
}

int32_t mt_k_gemm_tn(const uint16_t *At, int64_t lda, const uint16_t *Bt, int64_t ldb, float *C, int64_t ldc, int32_t M,
                     int32_t N, int32_t K, int32_t accumulate, void *stream) {
    if (!At || !Bt || !C) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = At; g.lda = lda; g.B = Bt; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = N; g.K = K; g.out_fp32 = 1; g.accumulate = accumulate != 0;
    const hipError_t e = gemm_tn(g, S(stream));
    if (e == hipErrorNotSupported) return MT_ERR_UNSUPPORTED;
    return to_status(e);
}

int32_t mt_k_gemm_tn_split(const uint16_t *At, int64_t lda, const uint16_t *Bt, int64_t ldb, float *C, int64_t ldc, int32_t M,
                           int32_t N, int32_t K, int32_t accumulate, int32_t split_k, float *ws, void *stream) {
    if (!At || !Bt || !C || split_k < 1 || (split_k > 1 && !ws)) return MT_ERR_INVALID_ARG;
    GemmArgs g;
    g.A = At; g.lda = lda; g.B = Bt; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = nullptr; g.ldr = 0;
    g.M = M; g.N = N; g.K = K; g.out_fp32 = 1; g.accumulate = accumulate != 0;
    g.split_k = split_k; g.split_ws = ws;
    const hipError_t e = gemm_tn(g, S(stream));
    if (e == hipErrorNotSupported) return MT_ERR_UNSUPPORTED;
    return to_status(e);
}
int32_t mt_k_gemm_tn_pick_split(int64_t M, int64_t N, int64_t K, int32_t n_cu) { return gemm_tn_pick_split(M, N, K, n_cu); }

size_t mt_k_bias_grad_ws_bytes(int32_t cols) { return bias_grad_ws_floats(cols) * sizeof(float); }
int32_t mt_k_bias_grad(float *db, const uint16_t *x, int64_t ld, int64_t n, int32_t cols, void *ws, void *stream) {
    if (!db || !x || !ws || !al16(x)) return MT_ERR_INVALID_ARG;
    return to_status(bias_grad(db, x, ld, n, cols, reinterpret_cast<float *>(ws), S(stream)));
}

int32_t mt_k_transpose(const uint16_t *in, uint16_t *out, int32_t rows, int32_t cols, int64_t ld_in, int64_t ld_out,
                       int32_t nb0, int32_t nb1, int64_t in_s0, int64_t in_s1, int64_t out_s0, int64_t out_s1,
                       void *stream) {
    if (!in || !out) return MT_ERR_INVALID_ARG;
    TransposeArgs t;
    t.in = in; t.out = out; t.rows = rows; t.cols = cols; t.ld_in = ld_in; t.ld_out = ld_out;
    t.nb0 = nb0; t.nb1 = nb1; t.in_s0 = in_s0; t.in_s1 = in_s1; t.out_s0 = out_s0; t.out_s1 = out_s1;
    return to_status(transpose_bf16(t, S(stream)));
}

int32_t mt_k_rmsnorm_fwd(uint16_t *y, const uint16_t *x, const uint16_t *gain, int64_t n, int32_t d, float eps,
                         void *stream) {
    if (!y || !x || !gain || !al16(y) || !al16(x) || !al16(gain)) return MT_ERR_INVALID_ARG;
    return to_status(rmsnorm_fwd(y, x, gain, n, d, eps, S(stream)));
}

size_t mt_k_rmsnorm_bwd_ws_bytes(int32_t d) { return d > 0 ? rmsnorm_bwd_ws_floats(d) * sizeof(float) : 0; }

int32_t mt_k_rmsnorm_bwd(uint16_t *dx, float *dgain, const uint16_t *dy, const uint16_t *x, const uint16_t *gain,
                         const uint16_t *dres, void *ws, int64_t n, int32_t d, float eps, void *stream) {
    if (!dx || !dgain || !dy || !x || !gain || !ws) return MT_ERR_INVALID_ARG;
    if (!al16(dx) || !al16(dy) || !al16(x) || !al16(gain) || !al16(dres)) return MT_ERR_INVALID_ARG;
    return to_status(rmsnorm_bwd(dx, dgain, dy, x, gain, dres, (float *)ws, n, d, eps, S(stream)));
}

int32_t mt_k_rmsnorm_bwd_noalloc(uint16_t *dx, float *dgain, const uint16_t *dy, const uint16_t *x, const uint16_t *gain,
                                 const uint16_t *dres, int64_t n, int32_t d, float eps, void *stream) {
    if (!dx || !dgain || !dy || !x || !gain) return MT_ERR_INVALID_ARG;
    if (!al16(dx) || !al16(dy) || !al16(x) || !al16(gain) || !al16(dres)) return MT_ERR_INVALID_ARG;
    if (n <= 0 || d <= 0 || (d & 7)) return MT_ERR_INVALID_ARG;
    if (d > MT_K_RMSNORM_BWD_NOALLOC_MAX_D) return MT_ERR_UNSUPPORTED;  // beyond the static workspace
    return to_status(rmsnorm_bwd_static(dx, dgain, dy, x, gain, dres, n, d, eps, S(stream)));
}

int32_t mt_k_rope_table(float *host_cos, float *host_sin, int32_t T, int32_t hd, double base) {
    if (!host_cos || !host_sin || T <= 0 || hd <= 0 || (hd & 1) || !(base > 0)) return MT_ERR_INVALID_ARG;
    rope_table(host_cos, host_sin, T, hd, base);
    return MT_OK;
}

int32_t mt_k_rope(uint16_t *x, int64_t ld, int64_t n, int32_t T, int32_t n_heads, int32_t hd, const float *cos_tab,
                  const float *sin_tab, int32_t sign, void *stream) {
    if (!x || !cos_tab || !sin_tab || !al16(x) || !al16(cos_tab) || !al16(sin_tab)) return MT_ERR_INVALID_ARG;
    if ((int64_t)n_heads * hd > ld) return MT_ERR_INVALID_ARG;
    return to_status(rope_inplace(x, ld, n, T, n_heads, hd, cos_tab, sin_tab, sign, S(stream)));
}

int32_t mt_k_swiglu_fwd(uint16_t *s, const uint16_t *gu, int64_t n, int32_t F, void *stream) {
    if (!s || !gu || !al16(s) || !al16(gu)) return MT_ERR_INVALID_ARG;
    return to_status(swiglu_fwd(s, gu, n, F, S(stream)));
}

int32_t mt_k_swiglu_bwd(uint16_t *dgu, const uint16_t *ds, const uint16_t *gu, int64_t n, int32_t F, void *stream) {
    if (!dgu || !ds || !gu || !al16(dgu) || !al16(ds) || !al16(gu)) return MT_ERR_INVALID_ARG;
    return to_status(swiglu_bwd(dgu, ds, gu, n, F, S(stream)));
}

int32_t mt_k_embed_gather(uint16_t *h, const uint16_t *table, const int32_t *tokens, int64_t n, int32_t d,
                          void *stream) {
    if (!h || !table || !tokens || !al16(h) || !al16(table)) return MT_ERR_INVALID_ARG;
    return to_status(embed_gather(h, table, tokens, n, d, S(stream)));
}

int32_t mt_k_embed_scatter(float *dtable, const uint16_t *dh, const int32_t *row_start, const int32_t *order,
                           int32_t V, int32_t d, void *stream) {
    if (!dtable || !dh || !row_start || !order || !al16(dtable) || !al16(dh)) return MT_ERR_INVALID_ARG;
    return to_status(embed_scatter(dtable, dh, row_start, order, V, d, S(stream)));
}

int32_t mt_k_cross_entropy(float *loss_rows, uint16_t *dlogits, const float *logits, const int32_t *labels, int64_t n,
                           int32_t V, float inv_n, void *stream) {
    if (!loss_rows || !dlogits || !logits || !labels || !al16(logits) || ((uintptr_t)dlogits & 7))
        return MT_ERR_INVALID_ARG;
    return to_status(cross_entropy(loss_rows, dlogits, logits, labels, n, V, inv_n, S(stream)));
}

int32_t mt_k_reduce_sum(float *out, const float *in, int64_t n, float scale, int32_t accumulate, void *stream) {
    if (!out || !in) return MT_ERR_INVALID_ARG;
    return to_status(reduce_sum(out, in, n, scale, accumulate, S(stream)));
}

int32_t mt_k_flash_fwd(uint16_t *o, int64_t ldo, float *lse, const uint16_t *q, int64_t ldq, const uint16_t *k,
                       int64_t ldk, const uint16_t *v, int64_t ldv, int32_t B, int32_t T, int32_t Hq, int32_t Hkv,
                       int32_t hd, float scale, void *stream) {
    if (!o || !lse || !q || !k || !v) return MT_ERR_INVALID_ARG;
    AttnArgs a = {};
    a.B = B; a.T = T; a.Hq = Hq; a.Hkv = Hkv; a.hd = hd; a.scale = scale;
    a.q = q; a.ldq = ldq; a.k = k; a.ldk = ldk; a.v = v; a.ldv = ldv; a.o = o; a.ldo = ldo; a.lse = lse;
    return to_status(flash_fwd(a, S(stream)));
}

int32_t mt_k_flash_bwd_rope(uint16_t *dq, int64_t lddq, uint16_t *dk, int64_t lddk, uint16_t *dv, int64_t lddv,
                            const uint16_t *dout, int64_t lddo, const uint16_t *q, int64_t ldq, const uint16_t *k,
                            int64_t ldk, const uint16_t *v, int64_t ldv, const uint16_t *o, int64_t ldo,
                            const float *lse, float *delta, const float *cos_tab, const float *sin_tab, int32_t B,
                            int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, float scale, void *stream) {
    if (!dq || !dk || !dv || !dout || !q || !k || !v || !o || !lse || !delta) return MT_ERR_INVALID_ARG;
    if (B <= 0 || T <= 0 || Hq <= 0 || (hd != 64 && hd != 128) || (T & 7) || (lddo & 7) || (ldo & 7) || !al16(dout) ||
        !al16(o))
        return MT_ERR_INVALID_ARG;
    if ((cos_tab == nullptr) != (sin_tab == nullptr)) return MT_ERR_INVALID_ARG;
    AttnArgs a = {};
    a.B = B; a.T = T; a.Hq = Hq; a.Hkv = Hkv; a.hd = hd; a.scale = scale;
    a.q = q; a.ldq = ldq; a.k = k; a.ldk = ldk; a.v = v; a.ldv = ldv;
    a.o = const_cast<uint16_t *>(o); a.ldo = ldo; a.lse = const_cast<float *>(lse);
    a.dout = dout; a.lddo = lddo; a.delta = delta;
    a.dq = dq; a.lddq = lddq; a.dk = dk; a.lddk = lddk; a.dv = dv; a.lddv = lddv;
    a.rope_cos = cos_tab; a.rope_sin = sin_tab;
    hipStream_t s = S(stream);
    hipError_t e = attn_delta(delta, dout, lddo, o, ldo, B, T, Hq, hd, s);
    if (e != hipSuccess) return to_status(e);
    e = flash_bwd_dkdv(a, s);
    if (e != hipSuccess) return to_status(e);
    return to_status(flash_bwd_dq(a, s));
}

int32_t mt_k_flash_bwd(uint16_t *dq, int64_t lddq, uint16_t *dk, int64_t lddk, uint16_t *dv, int64_t lddv,
                       const uint16_t *dout, int64_t lddo, const uint16_t *q, int64_t ldq, const uint16_t *k,
                       int64_t ldk, const uint16_t *v, int64_t ldv, const uint16_t *o, int64_t ldo, const float *lse,
                       float *delta, int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, float scale,
                       void *stream) {
    return mt_k_flash_bwd_rope(dq, lddq, dk, lddk, dv, lddv, dout, lddo, q, ldq, k, ldk, v, ldv, o, ldo, lse, delta, nullptr,
                               nullptr, B, T, Hq, Hkv, hd, scale, stream);
}

int32_t mt_k_host_adam(float *host_p, const float *host_g, float *host_m, float *host_v, uint16_t *host_shadow,
                       size_t n, float lr, float beta1, float beta2, float eps, float wd, int64_t step) {
    if (!host_p || !host_g || !host_m || !host_v || step < 1) return MT_ERR_INVALID_ARG;
    host_adam(host_p, host_g, host_m, host_v, host_shadow, n, lr, beta1, beta2, eps, wd, step);
    return MT_OK;
}

int32_t mt_k_host_f32_to_bf16(uint16_t *host_out, const float *host_in, size_t n) {
    if (!host_out || !host_in) return MT_ERR_INVALID_ARG;
    host_f32_to_bf16(host_out, host_in, n);
    return MT_OK;
}

}  // extern "C"
