/*
 * CPU oracle for the streamed decoder-only training step and the host Adam update.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct definition
 * of what one training step computes, used only by the tests, the smoke check and
 * the benchmark's CPU-baseline leg.  The GPU library never calls it and shares no
 * code, header, table or constant with it.
 *
 * What it follows (MegaTrain, Algorithm 1 "MegaTrain Training Step"):
 *   Phase 1  streaming forward   h_0 = Embed(x); h_i = f_i(h_{i-1}; theta_i)
 *   Phase 2  loss anchoring      l = L(h_L); g_L = dl/dh_L; head gradients
 *   Phase 3  block-wise backward for each block (here one layer = one block, K = 1):
 *            recompute the block from its checkpoint, then LocalBackward
 *   last     AdamUpdate(theta, grad, m, v) on the host (Section 3.1, "optimizer update")
 * The paper states (Section 4.2, accuracy paragraph) that recomputation and the
 * host master copy leave the result of ordinary back-propagation unchanged, so the
 * oracle is ordinary back-propagation written out, in two execution orders that
 * must agree: "monolithic" (store every activation, one sweep back) and
 * "streamed" (keep only h_0..h_L; recompute each layer right before its backward).
 *
 * The layer f_i is not specified by the paper beyond "Attention and MLP blocks"
 * (Section 3.4); the workloads fix it: pre-norm Llama-style block with RMSNorm,
 * rotary embedding (half-split pairing), causal softmax attention with grouped
 * KV heads, SwiGLU MLP, no biases, untied LM head, mean token cross-entropy.
 *
 * Precision: compile with -DREAL=double (reference and finite-difference judge)
 * or -DREAL=float (the fp32 variant that the benchmark times).  Plain loops,
 * OpenMP over independent outputs, no blocking or fusion.
 *
 * Parity pins (tests/test_oracle_*.py): central finite differences in double on
 * every tensor; agreement with PyTorch CPU autograd built from library ops
 * (rms_norm, scaled_dot_product_attention, cross_entropy, AdamW); closed forms
 * (loss = ln V for a zero head, Adam first step, RoPE isometry / relative phase,
 * uniform attention for q = 0); causality; batch independence; GQA == MHA with
 * replicated KV weights; streamed == monolithic.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t qkv_bias; /* 1: the q, k, v projections carry a bias vector each (Qwen2.5-style layers, the models of
                         Section 4.1); a layer then has 12 tensors instead of 9: ..., w_down, bq, bk, bv */
    int32_t tie_embeddings; /* 1: the output projection uses the embedding table (Appendix A.1, tied weights); the
                               parameter list then ends with final_norm and the table's gradient is the sum of
                               the head's weight gradient and the embedding's scatter-add */
    double rope_base, rms_eps;
} orc_cfg;

/* tensors per layer in the canonical order */
static int64_t per_layer(const orc_cfg *cf) { return cf->qkv_bias ? 12 : 9; }

int orc_real_bytes(void) { return (int)sizeof(real); }

/* ------------------------------------------------------------------ linear maps
 * y[n,out] = x[n,in] . w[out,in]^T  (a bias-free linear layer, weight stored [out,in]) */
void orc_linear_fwd(real *y, const real *x, const real *w, int64_t n, int64_t in, int64_t out) {
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        const real *wr = w + o * in;
        for (int64_t t = 0; t < n; ++t) {
            const real *xr = x + t * in;
            real acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int64_t i = 0; i < in; ++i) acc += xr[i] * wr[i];
            y[t * out + o] = acc;
        }
    }
}

/* dx[n,in] = dy[n,out] . w[out,in] */
void orc_linear_bwd_x(real *dx, const real *dy, const real *w, int64_t n, int64_t in, int64_t out) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        real *dxr = dx + t * in;
        for (int64_t i = 0; i < in; ++i) dxr[i] = 0;
        for (int64_t o = 0; o < out; ++o) {
            const real g = dy[t * out + o];
            const real *wr = w + o * in;
#pragma omp simd
            for (int64_t i = 0; i < in; ++i) dxr[i] += g * wr[i];
        }
    }
}

/* dw[out,in] = sum_t dy[t,out] x[t,in] */
void orc_linear_bwd_w(real *dw, const real *dy, const real *x, int64_t n, int64_t in, int64_t out) {
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        real *dwr = dw + o * in;
        for (int64_t i = 0; i < in; ++i) dwr[i] = 0;
        for (int64_t t = 0; t < n; ++t) {
            const real g = dy[t * out + o];
            const real *xr = x + t * in;
#pragma omp simd
            for (int64_t i = 0; i < in; ++i) dwr[i] += g * xr[i];
        }
    }
}

/* ------------------------------------------------------------------ RMSNorm
 * r = 1/sqrt(mean_j x_j^2 + eps);  y_j = x_j r g_j */
void orc_rmsnorm_fwd(real *y, const real *x, const real *g, int64_t n, int64_t d, double eps) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const real *xr = x + t * d;
        real ss = 0;
        for (int64_t j = 0; j < d; ++j) ss += xr[j] * xr[j];
        const real r = (real)(1.0 / sqrt((double)ss / (double)d + eps));
        for (int64_t j = 0; j < d; ++j) y[t * d + j] = xr[j] * r * g[j];
    }
}

/* With u = g (.) dy:  dx = r u - x r^3 mean_j(u_j x_j);  dg_j = sum_t dy_tj x_tj r_t.
 * dx is written, dg is written (not accumulated). */
void orc_rmsnorm_bwd(real *dx, real *dg, const real *dy, const real *x, const real *g, int64_t n, int64_t d,
                     double eps) {
    real *rs = (real *)malloc(sizeof(real) * (size_t)n);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const real *xr = x + t * d, *dyr = dy + t * d;
        real ss = 0;
        for (int64_t j = 0; j < d; ++j) ss += xr[j] * xr[j];
        const real r = (real)(1.0 / sqrt((double)ss / (double)d + eps));
        rs[t] = r;
        real dot = 0;
        for (int64_t j = 0; j < d; ++j) dot += g[j] * dyr[j] * xr[j];
        const real c = r * r * r * dot / (real)d;
        for (int64_t j = 0; j < d; ++j) dx[t * d + j] = r * g[j] * dyr[j] - xr[j] * c;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        real acc = 0;
        for (int64_t t = 0; t < n; ++t) acc += dy[t * d + j] * x[t * d + j] * rs[t];
        dg[j] = acc;
    }
    free(rs);
}

/* ------------------------------------------------------------------ rotary embedding
 * x is [B*T, H*hd]; position of row (b,t) is t.  Pair (j, j+hd/2), frequency
 * base^(-2j/hd), angle = t * frequency; sign = +1 rotates forward, -1 is the
 * transpose (the backward map of the rotation).  In place. */
void orc_rope(real *x, int64_t B, int64_t T, int64_t H, int64_t hd, double base, int sign) {
    const int64_t half = hd / 2;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < B * T; ++row) {
        const int64_t t = row % T;
        for (int64_t h = 0; h < H; ++h) {
            real *v = x + (row * H + h) * hd;
            for (int64_t j = 0; j < half; ++j) {
                const double freq = pow(base, -2.0 * (double)j / (double)hd);
                const double ang = (double)t * freq;
                const real c = (real)cos(ang), s = (real)(sign * sin(ang));
                const real a = v[j], b = v[j + half];
                v[j] = a * c - b * s;
                v[j + half] = b * c + a * s;
            }
        }
    }
}

/* ------------------------------------------------------------------ causal attention
 * q [B*T, Hq*hd], k and v [B*T, Hkv*hd]; query head h reads KV head h / (Hq/Hkv).
 * s_tu = q_t.k_u / sqrt(hd) for u <= t; p = softmax_u(s); a_t = sum_u p_tu v_u. */
void orc_attention_fwd(real *a, const real *q, const real *k, const real *v, int64_t B, int64_t T, int64_t Hq,
                       int64_t Hkv, int64_t hd) {
    const int64_t G = Hq / Hkv;
    const real scale = (real)(1.0 / sqrt((double)hd));
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < Hq; ++h) {
            const int64_t hk = h / G;
            real *p = (real *)malloc(sizeof(real) * (size_t)T);
            for (int64_t t = 0; t < T; ++t) {
                const real *qt = q + ((b * T + t) * Hq + h) * hd;
                real mx = -INFINITY;
                for (int64_t u = 0; u <= t; ++u) {
                    const real *ku = k + ((b * T + u) * Hkv + hk) * hd;
                    real s = 0;
                    for (int64_t j = 0; j < hd; ++j) s += qt[j] * ku[j];
                    p[u] = s * scale;
                    if (p[u] > mx) mx = p[u];
                }
                real den = 0;
                for (int64_t u = 0; u <= t; ++u) {
                    p[u] = (real)exp((double)(p[u] - mx));
                    den += p[u];
                }
                real *at = a + ((b * T + t) * Hq + h) * hd;
                for (int64_t j = 0; j < hd; ++j) at[j] = 0;
                for (int64_t u = 0; u <= t; ++u) {
                    const real w = p[u] / den;
                    const real *vu = v + ((b * T + u) * Hkv + hk) * hd;
                    for (int64_t j = 0; j < hd; ++j) at[j] += w * vu[j];
                }
            }
            free(p);
        }
}

/* Backward of the above.  dv_u = sum_t p_tu da_t; dp_tu = da_t.v_u;
 * ds = p (.) (dp - sum_u p dp); dq_t = sum_u ds_tu k_u / sqrt(hd); dk_u = sum_t ds_tu q_t / sqrt(hd).
 * dk, dv of a KV head are summed over the query heads of its group.  All three outputs are written. */
void orc_attention_bwd(real *dq, real *dk, real *dv, const real *da, const real *q, const real *k, const real *v,
                       int64_t B, int64_t T, int64_t Hq, int64_t Hkv, int64_t hd) {
    const int64_t G = Hq / Hkv;
    const real scale = (real)(1.0 / sqrt((double)hd));
    memset(dk, 0, sizeof(real) * (size_t)(B * T * Hkv * hd));
    memset(dv, 0, sizeof(real) * (size_t)(B * T * Hkv * hd));
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t hk = 0; hk < Hkv; ++hk) {
            real *p = (real *)malloc(sizeof(real) * (size_t)T);
            real *dp = (real *)malloc(sizeof(real) * (size_t)T);
            for (int64_t h = hk * G; h < (hk + 1) * G; ++h)
                for (int64_t t = 0; t < T; ++t) {
                    const real *qt = q + ((b * T + t) * Hq + h) * hd;
                    const real *dat = da + ((b * T + t) * Hq + h) * hd;
                    real mx = -INFINITY;
                    for (int64_t u = 0; u <= t; ++u) {
                        const real *ku = k + ((b * T + u) * Hkv + hk) * hd;
                        real s = 0;
                        for (int64_t j = 0; j < hd; ++j) s += qt[j] * ku[j];
                        p[u] = s * scale;
                        if (p[u] > mx) mx = p[u];
                    }
                    real den = 0;
                    for (int64_t u = 0; u <= t; ++u) {
                        p[u] = (real)exp((double)(p[u] - mx));
                        den += p[u];
                    }
                    real pdp = 0;
                    for (int64_t u = 0; u <= t; ++u) {
                        p[u] /= den;
                        const real *vu = v + ((b * T + u) * Hkv + hk) * hd;
                        real s = 0;
                        for (int64_t j = 0; j < hd; ++j) s += dat[j] * vu[j];
                        dp[u] = s;
                        pdp += p[u] * s;
                    }
                    real *dqt = dq + ((b * T + t) * Hq + h) * hd;
                    for (int64_t j = 0; j < hd; ++j) dqt[j] = 0;
                    for (int64_t u = 0; u <= t; ++u) {
                        const real ds = p[u] * (dp[u] - pdp) * scale;
                        const real *ku = k + ((b * T + u) * Hkv + hk) * hd;
                        real *dku = dk + ((b * T + u) * Hkv + hk) * hd;
                        real *dvu = dv + ((b * T + u) * Hkv + hk) * hd;
                        for (int64_t j = 0; j < hd; ++j) {
                            dqt[j] += ds * ku[j];
                            dku[j] += ds * qt[j];
                            dvu[j] += p[u] * dat[j];
                        }
                    }
                }
            free(p);
            free(dp);
        }
}

/* One query row of the causal attention above, and the gradient with respect to that query:
 * a = sum_u p_u v_u with p = softmax_u(q.k_u / sqrt(hd)) over the n_keys visible keys (k, v are
 * [n_keys, hd] contiguous); dq = sum_u p_u (dp_u - sum_w p_w dp_w) k_u / sqrt(hd), dp_u = da.v_u.
 * Used to check single rows of very long sequences, where the full O(T^2) routine is out of reach. */
void orc_attention_row(real *a, real *dq, const real *q, const real *da, const real *k, const real *v, int64_t n_keys,
                       int64_t hd) {
    const real scale = (real)(1.0 / sqrt((double)hd));
    real *p = (real *)malloc(sizeof(real) * (size_t)n_keys);
    real mx = -INFINITY;
    for (int64_t u = 0; u < n_keys; ++u) {
        real s = 0;
        for (int64_t j = 0; j < hd; ++j) s += q[j] * k[u * hd + j];
        p[u] = s * scale;
        if (p[u] > mx) mx = p[u];
    }
    real den = 0;
    for (int64_t u = 0; u < n_keys; ++u) {
        p[u] = (real)exp((double)(p[u] - mx));
        den += p[u];
    }
    for (int64_t j = 0; j < hd; ++j) a[j] = 0;
    for (int64_t u = 0; u < n_keys; ++u) {
        p[u] /= den;
        for (int64_t j = 0; j < hd; ++j) a[j] += p[u] * v[u * hd + j];
    }
    if (dq && da) {
        real pdp = 0;
        real *dp = (real *)malloc(sizeof(real) * (size_t)n_keys);
        for (int64_t u = 0; u < n_keys; ++u) {
            real s = 0;
            for (int64_t j = 0; j < hd; ++j) s += da[j] * v[u * hd + j];
            dp[u] = s;
            pdp += p[u] * s;
        }
        for (int64_t j = 0; j < hd; ++j) dq[j] = 0;
        for (int64_t u = 0; u < n_keys; ++u) {
            const real ds = p[u] * (dp[u] - pdp) * scale;
            for (int64_t j = 0; j < hd; ++j) dq[j] += ds * k[u * hd + j];
        }
        free(dp);
    }
    free(p);
}

/* One key row of the same attention (one head of one sequence): the gradients that key u and its value receive
 * from every query that sees it, t = u .. T-1.  q, da, k, v are [T, hd] contiguous (rows before u of q and da are
 * not read).  For each such query: p_t = softmax over keys 0..t, a_t = sum_w p_tw v_w,
 * dS_tu = p_tu (da_t.v_u - da_t.a_t);  dv_u = sum_t p_tu da_t,  dk_u = sum_t dS_tu q_t / sqrt(hd).
 * Costs (T-u) full softmax rows, so it reaches keys near the end of very long sequences. */
void orc_attention_key_row(real *dk, real *dv, const real *q, const real *da, const real *k, const real *v, int64_t T,
                           int64_t hd, int64_t u) {
    const real scale = (real)(1.0 / sqrt((double)hd));
    const int64_t nq = T - u;
    real *pu = (real *)malloc(sizeof(real) * (size_t)nq);  /* p_tu of query t = u + i */
    real *ds = (real *)malloc(sizeof(real) * (size_t)nq);  /* dS_tu / sqrt(hd) */
    /* the queries are independent of each other */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nq; ++i) {
        const int64_t t = u + i;
        const real *qt = q + t * hd, *dat = da + t * hd;
        real *p = (real *)malloc(sizeof(real) * (size_t)(t + 1));
        real *a = (real *)malloc(sizeof(real) * (size_t)hd);
        real mx = -INFINITY, den = 0;
        for (int64_t w = 0; w <= t; ++w) {
            real s = 0;
            for (int64_t j = 0; j < hd; ++j) s += qt[j] * k[w * hd + j];
            p[w] = s * scale;
            if (p[w] > mx) mx = p[w];
        }
        for (int64_t w = 0; w <= t; ++w) {
            p[w] = (real)exp((double)(p[w] - mx));
            den += p[w];
        }
        for (int64_t j = 0; j < hd; ++j) a[j] = 0;
        for (int64_t w = 0; w <= t; ++w) {
            p[w] /= den;
            for (int64_t j = 0; j < hd; ++j) a[j] += p[w] * v[w * hd + j];
        }
        real dp_u = 0, delta = 0;
        for (int64_t j = 0; j < hd; ++j) {
            dp_u += dat[j] * v[u * hd + j];
            delta += dat[j] * a[j];
        }
        pu[i] = p[u];
        ds[i] = p[u] * (dp_u - delta) * scale;
        free(a);
        free(p);
    }
    for (int64_t j = 0; j < hd; ++j) dk[j] = dv[j] = 0;
    for (int64_t i = 0; i < nq; ++i)
        for (int64_t j = 0; j < hd; ++j) {
            dv[j] += pu[i] * da[(u + i) * hd + j];
            dk[j] += ds[i] * q[(u + i) * hd + j];
        }
    free(ds);
    free(pu);
}

/* ------------------------------------------------------------------ SwiGLU
 * s = gate * sigmoid(gate) * up */
void orc_swiglu_fwd(real *s, const real *gate, const real *up, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const real sg = (real)(1.0 / (1.0 + exp(-(double)gate[i])));
        s[i] = gate[i] * sg * up[i];
    }
}

/* dgate = ds up sig (1 + gate (1 - sig));  dup = ds gate sig */
void orc_swiglu_bwd(real *dgate, real *dup, const real *ds, const real *gate, const real *up, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const real sg = (real)(1.0 / (1.0 + exp(-(double)gate[i])));
        dgate[i] = ds[i] * up[i] * sg * (1 + gate[i] * (1 - sg));
        dup[i] = ds[i] * gate[i] * sg;
    }
}

/* ------------------------------------------------------------------ cross-entropy
 * loss = -(1/Nv) sum_valid log softmax(z_t)[label_t]; a negative label is ignored.
 * dlogits = (softmax - onehot)/Nv on valid rows, 0 elsewhere (may be NULL). */
void orc_cross_entropy(real *loss, real *dlogits, const real *logits, const int32_t *labels, int64_t n, int64_t V) {
    int64_t nv = 0;
    for (int64_t t = 0; t < n; ++t) nv += labels[t] >= 0;
    double *rowloss = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const real *z = logits + t * V;
        if (labels[t] < 0) {
            if (dlogits)
                for (int64_t c = 0; c < V; ++c) dlogits[t * V + c] = 0;
            continue;
        }
        real mx = z[0];
        for (int64_t c = 1; c < V; ++c)
            if (z[c] > mx) mx = z[c];
        double den = 0;
        for (int64_t c = 0; c < V; ++c) den += exp((double)(z[c] - mx));
        const double lse = (double)mx + log(den);
        rowloss[t] = lse - (double)z[labels[t]];
        if (dlogits)
            for (int64_t c = 0; c < V; ++c) {
                const double p = exp((double)z[c] - lse);
                dlogits[t * V + c] = (real)((p - (c == labels[t] ? 1.0 : 0.0)) / (double)nv);
            }
    }
    double total = 0;
    for (int64_t t = 0; t < n; ++t) total += rowloss[t];
    free(rowloss);
    *loss = (real)(nv ? total / (double)nv : 0.0);
}

/* ------------------------------------------------------------------ embedding */
void orc_embed_fwd(real *h, const real *table, const int32_t *tokens, int64_t n, int64_t d) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) memcpy(h + t * d, table + (int64_t)tokens[t] * d, sizeof(real) * (size_t)d);
}

void orc_embed_bwd(real *dtable, const real *dh, const int32_t *tokens, int64_t n, int64_t V, int64_t d) {
    memset(dtable, 0, sizeof(real) * (size_t)(V * d));
    for (int64_t t = 0; t < n; ++t) {
        real *row = dtable + (int64_t)tokens[t] * d;
        for (int64_t j = 0; j < d; ++j) row[j] += dh[t * d + j];
    }
}

/* ------------------------------------------------------------------ Adam (decoupled weight decay)
 * p <- p (1 - lr wd);  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 * p <- p - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps),  t >= 1. */
void orc_adam(real *p, const real *g, real *m, real *v, int64_t n, double lr, double b1, double b2, double eps,
              double wd, int64_t t) {
    const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double gi = (double)g[i];
        const double mi = b1 * (double)m[i] + (1.0 - b1) * gi;
        const double vi = b2 * (double)v[i] + (1.0 - b2) * gi * gi;
        double pi = (double)p[i] * (1.0 - lr * wd);
        pi -= lr * (mi / c1) / (sqrt(vi / c2) + eps);
        m[i] = (real)mi;
        v[i] = (real)vi;
        p[i] = (real)pi;
    }
}

/* ------------------------------------------------------------------ one transformer block
 * Everything a block's backward needs besides its input x. */
/* y[t, :] += b  and its gradient  db = sum over rows of dy */
void orc_bias_add(real *y, const real *b, int64_t n, int64_t out) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t)
        for (int64_t o = 0; o < out; ++o) y[t * out + o] += b[o];
}
void orc_bias_bwd(real *db, const real *dy, int64_t n, int64_t out) {
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        real acc = 0;
        for (int64_t t = 0; t < n; ++t) acc += dy[t * out + o];
        db[o] = acc;
    }
}

typedef struct {
    real *xn;  /* RMSNorm(x; g1)              [n, d]        */
    real *q;   /* rotated queries             [n, Hq*hd]    */
    real *k;   /* rotated keys                [n, Hkv*hd]   */
    real *v;   /* values                      [n, Hkv*hd]   */
    real *a;   /* attention output            [n, Hq*hd]    */
    real *h1;  /* x + a Wo^T                  [n, d]        */
    real *yn;  /* RMSNorm(h1; g2)             [n, d]        */
    real *gt;  /* yn Wgate^T                  [n, F]        */
    real *up;  /* yn Wup^T                    [n, F]        */
    real *s;   /* silu(gt) * up               [n, F]        */
} block_cache;

static real *ralloc(int64_t n) { return (real *)malloc(sizeof(real) * (size_t)(n > 0 ? n : 1)); }

static void cache_alloc(block_cache *c, const orc_cfg *cf, int64_t n) {
    const int64_t d = cf->hidden, nq = (int64_t)cf->n_q_heads * cf->head_dim,
                  nkv = (int64_t)cf->n_kv_heads * cf->head_dim, F = cf->ffn;
    c->xn = ralloc(n * d); c->q = ralloc(n * nq); c->k = ralloc(n * nkv); c->v = ralloc(n * nkv);
    c->a = ralloc(n * nq); c->h1 = ralloc(n * d); c->yn = ralloc(n * d);
    c->gt = ralloc(n * F); c->up = ralloc(n * F); c->s = ralloc(n * F);
}

static void cache_free(block_cache *c) {
    free(c->xn); free(c->q); free(c->k); free(c->v); free(c->a);
    free(c->h1); free(c->yn); free(c->gt); free(c->up); free(c->s);
}

/* tensors of one block in canonical order:
 * 0 attn_norm[d] 1 wq[Hq*hd,d] 2 wk[Hkv*hd,d] 3 wv[Hkv*hd,d] 4 wo[d,Hq*hd]
 * 5 mlp_norm[d]  6 w_gate[F,d] 7 w_up[F,d]    8 w_down[d,F] */
static void block_forward(real *y, const real *x, const real *const *w, block_cache *c, const orc_cfg *cf,
                          int64_t B, int64_t T) {
    const int64_t n = B * T, d = cf->hidden, Hq = cf->n_q_heads, Hkv = cf->n_kv_heads, hd = cf->head_dim,
                  nq = Hq * hd, nkv = Hkv * hd, F = cf->ffn;
    orc_rmsnorm_fwd(c->xn, x, w[0], n, d, cf->rms_eps);
    orc_linear_fwd(c->q, c->xn, w[1], n, d, nq);
    orc_linear_fwd(c->k, c->xn, w[2], n, d, nkv);
    orc_linear_fwd(c->v, c->xn, w[3], n, d, nkv);
    if (cf->qkv_bias) {
        orc_bias_add(c->q, w[9], n, nq);
        orc_bias_add(c->k, w[10], n, nkv);
        orc_bias_add(c->v, w[11], n, nkv);
    }
    orc_rope(c->q, B, T, Hq, hd, cf->rope_base, +1);
    orc_rope(c->k, B, T, Hkv, hd, cf->rope_base, +1);
    orc_attention_fwd(c->a, c->q, c->k, c->v, B, T, Hq, Hkv, hd);
    orc_linear_fwd(c->h1, c->a, w[4], n, nq, d);
    for (int64_t i = 0; i < n * d; ++i) c->h1[i] += x[i];
    orc_rmsnorm_fwd(c->yn, c->h1, w[5], n, d, cf->rms_eps);
    orc_linear_fwd(c->gt, c->yn, w[6], n, d, F);
    orc_linear_fwd(c->up, c->yn, w[7], n, d, F);
    orc_swiglu_fwd(c->s, c->gt, c->up, n * F);
    orc_linear_fwd(y, c->s, w[8], n, F, d);
    for (int64_t i = 0; i < n * d; ++i) y[i] += c->h1[i];
}

/* LocalBackward of Algorithm 1: from g = dl/dy to dl/dx (written to dx) and the
 * nine weight gradients (written to gw[0..8]). */
static void block_backward(real *dx, const real *dy, const real *x, const real *const *w, real *const *gw,
                           const block_cache *c, const orc_cfg *cf, int64_t B, int64_t T) {
    const int64_t n = B * T, d = cf->hidden, Hq = cf->n_q_heads, Hkv = cf->n_kv_heads, hd = cf->head_dim,
                  nq = Hq * hd, nkv = Hkv * hd, F = cf->ffn;
    real *ds = ralloc(n * F), *dgt = ralloc(n * F), *dup = ralloc(n * F);
    real *dyn = ralloc(n * d), *tmp = ralloc(n * d), *dh1 = ralloc(n * d);
    real *da = ralloc(n * nq), *dq = ralloc(n * nq), *dk = ralloc(n * nkv), *dv = ralloc(n * nkv);
    real *dxn = ralloc(n * d);

    /* y = h1 + s Wd^T */
    orc_linear_bwd_w(gw[8], dy, c->s, n, F, d);
    orc_linear_bwd_x(ds, dy, w[8], n, F, d);
    orc_swiglu_bwd(dgt, dup, ds, c->gt, c->up, n * F);
    orc_linear_bwd_w(gw[6], dgt, c->yn, n, d, F);
    orc_linear_bwd_w(gw[7], dup, c->yn, n, d, F);
    orc_linear_bwd_x(dyn, dgt, w[6], n, d, F);
    orc_linear_bwd_x(tmp, dup, w[7], n, d, F);
    for (int64_t i = 0; i < n * d; ++i) dyn[i] += tmp[i];
    orc_rmsnorm_bwd(dh1, gw[5], dyn, c->h1, w[5], n, d, cf->rms_eps);
    for (int64_t i = 0; i < n * d; ++i) dh1[i] += dy[i];
    /* h1 = x + a Wo^T */
    orc_linear_bwd_w(gw[4], dh1, c->a, n, nq, d);
    orc_linear_bwd_x(da, dh1, w[4], n, nq, d);
    orc_attention_bwd(dq, dk, dv, da, c->q, c->k, c->v, B, T, Hq, Hkv, hd);
    orc_rope(dq, B, T, Hq, hd, cf->rope_base, -1);
    orc_rope(dk, B, T, Hkv, hd, cf->rope_base, -1);
    if (cf->qkv_bias) {
        orc_bias_bwd(gw[9], dq, n, nq);
        orc_bias_bwd(gw[10], dk, n, nkv);
        orc_bias_bwd(gw[11], dv, n, nkv);
    }
    orc_linear_bwd_w(gw[1], dq, c->xn, n, d, nq);
    orc_linear_bwd_w(gw[2], dk, c->xn, n, d, nkv);
    orc_linear_bwd_w(gw[3], dv, c->xn, n, d, nkv);
    orc_linear_bwd_x(dxn, dq, w[1], n, d, nq);
    orc_linear_bwd_x(tmp, dk, w[2], n, d, nkv);
    for (int64_t i = 0; i < n * d; ++i) dxn[i] += tmp[i];
    orc_linear_bwd_x(tmp, dv, w[3], n, d, nkv);
    for (int64_t i = 0; i < n * d; ++i) dxn[i] += tmp[i];
    orc_rmsnorm_bwd(dx, gw[0], dxn, x, w[0], n, d, cf->rms_eps);
    for (int64_t i = 0; i < n * d; ++i) dx[i] += dh1[i];

    free(ds); free(dgt); free(dup); free(dyn); free(tmp); free(dh1);
    free(da); free(dq); free(dk); free(dv); free(dxn);
}

/* ------------------------------------------------------------------ the training step
 * params / grads: 9L+3 arrays in canonical order
 *   0 embed[V,d]; per layer the nine tensors above; final_norm[d]; lm_head[V,d].
 * mode 0 = monolithic (all block caches kept); mode K >= 1 = streamed, Algorithm 1 with
 * checkpoint interval K: after the forward only h_0, h_K, h_2K, ... survive (every other boundary
 * is overwritten with NaN to prove it is never read again); the backward walks the blocks of K
 * layers last to first, recomputes a block's forward from its checkpoint (keeping that block's
 * activations only) and then runs LocalBackward through the block in reverse.
 * Returns 0, or -1 for a token/label outside the vocabulary. */
int orc_train_step(const orc_cfg *cf, const real *const *params, const int32_t *tokens, const int32_t *labels,
                   int64_t B, int64_t T, real *const *grads, real *loss, int mode) {
    const int64_t L = cf->n_layers, d = cf->hidden, V = cf->vocab, n = B * T;
    const int64_t K = mode < 1 ? 1 : (mode > L ? (L > 0 ? L : 1) : mode), PL = per_layer(cf);
    for (int64_t t = 0; t < n; ++t)
        if (tokens[t] < 0 || tokens[t] >= V || labels[t] >= V) return -1;

    /* Phase 1: streaming forward */
    real **h = (real **)malloc(sizeof(real *) * (size_t)(L + 1));
    for (int64_t i = 0; i <= L; ++i) h[i] = ralloc(n * d);
    const int64_t ncache = mode == 0 ? L : K;
    block_cache *caches = (block_cache *)calloc((size_t)(ncache > 0 ? ncache : 1), sizeof(block_cache));
    for (int64_t i = 0; i < ncache; ++i) cache_alloc(&caches[i], cf, n);

    orc_embed_fwd(h[0], params[0], tokens, n, d);
    for (int64_t i = 0; i < L; ++i)
        block_forward(h[i + 1], h[i], params + 1 + PL * i, mode == 0 ? &caches[i] : &caches[0], cf, B, T);

    /* Phase 2: loss anchoring */
    const real *gf = params[1 + PL * L], *wlm = cf->tie_embeddings ? params[0] : params[2 + PL * L];
    real *zn = ralloc(n * d), *logits = ralloc(n * V), *dlogits = ralloc(n * V), *dzn = ralloc(n * d);
    real *g = ralloc(n * d), *gprev = ralloc(n * d);
    real *dhead = cf->tie_embeddings ? ralloc(V * d) : grads[2 + PL * L]; /* tied: added to the table's gradient below */
    orc_rmsnorm_fwd(zn, h[L], gf, n, d, cf->rms_eps);
    orc_linear_fwd(logits, zn, wlm, n, d, V);
    orc_cross_entropy(loss, dlogits, logits, labels, n, V);
    orc_linear_bwd_w(dhead, dlogits, zn, n, d, V);
    orc_linear_bwd_x(dzn, dlogits, wlm, n, d, V);
    orc_rmsnorm_bwd(g, grads[1 + PL * L], dzn, h[L], gf, n, d, cf->rms_eps);

    /* Phase 3: block-wise backward, last block first */
    real *ydummy = ralloc(n * d);
    if (mode == 0) {
        for (int64_t i = L - 1; i >= 0; --i) {
            block_backward(gprev, g, h[i], params + 1 + PL * i, grads + 1 + PL * i, &caches[i], cf, B, T);
            real *sw = g; g = gprev; gprev = sw;
        }
    } else {
        /* only the checkpoints are kept on the device */
        for (int64_t i = 1; i <= L; ++i)
            if (i % K != 0)
                for (int64_t e = 0; e < n * d; ++e) h[i][e] = (real)NAN;
        for (int64_t b = (L - 1) / K; b >= 0 && L > 0; --b) {
            const int64_t lo = b * K, hi = (lo + K < L ? lo + K : L) - 1; /* layers lo..hi (0-based) */
            for (int64_t i = lo; i <= hi; ++i) /* RecomputeBlock from the checkpoint h[lo] */
                block_forward(i < hi ? h[i + 1] : ydummy, h[i], params + 1 + PL * i, &caches[i - lo], cf, B, T);
            for (int64_t i = hi; i >= lo; --i) { /* LocalBackward, reverse order */
                block_backward(gprev, g, h[i], params + 1 + PL * i, grads + 1 + PL * i, &caches[i - lo], cf, B, T);
                real *sw = g; g = gprev; gprev = sw;
            }
        }
    }
    orc_embed_bwd(grads[0], g, tokens, n, V, d);
    if (cf->tie_embeddings) {
        for (int64_t i = 0; i < V * d; ++i) grads[0][i] += dhead[i];
        free(dhead);
    }

    free(ydummy); free(zn); free(logits); free(dlogits); free(dzn); free(g); free(gprev);
    for (int64_t i = 0; i < ncache; ++i) cache_free(&caches[i]);
    free(caches);
    for (int64_t i = 0; i <= L; ++i) free(h[i]);
    free(h);
    return 0;
}

/* Forward only: loss (and, if logits_out is not NULL, the [n,V] logits). */
int orc_forward_loss(const orc_cfg *cf, const real *const *params, const int32_t *tokens, const int32_t *labels,
                     int64_t B, int64_t T, real *loss, real *logits_out, real *hL_out) {
    const int64_t L = cf->n_layers, d = cf->hidden, V = cf->vocab, n = B * T, PL = per_layer(cf);
    for (int64_t t = 0; t < n; ++t)
        if (tokens[t] < 0 || tokens[t] >= V || labels[t] >= V) return -1;
    real *x = ralloc(n * d), *y = ralloc(n * d);
    block_cache scratch;
    cache_alloc(&scratch, cf, n);
    orc_embed_fwd(x, params[0], tokens, n, d);
    for (int64_t i = 0; i < L; ++i) {
        block_forward(y, x, params + 1 + PL * i, &scratch, cf, B, T);
        real *sw = x; x = y; y = sw;
    }
    if (hL_out) memcpy(hL_out, x, sizeof(real) * (size_t)(n * d));
    real *zn = ralloc(n * d), *logits = logits_out ? logits_out : ralloc(n * V);
    orc_rmsnorm_fwd(zn, x, params[1 + PL * L], n, d, cf->rms_eps);
    orc_linear_fwd(logits, zn, cf->tie_embeddings ? params[0] : params[2 + PL * L], n, d, V);
    orc_cross_entropy(loss, NULL, logits, labels, n, V);
    if (!logits_out) free(logits);
    free(zn); free(x); free(y);
    cache_free(&scratch);
    return 0;
}
