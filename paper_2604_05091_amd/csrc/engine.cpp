// The streamed training step: host-resident state, double-buffered weight streaming,
// per-block recompute + backward, asynchronous gradient offload (Algorithm 1 and
// Sections 3.2-3.4 of the MegaTrain paper), scheduled on three HIP streams.
//
// Units.  The model is cut into L+2 streamed units: E (embedding table), blocks 1..L and
// H (final norm + LM head).  Each unit owns one contiguous pinned bf16 block on the host
// (what StreamIn copies, one DMA per unit) and one contiguous fp32 gradient block (what
// Offload fills).  Inside a block the tensors are ordered
//     wq | wk | wv | wo | attn_norm | (bq | bk | bv) | mlp_norm | w_gate | w_up | w_down
// so q/k/v and gate/up form single [out,in] matrices and run as one GEMM each, and the MLP
// part is one contiguous tail: its gradients are complete half-way through the block's
// backward and leave as an early DMA of their own (gm_ready / gm_free below), the attention
// part follows at the end of the block.  The device
// "templates" are just kernels taking pointers: binding a streamed buffer is pointer
// arithmetic on the buffer base, done at launch.
//
// Streams and events.  S_comp runs kernels, S_h2d the weight copies, S_d2h the gradient
// copies.  Weight loads are numbered s = 0..2L+1 (E, 1..L, H, L..1) and use device buffer
// s % 2; gradient blocks are numbered r = 0..L+1 (H, L..1, E) and use buffer r % 2.
//   w_ready[s]  recorded on S_h2d after load s          -> S_comp waits before using it
//   w_free[s]   recorded on S_comp after its last use    -> S_h2d waits before load s+2
//   g_ready[r]  recorded on S_comp after grads r exist   -> S_d2h waits before copying
//   g_free[r]   recorded on S_d2h after the copy         -> S_comp waits before grads r+2
//   gm_ready[r] / gm_free[r]: the same pair for the early MLP piece of a layer's block; the host
//   optimizer waits for gm_free[r] or g_free[r], whichever covers the tensors it updates next
// The paper names three of these (Weights-Ready, Backward-Done, Buffer-Free); w_free is the
// event behind its "Release(theta_i)".
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <memory>
#include <chrono>
#include <string>
#include <vector>
#include <condition_variable>
#include <deque>
#include <functional>
#include <set>
#include <mutex>
#include <thread>

#include "../../include/megatrain.h"
#include "common.h"
#include "host_ops.h"

using namespace mt;

namespace {

thread_local char g_err[512] = "";

mt_status fail(mt_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIPCHK(expr)                                                                                  \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return fail(MT_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

double now_ms() {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

struct Dims {
    int L, d, Hq, Hkv, hd, F, V;
    int64_t Nq, Nkv, Nqkv;
    int bias = 0;  // q, k, v projections carry biases
    int PL = 9;    // tensors per layer in the canonical order
    int tied = 0;  // the output projection reuses the embedding table (no lm_head tensor)
    int n_tensors() const { return PL * L + (tied ? 2 : 3); }
};

struct TensorRef {
    int unit;        // which streamed unit
    size_t off;      // element offset inside the unit block
    size_t numel;
};

struct Unit {
    size_t numel = 0;
    uint16_t *h_shadow = nullptr;  // pinned bf16 block
    float *h_grad = nullptr;       // fp32 gradient block: pinned, or pageable when the slab pool is in use
};

// element offsets inside a block unit
struct LayerOff {
    size_t wqkv, wo, wgu, wd, g1, g2, bqkv, total;  // bqkv: bq | bk | bv (only with biases)
    size_t mlp;  // first element of the MLP part (g2 | wgu | wd), which ends the block
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

mt_status check_cfg(const mt_model_cfg *c) {
    if (!c) return fail(MT_ERR_INVALID_ARG, "cfg is NULL");
    if (c->struct_size != sizeof(mt_model_cfg)) return fail(MT_ERR_INVALID_ARG, "cfg.struct_size mismatch");
    if (c->abi_version != MT_ABI_VERSION) return fail(MT_ERR_INVALID_ARG, "cfg.abi_version mismatch");
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->ffn <= 0 || c->vocab <= 0)
        return fail(MT_ERR_INVALID_ARG, "model dimensions must be positive");
    if (c->n_q_heads % c->n_kv_heads) return fail(MT_ERR_INVALID_ARG, "n_q_heads must be a multiple of n_kv_heads");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(MT_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if ((c->hidden & 7) || (c->ffn & 7) || (c->vocab & 7))
        return fail(MT_ERR_UNSUPPORTED, "hidden, ffn and vocab must be multiples of 8");
    if (c->hidden > 8192) return fail(MT_ERR_UNSUPPORTED, "hidden > 8192 is not supported");
    if (c->ckpt_interval < 1) return fail(MT_ERR_INVALID_ARG, "ckpt_interval must be >= 1");
    if (c->mlp_chunk & 7) return fail(MT_ERR_INVALID_ARG, "mlp_chunk must be a multiple of 8");
    if (!(c->rope_base > 0.f) || !(c->rms_eps > 0.f)) return fail(MT_ERR_INVALID_ARG, "rope_base and rms_eps must be > 0");
    return MT_OK;
}

Dims dims_of(const mt_model_cfg *c) {
    Dims D;
    D.L = c->n_layers; D.d = c->hidden; D.Hq = c->n_q_heads; D.Hkv = c->n_kv_heads; D.hd = c->head_dim;
    D.F = c->ffn; D.V = c->vocab;
    D.Nq = (int64_t)D.Hq * D.hd; D.Nkv = (int64_t)D.Hkv * D.hd; D.Nqkv = D.Nq + 2 * D.Nkv;
    D.bias = c->qkv_bias ? 1 : 0;
    D.PL = D.bias ? 12 : 9;
    D.tied = c->tie_embeddings ? 1 : 0;
    return D;
}

LayerOff layer_off(const Dims &D) {
    // attention part first, MLP part last: the MLP gradients are complete half-way through a block's backward and
    // leave for the host as one contiguous piece while the attention part is still being computed
    LayerOff o;
    o.wqkv = 0;
    o.wo = o.wqkv + (size_t)D.Nqkv * D.d;
    o.g1 = o.wo + (size_t)D.d * D.Nq;
    o.bqkv = o.g1 + D.d;
    o.g2 = o.bqkv + (D.bias ? (size_t)D.Nqkv : 0);
    o.mlp = o.g2;
    o.wgu = o.g2 + D.d;
    o.wd = o.wgu + (size_t)2 * D.F * D.d;
    o.total = o.wd + (size_t)D.d * D.F;
    return o;
}

void tensor_shape(const Dims &D, int idx, int64_t *rows, int64_t *cols, std::string *name) {
    auto set = [&](int64_t r, int64_t c, const std::string &s) {
        *rows = r; *cols = c;
        if (name) *name = s;
    };
    if (idx == 0) return set(D.V, D.d, "embed");
    if (idx == 1 + D.PL * D.L) return set(D.d, 1, "final_norm");
    if (idx == 2 + D.PL * D.L) return set(D.V, D.d, "lm_head");
    const int l = (idx - 1) / D.PL, k = (idx - 1) % D.PL;
    const std::string p = "l" + std::to_string(l) + ".";
    switch (k) {
        case 0: return set(D.d, 1, p + "attn_norm");
        case 1: return set(D.Nq, D.d, p + "wq");
        case 2: return set(D.Nkv, D.d, p + "wk");
        case 3: return set(D.Nkv, D.d, p + "wv");
        case 4: return set(D.d, D.Nq, p + "wo");
        case 5: return set(D.d, 1, p + "mlp_norm");
        case 6: return set(D.F, D.d, p + "w_gate");
        case 7: return set(D.F, D.d, p + "w_up");
        case 8: return set(D.d, D.F, p + "w_down");
        case 9: return set(D.Nq, 1, p + "bq");
        case 10: return set(D.Nkv, 1, p + "bk");
        default: return set(D.Nkv, 1, p + "bv");
    }
}

}  // namespace

struct mt_handle {
    mt_model_cfg cfg;
    Dims D;
    LayerOff lo;
    int n_tensors = 0;
    std::vector<float *> params;      // caller-owned fp32 master
    std::vector<TensorRef> tref;      // where each tensor lives inside its unit
    std::vector<Unit> units;          // 0 = E, 1..L = blocks, L+1 = H
    std::vector<float *> adam_m, adam_v;  // per unit, pageable
    size_t pmax = 0;                  // largest unit, elements

    // device
    char *arena = nullptr;
    size_t arena_bytes = 0;
    uint16_t *Wbuf[2] = {nullptr, nullptr};
    float *Gbuf[2] = {nullptr, nullptr};
    // Block boundaries (Algorithm 1, checkpoint interval K): h_i with i % K == 0 are checkpoints that
    // live through the step; the other boundaries of the block in flight share K-1 buffers.
    int K = 1;
    std::vector<uint16_t *> anchors;  // h_0, h_K, h_2K, ...
    std::vector<uint16_t *> blk_h;    // h_i, i % K = 1 .. K-1 of the current block
    uint16_t *boundary(int i) const { return i % K == 0 ? anchors[i / K] : blk_h[i % K - 1]; }
    // One layer's saved activations; K sets, one per layer of a recomputation block.  xn .. lse below are
    // the set the kernels currently work on (select_acts).
    struct ActSet { uint16_t *xn, *yn, *qkv, *att, *h1, *gu, *sact; float *lse; };
    std::vector<ActSet> acts;
    void select_acts(int slot) {
        const ActSet &a = acts[slot];
        xn = a.xn; yn = a.yn; qkv = a.qkv; att = a.att; h1 = a.h1; gu = a.gu; sact = a.sact; lse = a.lse;
    }
    uint16_t *xn, *yn, *qkv, *att, *h1, *gu, *sact;
    uint16_t *dsact, *dgu, *dyn, *dh1, *datt, *dqkv, *dxn, *gA, *gB, *tA, *tB, *wT, *wT2;
    int64_t mlp_rows = 0;  // rows of the MLP buffers: all tokens, or cfg.mlp_chunk
    bool mlp_chunked = false;
    uint16_t *dlogits, *dlT;
    float *lse, *delta, *logits, *loss_rows, *loss_dev, *norm_ws, *bias_ws, *rope_cos, *rope_sin;
    float *split_ws = nullptr;   // partial results of weight-gradient products whose reduction is split
    size_t split_ws_floats = 0;
    int n_cu = 256;
    int32_t *tok_dev, *lab_dev, *rowstart_dev, *order_dev;
    int64_t ce_chunk = 0;
    // gradient slab pool (Section 3.3 / Appendix A.3): when the fp32 gradient blocks cannot all be pinned,
    // they live in pageable memory and every device-to-host copy lands in one of n_slabs pinned slabs of
    // P_max floats first; a host thread then folds the slab into the unit's gradient block and recycles it.
    bool grad_slabs = false;
    int n_slabs = 0;
    std::vector<float *> slabs;
    // staged weights (Section 3.3, layer-contiguous tiling with pinned slab recycling): no persistent bf16
    // copy; a host thread converts the fp32 master tensors of the unit to be streamed next into one of a
    // few pinned slabs of P_max bf16 elements just in time, and the H2D copy reads the slab.
    bool staged = false;
    std::vector<uint16_t *> wslabs;

    // pinned staging
    int32_t *tok_host = nullptr;  // tokens | labels | row_start | order
    float *loss_host = nullptr;

    hipStream_t s_comp = nullptr, s_h2d = nullptr, s_d2h = nullptr;
    std::vector<hipEvent_t> w_ready, w_free, g_ready, g_free, h2d_start, comp_start, d2h_start;
    std::vector<hipEvent_t> gm_ready, gm_free, d2hm_start;  // the same three for a block's early (MLP) gradient piece
    std::vector<hipEvent_t> sub_copied;  // copy-done events of the sub-ranges a large gradient piece is cut into (grown on demand)
    hipEvent_t ev_ref = nullptr, ev_inputs = nullptr;
    int resident[2] = {-1, -1};

    // optional per-kernel-class timing (MT_FLAG_KERNEL_TIMING): event pairs around launches on S_comp
    struct Span { hipEvent_t a, b; int cls; double flops, bytes; };
    std::vector<Span> spans;
    size_t spans_used = 0;
    bool timing = false;

    mt_stats stats;
    bool have_grads = false;
    // an overlapped step (mt_train_step_adam) failed after its host worker had started: some units may carry this
    // step's Adam update and others not.  Optimizer calls are refused until mt_refresh_shadow acknowledges it.
    bool opt_partial = false;
    size_t pinned_bytes = 0, pageable_bytes = 0;
};

namespace {

// ------------------------------------------------------------------ small launch helpers
#define KCHK(expr)                                                                                   \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return fail(MT_ERR_HIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

enum { CLS_GEMM = 0, CLS_ATTN_FWD = 1, CLS_ATTN_BWD = 2, CLS_COUNT = 3 };

// Brackets a launch with two events when kernel timing is on.
struct Timed {
    mt_handle *h;
    mt_handle::Span *sp = nullptr;
    Timed(mt_handle *h_, int cls, double flops, double bytes) : h(h_) {
        if (!h->timing) return;
        if (h->spans_used == h->spans.size()) {
            mt_handle::Span n{nullptr, nullptr, 0, 0.0, 0.0};
            if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess) return;
            h->spans.push_back(n);
        }
        sp = &h->spans[h->spans_used++];
        sp->cls = cls;
        sp->flops = flops;
        sp->bytes = bytes;
        (void)hipEventRecord(sp->a, h->s_comp);
    }
    ~Timed() {
        if (sp) (void)hipEventRecord(sp->b, h->s_comp);
    }
};

hipError_t gemm_raw(hipStream_t s, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, void *C, int64_t ldc,
                int64_t M, int64_t N, int64_t K, bool out_fp32 = false, bool accumulate = false,
                const uint16_t *R = nullptr, int64_t ldr = 0, const uint16_t *bias = nullptr) {
    GemmArgs g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.R = R; g.ldr = ldr;
    g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K;
    g.out_fp32 = out_fp32; g.accumulate = accumulate;
    g.bias = bias;
    return gemm_nt(g, s);
}

hipError_t gemm(mt_handle *h, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, void *C, int64_t ldc,
                int64_t M, int64_t N, int64_t K, bool out_fp32 = false, bool accumulate = false,
                const uint16_t *R = nullptr, int64_t ldr = 0, const uint16_t *bias = nullptr) {
    // algorithmic bytes: both operands once, the result once (plus the residual / the accumulated-into result read)
    const double out_b = out_fp32 ? 4.0 : 2.0;
    const double bytes = 2.0 * ((double)M * K + (double)N * K) + (double)M * N * (out_b + (R ? 2.0 : 0.0) + (accumulate ? 4.0 : 0.0));
    Timed t(h, CLS_GEMM, 2.0 * (double)M * (double)N * (double)K, bytes);
    return gemm_raw(h->s_comp, A, lda, B, ldb, C, ldc, M, N, K, out_fp32, accumulate, R, ldr, bias);
}

// qkv = xn Wqkv^T (+ b) followed by the rotary embedding of the q and k heads: in the GEMM's store where that
// kernel supports it (head_dim 128, large grids), otherwise as a pass of its own over q and k.
hipError_t qkv_projection(mt_handle *h, const uint16_t *xn, const uint16_t *wqkv, const uint16_t *bqkv, int64_t n, int T) {
    const Dims &D = h->D;
    GemmArgs g;
    g.A = xn; g.lda = D.d; g.B = wqkv; g.ldb = D.d; g.C = h->qkv; g.ldc = D.Nqkv; g.R = nullptr; g.ldr = 0;
    g.M = (int32_t)n; g.N = (int32_t)D.Nqkv; g.K = D.d;
    g.out_fp32 = 0; g.accumulate = 0;
    g.bias = bqkv;
    g.rope_cos = h->rope_cos; g.rope_sin = h->rope_sin; g.rope_T = T; g.rope_cols = (int32_t)(D.Nq + D.Nkv);
    const bool fused = D.hd == 128 && gemm_nt_fuses_rope(g);
    if (!fused) g.rope_cos = g.rope_sin = nullptr;
    {
        const double M = (double)n, N = (double)D.Nqkv, K = (double)D.d;
        Timed t(h, CLS_GEMM, 2.0 * M * N * K, 2.0 * (M * K + N * K) + 2.0 * M * N);
        const hipError_t e = gemm_nt(g, h->s_comp);
        if (e != hipSuccess) return e;
    }
    if (fused) return hipSuccess;
    return rope_inplace(h->qkv, D.Nqkv, n, T, D.Hq + D.Hkv, D.hd, h->rope_cos, h->rope_sin, +1, h->s_comp);
}

// out[cols, rows] = in[rows, cols]^T
hipError_t transpose2d(hipStream_t s, const uint16_t *in, uint16_t *out, int64_t rows, int64_t cols, int64_t ld_in,
                       int64_t ld_out) {
    TransposeArgs t;
    t.in = in; t.out = out; t.rows = (int32_t)rows; t.cols = (int32_t)cols; t.ld_in = ld_in; t.ld_out = ld_out;
    t.nb0 = 1; t.nb1 = 1; t.in_s0 = t.in_s1 = t.out_s0 = t.out_s1 = 0;
    return transpose_bf16(t, s);
}

#define WG(expr)                      \
    do {                              \
        const mt_status st_ = (expr); \
        if (st_ != MT_OK) return st_; \
    } while (0)

// Weight gradient dW[out,in] (fp32, row pitch in) (+)= dY^T X from token-major dY [rows, out] (ldy) and
// X [rows, in] (ldx).  Taken straight from the operands when the token count allows it, otherwise through
// transposed copies (tA, tB) and the general kernel.
mt_status weight_grad(mt_handle *h, const uint16_t *dY, int64_t ldy, const uint16_t *X, int64_t ldx, float *dW,
                      int64_t out, int64_t in, int64_t rows, bool accumulate) {
    hipStream_t s = h->s_comp;
    if (rows % 64 == 0 && !(out & 7) && !(in & 7)) {
        GemmArgs g;
        g.A = dY; g.lda = ldy; g.B = X; g.ldb = ldx; g.C = dW; g.ldc = in; g.R = nullptr; g.ldr = 0;
        g.M = (int32_t)out; g.N = (int32_t)in; g.K = (int32_t)rows;
        g.out_fp32 = 1; g.accumulate = accumulate;
        // tile counts that fill the last round of workgroups badly: split the reduction (deterministic, fixed order)
        int sp = gemm_tn_pick_split(out, in, rows, h->n_cu);
        while (sp > 1 && (size_t)(sp - 1) * (size_t)out * (size_t)in > h->split_ws_floats) --sp;
        if ((in & 3) || ((uintptr_t)dW & 15)) sp = 1;
        g.split_k = sp;
        g.split_ws = h->split_ws;
        const double bytes = 2.0 * ((double)out * rows + (double)in * rows) + (double)out * in * (accumulate ? 8.0 : 4.0);
        Timed t(h, CLS_GEMM, 2.0 * (double)out * (double)in * (double)rows, bytes);
        KCHK(gemm_tn(g, s));
        return MT_OK;
    }
    KCHK(transpose2d(s, dY, h->tA, rows, out, ldy, rows));
    KCHK(transpose2d(s, X, h->tB, rows, in, ldx, rows));
    KCHK(gemm(h, h->tA, rows, h->tB, rows, dW, in, out, in, rows, true, accumulate));
    return MT_OK;
}

struct LayerW {
    const uint16_t *wqkv, *wo, *wgu, *wd, *g1, *g2, *bqkv;  // bqkv = NULL without biases
};
LayerW bind_layer(const uint16_t *base, const LayerOff &o) {
    return {base + o.wqkv, base + o.wo, base + o.wgu, base + o.wd, base + o.g1, base + o.g2,
            o.g2 > o.bqkv ? base + o.bqkv : nullptr};  // the bias slot is empty without biases
}

AttnArgs attn_args(const mt_handle *h, int B, int T) {
    const Dims &D = h->D;
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    a.B = B; a.T = T; a.Hq = D.Hq; a.Hkv = D.Hkv; a.hd = D.hd;
    a.scale = 1.0f / sqrtf((float)D.hd);
    a.q = h->qkv; a.ldq = D.Nqkv;
    a.k = h->qkv + D.Nq; a.ldk = D.Nqkv;
    a.v = h->qkv + D.Nq + D.Nkv; a.ldv = D.Nqkv;
    a.o = h->att; a.ldo = D.Nq;
    a.lse = h->lse;
    a.dout = h->datt; a.lddo = D.Nq;
    a.delta = h->delta;
    a.dq = h->dqkv; a.lddq = D.Nqkv;
    a.dk = h->dqkv + D.Nq; a.lddk = D.Nqkv;
    a.dv = h->dqkv + D.Nq + D.Nkv; a.lddv = D.Nqkv;
    return a;
}

// yn, sact and (keep_gu: what the backward reads) gu of m rows starting at h1: the block's MLP up to the activation.
// The activation is computed in the store of the gate|up GEMM where that kernel supports it (large grids, ffn a
// multiple of 128), otherwise by a pass of its own over gu.
mt_status mlp_forward_rows(mt_handle *h, const LayerW &w, const uint16_t *h1, int64_t m, bool keep_gu) {
    const Dims &D = h->D;
    hipStream_t s = h->s_comp;
    KCHK(rmsnorm_fwd(h->yn, h1, w.g2, m, D.d, h->cfg.rms_eps, s));
    GemmArgs g;
    g.A = h->yn; g.lda = D.d; g.B = w.wgu; g.ldb = D.d; g.C = keep_gu ? h->gu : nullptr; g.ldc = 2 * D.F;
    g.R = nullptr; g.ldr = 0;
    g.M = (int32_t)m; g.N = 2 * D.F; g.K = D.d;
    g.out_fp32 = 0; g.accumulate = 0;
    g.glu_F = D.F; g.glu_out = h->sact; g.ld_glu = D.F;
    // Measured on the 7B shape: plain GEMM 9.6 ms, GEMM + SwiGLU kernel 10.35 ms, fused with the activation only
    // 9.55 ms, fused with gate | up stored as well (what the backward reads) 9.8 ms.
    if (gemm_nt_fuses_glu(g)) {
        const double M = (double)m, N = 2.0 * D.F, K = (double)D.d;
        Timed t(h, CLS_GEMM, 2.0 * M * N * K, 2.0 * (M * K + N * K) + (keep_gu ? 3.0 : 1.0) * M * N);
        KCHK(gemm_nt(g, s));
        return MT_OK;
    }
    KCHK(gemm(h, h->yn, D.d, w.wgu, D.d, h->gu, 2 * D.F, m, 2 * D.F, D.d));
    KCHK(swiglu_fwd(h->sact, h->gu, m, D.F, s));
    return MT_OK;
}

// f_i of Algorithm 1.  y may be NULL (recompute before backward does not need the block output).
// keep_internals: the block's backward follows (recomputation), so everything it reads has to be stored;
// the streaming forward only needs the block output.
mt_status layer_forward(mt_handle *h, const LayerW &w, const uint16_t *x, uint16_t *y, int B, int T, bool keep_internals) {
    const Dims &D = h->D;
    const int64_t n = (int64_t)B * T;
    hipStream_t s = h->s_comp;
    KCHK(rmsnorm_fwd(h->xn, x, w.g1, n, D.d, h->cfg.rms_eps, s));
    KCHK(qkv_projection(h, h->xn, w.wqkv, w.bqkv, n, T));
    const AttnArgs a = attn_args(h, B, T);
    {
        Timed t(h, CLS_ATTN_FWD, 2.0 * (double)B * D.Hq * D.hd * (double)T * ((double)T + 1.0),
                2.0 * (double)B * T * (2.0 * D.Nq + 2.0 * D.Nkv));
        KCHK(flash_fwd(a, s));
    }
    KCHK(gemm(h, h->att, D.Nq, w.wo, D.Nq, h->h1, D.d, n, D.d, D.Nq, false, false, x, D.d));
    // MLP, in chunks of mlp_rows tokens (one chunk unless cfg.mlp_chunk is set).  A chunked MLP saves nothing for
    // the backward, so the recomputation pass (y == NULL) skips it.
    if (h->mlp_chunked && !y) return MT_OK;
    for (int64_t r0 = 0; r0 < n; r0 += h->mlp_rows) {
        const int64_t m = std::min(h->mlp_rows, n - r0);
        {
            const mt_status st = mlp_forward_rows(h, w, h->h1 + r0 * D.d, m, keep_internals && !h->mlp_chunked);
            if (st != MT_OK) return st;
        }
        if (y) KCHK(gemm(h, h->sact, D.F, w.wd, D.F, y + r0 * D.d, D.d, m, D.d, D.F, false, false, h->h1 + r0 * D.d, D.d));
    }
    return MT_OK;
}

// LocalBackward of Algorithm 1: the block's internals are in the work buffers (just recomputed).
// gy = dl/dy, gx receives dl/dx; fp32 weight gradients go to G (unit layout).
// mlp_grads_done is called once the MLP part of G (gain, gate/up and down weights) is complete.
mt_status layer_backward(mt_handle *h, const LayerW &w, float *G, const uint16_t *x, const uint16_t *gy, uint16_t *gx,
                         int B, int T, const std::function<mt_status()> &mlp_grads_done) {
    const Dims &D = h->D;
    const LayerOff &o = h->lo;
    const int64_t n = (int64_t)B * T;
    hipStream_t s = h->s_comp;
    // MLP: y = h1 + s Wd^T, gu = yn Wgu^T, in chunks of mlp_rows tokens.  Weight and gain gradients of the second
    // and later chunks are added to the first chunk's; a chunked MLP is recomputed chunk by chunk here.
    KCHK(transpose2d(s, w.wd, h->wT, D.d, D.F, D.F, D.d));
    KCHK(transpose2d(s, w.wgu, h->wT2, 2 * D.F, D.d, D.d, 2 * D.F));
    for (int64_t r0 = 0; r0 < n; r0 += h->mlp_rows) {
        const int64_t m = std::min(h->mlp_rows, n - r0);
        const bool acc = r0 > 0;
        const uint16_t *gyc = gy + r0 * D.d, *h1c = h->h1 + r0 * D.d;
        if (h->mlp_chunked) {
            const mt_status st = mlp_forward_rows(h, w, h1c, m, true);
            if (st != MT_OK) return st;
        }
        WG(weight_grad(h, gyc, D.d, h->sact, D.F, G + o.wd, D.d, D.F, m, acc));
        {
            // ds = gy Wd, then the SwiGLU backward: in the GEMM's store where that kernel supports it
            GemmArgs g;
            g.A = gyc; g.lda = D.d; g.B = h->wT; g.ldb = D.d; g.C = h->dgu; g.ldc = 2 * D.F; g.R = nullptr; g.ldr = 0;
            g.M = (int32_t)m; g.N = D.F; g.K = D.d;
            g.out_fp32 = 0; g.accumulate = 0;
            g.glu_bwd_gu = h->gu; g.ld_glu_bwd = 2 * D.F;
            if (gemm_nt_fuses_glu_bwd(g)) {
                const double M = (double)m, N = (double)D.F, K = (double)D.d;
                Timed t(h, CLS_GEMM, 2.0 * M * N * K, 2.0 * (M * K + N * K) + 8.0 * M * N);
                KCHK(gemm_nt(g, s));
            } else {
                KCHK(gemm(h, gyc, D.d, h->wT, D.d, h->dsact, D.F, m, D.F, D.d));
                KCHK(swiglu_bwd(h->dgu, h->dsact, h->gu, m, D.F, s));
            }
        }
        WG(weight_grad(h, h->dgu, 2 * D.F, h->yn, D.d, G + o.wgu, 2 * D.F, D.d, m, acc));
        KCHK(gemm(h, h->dgu, 2 * D.F, h->wT2, 2 * D.F, h->dyn, D.d, m, D.d, 2 * D.F));
        KCHK(rmsnorm_bwd(h->dh1 + r0 * D.d, G + o.g2, h->dyn, h1c, w.g2, gyc, h->norm_ws, m, D.d, h->cfg.rms_eps, s, acc));
    }
    {
        const mt_status st = mlp_grads_done();
        if (st != MT_OK) return st;
    }
    // h1 = x + att Wo^T
    WG(weight_grad(h, h->dh1, D.d, h->att, D.Nq, G + o.wo, D.d, D.Nq, n, false));
    KCHK(transpose2d(s, w.wo, h->wT, D.d, D.Nq, D.Nq, D.d));
    KCHK(gemm(h, h->dh1, D.d, h->wT, D.d, h->datt, D.Nq, n, D.Nq, D.d));
    // attention
    AttnArgs a = attn_args(h, B, T);
    a.rope_cos = h->rope_cos;  // dq and dk leave the kernels already rotated back
    a.rope_sin = h->rope_sin;
    KCHK(attn_delta(h->delta, h->datt, D.Nq, h->att, D.Nq, B, T, D.Hq, D.hd, s));
    {
        // 7 tile products (4 in the dK/dV kernel, 3 in the dQ kernel), causal half of T^2
        Timed t(h, CLS_ATTN_BWD, 7.0 * (double)B * D.Hq * D.hd * (double)T * ((double)T + 1.0),
                2.0 * (double)B * T * (4.0 * D.Nq + 4.0 * D.Nkv));
        KCHK(flash_bwd_dkdv(a, s));
        KCHK(flash_bwd_dq(a, s));
    }
    if (D.bias) KCHK(bias_grad(G + o.bqkv, h->dqkv, D.Nqkv, n, (int32_t)D.Nqkv, h->bias_ws, s));
    // qkv = xn Wqkv^T + b
    WG(weight_grad(h, h->dqkv, D.Nqkv, h->xn, D.d, G + o.wqkv, D.Nqkv, D.d, n, false));
    KCHK(transpose2d(s, w.wqkv, h->wT, D.Nqkv, D.d, D.d, D.Nqkv));
    KCHK(gemm(h, h->dqkv, D.Nqkv, h->wT, D.Nqkv, h->dxn, D.d, n, D.d, D.Nqkv));
    KCHK(rmsnorm_bwd(gx, G + o.g1, h->dxn, x, w.g1, h->dh1, h->norm_ws, n, D.d, h->cfg.rms_eps, s));
    return MT_OK;
}

// Phase 2 of Algorithm 1: loss, g_L and the head gradients, in token chunks so the logits stay small.
mt_status head_forward_backward(mt_handle *h, const uint16_t *W, float *G, const uint16_t *x, uint16_t *gx, int64_t n,
                                float inv_n) {
    const Dims &D = h->D;
    hipStream_t s = h->s_comp;
    const uint16_t *wlm = W, *gf = W + (size_t)D.V * D.d;
    float *dWlm = G, *dgf = G + (size_t)D.V * D.d;
    uint16_t *zn = h->dh1, *dzn = h->dxn;  // backward temporaries: the activation sets hold the last block's internals
    KCHK(rmsnorm_fwd(zn, x, gf, n, D.d, h->cfg.rms_eps, s));
    KCHK(transpose2d(s, wlm, h->wT, D.V, D.d, D.d, D.V));   // [d, V]
    for (int64_t c0 = 0; c0 < n; c0 += h->ce_chunk) {
        const int64_t rows = std::min<int64_t>(h->ce_chunk, n - c0);
        KCHK(gemm(h, zn + c0 * D.d, D.d, wlm, D.d, h->logits, D.V, rows, D.V, D.d, true));
        KCHK(cross_entropy(h->loss_rows + c0, h->dlogits, h->logits, h->lab_dev + c0, rows, D.V, inv_n, s));
        KCHK(gemm(h, h->dlogits, D.V, h->wT, D.V, dzn + c0 * D.d, D.d, rows, D.d, D.V));
        if (rows % 64 == 0) {
            WG(weight_grad(h, h->dlogits, D.V, zn + c0 * D.d, D.d, dWlm, D.V, D.d, rows, c0 > 0));
        } else {  // ragged chunk: transposed copies (dlT holds [V, rows], tB [d, rows])
            KCHK(transpose2d(s, h->dlogits, h->dlT, rows, D.V, D.V, rows));
            KCHK(transpose2d(s, zn + c0 * D.d, h->tB, rows, D.d, D.d, rows));
            KCHK(gemm(h, h->dlT, rows, h->tB, rows, dWlm, D.d, D.V, D.d, rows, true, c0 > 0));
        }
    }
    KCHK(reduce_sum(h->loss_dev, h->loss_rows, n, inv_n, 0, s));
    KCHK(rmsnorm_bwd(gx, dgf, dzn, x, gf, nullptr, h->norm_ws, n, D.d, h->cfg.rms_eps, s));
    return MT_OK;
}

void build_shadow(mt_handle *h) {
    h->resident[0] = h->resident[1] = -1;
    if (h->staged) return;  // nothing persistent to rebuild: every step converts from the master copy
    for (int i = 0; i < h->n_tensors; ++i) {
        const TensorRef &t = h->tref[i];
        host_f32_to_bf16(h->units[t.unit].h_shadow + t.off, h->params[i], t.numel);
    }
    h->resident[0] = h->resident[1] = -1;
}

void free_handle(mt_handle *h) {
    if (!h) return;
    (void)hipSetDevice(h->cfg.device_id);
    (void)hipDeviceSynchronize();
    auto kill_events = [](std::vector<hipEvent_t> &v) {
        for (auto e : v)
            if (e) (void)hipEventDestroy(e);
        v.clear();
    };
    kill_events(h->w_ready); kill_events(h->w_free); kill_events(h->g_ready); kill_events(h->g_free);
    kill_events(h->gm_ready); kill_events(h->gm_free); kill_events(h->d2hm_start); kill_events(h->sub_copied);
    kill_events(h->h2d_start); kill_events(h->comp_start); kill_events(h->d2h_start);
    for (auto &sp : h->spans) {
        if (sp.a) (void)hipEventDestroy(sp.a);
        if (sp.b) (void)hipEventDestroy(sp.b);
    }
    if (h->ev_ref) (void)hipEventDestroy(h->ev_ref);
    if (h->ev_inputs) (void)hipEventDestroy(h->ev_inputs);
    if (h->s_comp) (void)hipStreamDestroy(h->s_comp);
    if (h->s_h2d) (void)hipStreamDestroy(h->s_h2d);
    if (h->s_d2h) (void)hipStreamDestroy(h->s_d2h);
    if (h->arena) (void)hipFree(h->arena);
    for (auto &u : h->units) {
        if (u.h_shadow) (void)hipHostFree(u.h_shadow);
        if (u.h_grad) {
            if (h->grad_slabs) free(u.h_grad);
            else (void)hipHostFree(u.h_grad);
        }
    }
    for (auto p : h->slabs)
        if (p) (void)hipHostFree(p);
    for (auto p : h->wslabs)
        if (p) (void)hipHostFree(p);
    for (auto p : h->adam_m) free(p);
    for (auto p : h->adam_v) free(p);
    if (h->tok_host) (void)hipHostFree(h->tok_host);
    if (h->loss_host) (void)hipHostFree(h->loss_host);
    delete h;
}

// interval arithmetic for the overlap statistics
struct Iv { double a, b; };
double overlap_with_union(const std::vector<Iv> &xs, std::vector<Iv> busy) {
    std::sort(busy.begin(), busy.end(), [](const Iv &p, const Iv &q) { return p.a < q.a; });
    std::vector<Iv> u;
    for (const Iv &iv : busy) {
        if (iv.b <= iv.a) continue;
        if (!u.empty() && iv.a <= u.back().b) u.back().b = std::max(u.back().b, iv.b);
        else u.push_back(iv);
    }
    double tot = 0;
    for (const Iv &x : xs)
        for (const Iv &y : u) {
            const double lo = std::max(x.a, y.a), hi = std::min(x.b, y.b);
            if (hi > lo) tot += hi - lo;
        }
    return tot;
}

struct AdamHyper {
    float lr, beta1, beta2, eps, wd;
    int64_t step;
};

// Adam on the part of a unit's tensors that lies inside [off, off + count) of its block (the update is
// elementwise, so ranges that partition the block may cut through tensors)
void adam_range(mt_handle *h, int unit, size_t off, size_t count, const AdamHyper &hp) {
    for (int i = 0; i < h->n_tensors; ++i) {
        const TensorRef &t = h->tref[i];
        if (t.unit != unit) continue;
        const size_t b = std::max(off, (size_t)t.off), e = std::min(off + count, (size_t)t.off + (size_t)t.numel);
        if (b >= e) continue;
        Unit &u = h->units[unit];
        host_adam(h->params[i] + (b - t.off), u.h_grad + b, h->adam_m[unit] + b, h->adam_v[unit] + b,
                  u.h_shadow ? u.h_shadow + b : nullptr, e - b, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.wd, hp.step);
    }
}

// Host optimizer running beside the GPU (Algorithm 1, optimizer phase; Section 3.3: a background CPU thread
// applies the update as gradient blocks land).  The step pushes
// (copy-done event, unit u, element range) right after enqueueing a device-to-host copy of gradients; the worker
// waits for that event and updates the tensors of the unit inside the range.  A unit's weights are never streamed again in the same
// step once its gradients exist, so updating its master copy and bf16 copy in place is safe.
class HostWorker {
  public:
    // opt == nullptr: no optimizer, the worker only drains gradient slabs
    HostWorker(mt_handle *h, const AdamHyper *opt) : h_(h), has_opt_(opt != nullptr), slab_busy_(h->n_slabs, 0) {
        if (opt) hp_ = *opt;
        th_ = std::thread([this] { run(); });
    }
    ~HostWorker() { finish(true); }
    // main thread, slab mode: block until the slab is drained; false if the worker failed or was aborted
    bool acquire_slab(int slab) {
        std::unique_lock<std::mutex> lk(mu_);
        cv_main_.wait(lk, [&] { return !slab_busy_[slab] || failed_ || abort_; });
        if (failed_ || abort_) return false;
        slab_busy_[slab] = 1;
        return true;
    }
    // add = true: the slab is added to the gradient block instead of replacing it (micro-batch accumulation)
    // run_adam = false: only land the gradient (a tied table's head part; its update follows the embedding part)
    void push(hipEvent_t copied, int unit, size_t off, size_t count, int slab, bool add, bool run_adam) {
        {
            std::lock_guard<std::mutex> lk(mu_);
            q_.push_back({copied, unit, off, count, slab, add, run_adam});
        }
        cv_.notify_one();
    }
    // abort = true drops whatever has not started yet
    double finish(bool abort) {
        if (th_.joinable()) {
            {
                std::lock_guard<std::mutex> lk(mu_);
                done_ = true;
                abort_ = abort_ || abort;
            }
            cv_.notify_one();
            cv_main_.notify_all();
            th_.join();
        }
        return busy_ms_;
    }
    bool failed() const { return failed_; }

  private:
    struct Item { hipEvent_t copied; int unit; size_t off, count; int slab; bool add, run_adam; };
    void run() {
        if (hipSetDevice(h_->cfg.device_id) != hipSuccess) set_failed();
        for (;;) {
            Item item;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [this] { return done_ || !q_.empty(); });
                if (abort_ || (q_.empty() && done_)) return;
                item = q_.front();
                q_.pop_front();
            }
            if (failed_) continue;
            if (hipEventSynchronize(item.copied) != hipSuccess) {
                (void)hipGetLastError();
                set_failed();
                continue;
            }
            const double t0 = now_ms();
            if (item.slab >= 0) {
                // "Acc" of the paper's slab pool: fold the slab into the master gradient store, then recycle it
                Unit &u = h_->units[item.unit];
                const char *src = reinterpret_cast<const char *>(h_->slabs[item.slab]);
                char *dst = reinterpret_cast<char *>(u.h_grad + item.off);
                if (item.add) {
                    const float *sf = h_->slabs[item.slab];
                    float *df = u.h_grad + item.off;
                    parallel_for(item.count, 1 << 20, [&](size_t b, size_t e) {
                        for (size_t i = b; i < e; ++i) df[i] += sf[i];
                    });
                } else {
                    parallel_for(item.count * sizeof(float), 1 << 22, [&](size_t b, size_t e) { memcpy(dst + b, src + b, e - b); });
                }
                {
                    std::lock_guard<std::mutex> lk(mu_);
                    slab_busy_[item.slab] = 0;
                }
                cv_main_.notify_all();
            }
            if (has_opt_ && item.run_adam) adam_range(h_, item.unit, item.off, item.count, hp_);
            busy_ms_ += now_ms() - t0;
        }
    }
    void set_failed() {
        {
            std::lock_guard<std::mutex> lk(mu_);
            failed_ = true;
        }
        cv_main_.notify_all();
    }
    mt_handle *h_;
    bool has_opt_;
    AdamHyper hp_ = {};
    std::mutex mu_;
    std::condition_variable cv_, cv_main_;
    std::deque<Item> q_;
    std::vector<char> slab_busy_;
    bool done_ = false, abort_ = false, failed_ = false;
    double busy_ms_ = 0;
    std::thread th_;
};

// Just-in-time packing of streamed weights (Section 3.3; Appendix A.2): a host thread converts the fp32
// master tensors of a unit into a pinned bf16 slab while the GPU works on earlier units.  The main thread
// requests load s (slab = running count of requests modulo the number of slabs), later waits for it,
// enqueues the host-to-device copy and reports that; before a slab is reused the worker waits for the
// w_ready event of the load that last read it.
class PackWorker {
  public:
    explicit PackWorker(mt_handle *h) : h_(h), slab_user_(h->wslabs.size(), -1) { th_ = std::thread([this] { run(); }); }
    ~PackWorker() { finish(); }
    // pieces: (unit, element offset of that unit's image inside the slab)
    int request(int s, const std::vector<std::pair<int, size_t>> &pieces) {
        const int slab = (int)(n_req_++ % h_->wslabs.size());
        {
            std::lock_guard<std::mutex> lk(mu_);
            q_.push_back({s, slab, pieces});
        }
        cv_.notify_all();
        return slab;
    }
    bool wait_packed(int s) {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return packed_.count(s) || failed_; });
        return !failed_;
    }
    void copy_enqueued(int s) {
        {
            std::lock_guard<std::mutex> lk(mu_);
            enqueued_.insert(s);
        }
        cv_.notify_all();
    }
    void finish() {
        if (!th_.joinable()) return;
        {
            std::lock_guard<std::mutex> lk(mu_);
            done_ = true;
        }
        cv_.notify_all();
        th_.join();
    }
    double busy_ms() const { return busy_ms_; }

  private:
    struct Item { int s, slab; std::vector<std::pair<int, size_t>> pieces; };
    void run() {
        if (hipSetDevice(h_->cfg.device_id) != hipSuccess) return set_failed();
        for (;;) {
            Item it;
            int prev;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [this] { return done_ || !q_.empty(); });
                if (q_.empty()) return;
                it = q_.front();
                q_.pop_front();
                prev = slab_user_[it.slab];
                // the copy that last read this slab must have been enqueued before its event means anything
                if (prev >= 0) cv_.wait(lk, [&] { return done_ || enqueued_.count(prev); });
                if (prev >= 0 && !enqueued_.count(prev)) return;
                slab_user_[it.slab] = it.s;
            }
            if (prev >= 0 && hipEventSynchronize(h_->w_ready[prev]) != hipSuccess) {
                (void)hipGetLastError();
                return set_failed();
            }
            const double t0 = now_ms();
            uint16_t *dst = h_->wslabs[it.slab];
            for (const auto &pc : it.pieces)
                for (int i = 0; i < h_->n_tensors; ++i) {
                    const TensorRef &t = h_->tref[i];
                    if (t.unit == pc.first) host_f32_to_bf16(dst + pc.second + t.off, h_->params[i], t.numel);
                }
            busy_ms_ += now_ms() - t0;
            {
                std::lock_guard<std::mutex> lk(mu_);
                packed_.insert(it.s);
            }
            cv_.notify_all();
        }
    }
    void set_failed() {
        {
            std::lock_guard<std::mutex> lk(mu_);
            failed_ = true;
        }
        cv_.notify_all();
    }
    mt_handle *h_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::deque<Item> q_;
    std::set<int> packed_, enqueued_;
    std::vector<int> slab_user_;
    size_t n_req_ = 0;
    bool done_ = false, failed_ = false;
    double busy_ms_ = 0;
    std::thread th_;
};

mt_status train_step_core(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                          float *loss, const AdamHyper *opt, bool accumulate);
mt_status ensure_slabs(mt_handle *h);

}  // namespace

// ====================================================================== C ABI
extern "C" {

const char *mt_last_error(void) { return g_err; }

mt_status mt_tensor_count(const mt_model_cfg *cfg, int32_t *n) {
    if (!cfg || !n) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (cfg->n_layers <= 0) return fail(MT_ERR_INVALID_ARG, "n_layers must be positive");
    *n = dims_of(cfg).n_tensors();
    return MT_OK;
}

mt_status mt_tensor_info(const mt_model_cfg *cfg, int32_t idx, int64_t *rows, int64_t *cols, const char **name) {
    if (!cfg || !rows || !cols) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (cfg->n_layers <= 0 || idx < 0 || idx >= dims_of(cfg).n_tensors())
        return fail(MT_ERR_INVALID_ARG, "tensor index out of range");
    static thread_local std::string nm;
    const Dims D = dims_of(cfg);
    tensor_shape(D, idx, rows, cols, &nm);
    if (name) *name = nm.c_str();
    return MT_OK;
}

void *mt_host_alloc(size_t bytes) {
    void *p = nullptr;
    if (bytes == 0) return nullptr;
    if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return p;
}

void mt_host_free(void *p) {
    if (p) (void)hipHostFree(p);
}

mt_status mt_create(const mt_model_cfg *cfg, float *const *host_param_ptrs, mt_handle **out) {
    if (!out) return fail(MT_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    mt_status st = check_cfg(cfg);
    if (st != MT_OK) return st;
    if (!host_param_ptrs) return fail(MT_ERR_INVALID_ARG, "host_param_ptrs is NULL");
    if (cfg->max_batch <= 0 || cfg->max_seq <= 0) return fail(MT_ERR_INVALID_ARG, "max_batch and max_seq must be positive");
    if (cfg->max_seq & 7) return fail(MT_ERR_UNSUPPORTED, "max_seq must be a multiple of 8");
    const Dims D = dims_of(cfg);
    const int nt = D.n_tensors();
    for (int i = 0; i < nt; ++i)
        if (!host_param_ptrs[i]) return fail(MT_ERR_INVALID_ARG, "host_param_ptrs[%d] is NULL", i);
    const int64_t n = (int64_t)cfg->max_batch * cfg->max_seq;
    if (n > (int64_t)1 << 24) return fail(MT_ERR_UNSUPPORTED, "more than 2^24 tokens per step");

    mt_handle *h = new (std::nothrow) mt_handle();
    if (!h) return fail(MT_ERR_HOST_OOM, "handle allocation failed");
    h->cfg = *cfg;
    h->D = D;
    h->lo = layer_off(D);
    h->n_tensors = nt;
    h->timing = (cfg->flags & MT_FLAG_KERNEL_TIMING) != 0;
    h->params.assign(host_param_ptrs, host_param_ptrs + nt);
    memset(&h->stats, 0, sizeof(h->stats));

    // ---- unit table and where every canonical tensor sits inside its unit
    h->units.resize(D.L + 2);
    h->units[0].numel = (size_t)D.V * D.d;
    for (int l = 1; l <= D.L; ++l) h->units[l].numel = h->lo.total;
    // head unit: lm_head | final_norm; with tied embeddings only final_norm (the table is unit 0)
    h->units[D.L + 1].numel = D.tied ? (size_t)D.d : (size_t)D.V * D.d + D.d;
    h->tref.resize(nt);
    h->tref[0] = {0, 0, (size_t)D.V * D.d};
    for (int l = 0; l < D.L; ++l) {
        const int u = l + 1, b = 1 + D.PL * l;
        const LayerOff &o = h->lo;
        h->tref[b + 0] = {u, o.g1, (size_t)D.d};
        h->tref[b + 1] = {u, o.wqkv, (size_t)D.Nq * D.d};
        h->tref[b + 2] = {u, o.wqkv + (size_t)D.Nq * D.d, (size_t)D.Nkv * D.d};
        h->tref[b + 3] = {u, o.wqkv + (size_t)(D.Nq + D.Nkv) * D.d, (size_t)D.Nkv * D.d};
        h->tref[b + 4] = {u, o.wo, (size_t)D.d * D.Nq};
        h->tref[b + 5] = {u, o.g2, (size_t)D.d};
        h->tref[b + 6] = {u, o.wgu, (size_t)D.F * D.d};
        h->tref[b + 7] = {u, o.wgu + (size_t)D.F * D.d, (size_t)D.F * D.d};
        h->tref[b + 8] = {u, o.wd, (size_t)D.d * D.F};
        if (D.bias) {
            h->tref[b + 9] = {u, o.bqkv, (size_t)D.Nq};
            h->tref[b + 10] = {u, o.bqkv + (size_t)D.Nq, (size_t)D.Nkv};
            h->tref[b + 11] = {u, o.bqkv + (size_t)(D.Nq + D.Nkv), (size_t)D.Nkv};
        }
    }
    if (D.tied) {
        h->tref[nt - 1] = {D.L + 1, 0, (size_t)D.d};
    } else {
        h->tref[nt - 2] = {D.L + 1, (size_t)D.V * D.d, (size_t)D.d};
        h->tref[nt - 1] = {D.L + 1, 0, (size_t)D.V * D.d};
    }
    h->pmax = (size_t)D.V * D.d + D.d;  // the head's device image (table | final norm), also when the table is tied
    size_t total = 0;
    for (auto &u : h->units) {
        h->pmax = std::max(h->pmax, u.numel);
        total += u.numel;
    }
    h->stats.n_params = total;

    // ---- device arena plan (all offsets 256-byte aligned)
    const int64_t chunk = std::min<int64_t>(n, 8192);
    h->ce_chunk = chunk;
    size_t off = 0;
    auto plan = [&](size_t bytes) {
        const size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    const size_t e2 = sizeof(uint16_t), e4 = sizeof(float);
    const size_t wT_elems = std::max<size_t>(std::max<size_t>((size_t)2 * D.F * D.d, (size_t)D.Nqkv * D.d),
                                            std::max<size_t>((size_t)D.V * D.d, (size_t)D.d * D.Nq));
    struct ActPlan { size_t xn, yn, qkv, att, h1, gu, sact, lse; };
    struct Plan {
        size_t W[2], G[2], anchors, blk_h, dsact, dgu, dyn, dh1, datt, dqkv,
            dxn, gA, gB, tA, tB, wT, wT2, dlogits, dlT, delta, logits, loss_rows, loss_dev, norm_ws, bias_ws, split_ws, rope_cos, rope_sin,
            tok, lab, rowstart, order;
    } P;
    const int K = std::min<int>(cfg->ckpt_interval, D.L);
    h->K = K;
    const int n_ck = D.L / K + 1;
    std::vector<ActPlan> AP(K);
    for (int i = 0; i < 2; ++i) P.W[i] = plan(h->pmax * e2);
    for (int i = 0; i < 2; ++i) P.G[i] = plan(h->pmax * e4);
    P.anchors = plan((size_t)n_ck * n * D.d * e2);
    P.blk_h = plan((size_t)(K - 1) * n * D.d * e2);
    // MLP buffers hold all tokens, or one chunk; a chunked MLP keeps nothing per activation set
    h->mlp_chunked = cfg->mlp_chunk > 0 && (int64_t)cfg->mlp_chunk < n;
    const size_t mm = h->mlp_chunked ? (size_t)cfg->mlp_chunk : (size_t)n;
    h->mlp_rows = (int64_t)mm;
    for (size_t i = 0; i < AP.size(); ++i) {
        ActPlan &ap = AP[i];
        ap.xn = plan(n * D.d * e2);
        ap.qkv = plan(n * D.Nqkv * e2); ap.att = plan(n * D.Nq * e2); ap.h1 = plan(n * D.d * e2);
        ap.lse = plan((size_t)n * D.Hq * e4);
        if (h->mlp_chunked && i > 0) {
            ap.yn = AP[0].yn; ap.gu = AP[0].gu; ap.sact = AP[0].sact;
        } else {
            ap.yn = plan(mm * D.d * e2); ap.gu = plan(mm * 2 * D.F * e2); ap.sact = plan(mm * D.F * e2);
        }
    }
    P.dsact = plan(mm * D.F * e2); P.dgu = plan(mm * 2 * D.F * e2);
    P.dyn = plan(mm * D.d * e2); P.dh1 = plan(n * D.d * e2); P.datt = plan(n * D.Nq * e2);
    P.dqkv = plan(n * D.Nqkv * e2); P.dxn = plan(n * D.d * e2);
    P.gA = plan(n * D.d * e2); P.gB = plan(n * D.d * e2);
    // transposed-operand scratch: MLP operands have mlp_rows columns, the attention-side ones all tokens
    P.tA = plan(std::max<size_t>((size_t)2 * D.F * mm, (size_t)std::max<int64_t>(D.Nqkv, D.d) * n) * e2);
    P.tB = plan(std::max<size_t>((size_t)D.F * mm, (size_t)std::max<int64_t>(D.Nq, D.d) * n) * e2);
    P.wT = plan(wT_elems * e2);
    P.wT2 = plan((size_t)2 * D.F * D.d * e2);
    P.dlogits = plan((size_t)chunk * D.V * e2); P.dlT = plan((size_t)chunk * D.V * e2);
    P.delta = plan((size_t)n * D.Hq * e4);
    P.logits = plan((size_t)chunk * D.V * e4);
    P.loss_rows = plan(n * e4); P.loss_dev = plan(256);
    P.norm_ws = plan(rmsnorm_bwd_ws_floats(D.d) * e4);
    P.bias_ws = plan(D.bias ? bias_grad_ws_floats((int32_t)D.Nqkv) * e4 : 0);
    // workspace for split reductions of the weight-gradient products, sized for the full token count
    {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            h->n_cu = v;
        else
            (void)hipGetLastError();
        const int64_t rows = (int64_t)cfg->max_batch * cfg->max_seq;
        const int64_t shp[5][2] = {{D.Nqkv, D.d}, {D.d, D.Nq}, {2 * (int64_t)D.F, D.d}, {D.d, D.F}, {D.V, D.d}};
        size_t need = 0;
        for (auto &sh : shp) {
            const int sp = gemm_tn_pick_split(sh[0], sh[1], sh[0] == D.V ? std::min<int64_t>(rows, chunk) : rows, h->n_cu);
            need = std::max(need, (size_t)(sp - 1) * (size_t)sh[0] * (size_t)sh[1]);
        }
        h->split_ws_floats = need;
    }
    P.split_ws = plan(h->split_ws_floats * e4);
    P.rope_cos = plan((size_t)cfg->max_seq * (D.hd / 2) * e4);
    P.rope_sin = plan((size_t)cfg->max_seq * (D.hd / 2) * e4);
    P.tok = plan(n * 4); P.lab = plan(n * 4); P.rowstart = plan(((size_t)D.V + 1) * 4); P.order = plan(n * 4);
    h->arena_bytes = off;
    h->stats.device_arena_bytes = off;
    if (cfg->max_device_bytes && off > cfg->max_device_bytes) {
        const size_t need = off;
        delete h;
        return fail(MT_ERR_DEVICE_OOM, "device arena needs %zu bytes, cap is %llu", need,
                    (unsigned long long)cfg->max_device_bytes);
    }

#define CREATE_HIP(expr)                                                                            \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess) {                                                                     \
            fail(MT_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));                        \
            (void)hipGetLastError();                                                                \
            free_handle(h);                                                                         \
            return MT_ERR_HIP;                                                                      \
        }                                                                                           \
    } while (0)

    CREATE_HIP(hipSetDevice(cfg->device_id));
    {
        hipError_t e = hipMalloc((void **)&h->arena, h->arena_bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            h->arena = nullptr;
            const size_t need = h->arena_bytes;
            free_handle(h);
            return fail(MT_ERR_DEVICE_OOM, "hipMalloc of the %zu-byte device arena failed: %s", need,
                        hipGetErrorString(e));
        }
    }
    char *A = h->arena;
    for (int i = 0; i < 2; ++i) {
        h->Wbuf[i] = (uint16_t *)(A + P.W[i]);
        h->Gbuf[i] = (float *)(A + P.G[i]);
    }
    h->anchors.resize(n_ck);
    for (int i = 0; i < n_ck; ++i) h->anchors[i] = (uint16_t *)(A + P.anchors) + (size_t)i * n * D.d;
    h->blk_h.resize(K - 1);
    for (int i = 0; i < K - 1; ++i) h->blk_h[i] = (uint16_t *)(A + P.blk_h) + (size_t)i * n * D.d;
    h->acts.resize(K);
    for (int i = 0; i < K; ++i) {
        const ActPlan &ap = AP[i];
        h->acts[i] = {(uint16_t *)(A + ap.xn), (uint16_t *)(A + ap.yn), (uint16_t *)(A + ap.qkv), (uint16_t *)(A + ap.att),
                      (uint16_t *)(A + ap.h1), (uint16_t *)(A + ap.gu), (uint16_t *)(A + ap.sact), (float *)(A + ap.lse)};
    }
    h->select_acts(0);
    h->dsact = (uint16_t *)(A + P.dsact);
    h->dgu = (uint16_t *)(A + P.dgu); h->dyn = (uint16_t *)(A + P.dyn); h->dh1 = (uint16_t *)(A + P.dh1);
    h->datt = (uint16_t *)(A + P.datt); h->dqkv = (uint16_t *)(A + P.dqkv); h->dxn = (uint16_t *)(A + P.dxn);
    h->gA = (uint16_t *)(A + P.gA); h->gB = (uint16_t *)(A + P.gB); h->tA = (uint16_t *)(A + P.tA);
    h->tB = (uint16_t *)(A + P.tB); h->wT = (uint16_t *)(A + P.wT); h->wT2 = (uint16_t *)(A + P.wT2); h->dlogits = (uint16_t *)(A + P.dlogits);
    h->dlT = (uint16_t *)(A + P.dlT); h->delta = (float *)(A + P.delta);
    h->logits = (float *)(A + P.logits); h->loss_rows = (float *)(A + P.loss_rows);
    h->loss_dev = (float *)(A + P.loss_dev); h->norm_ws = (float *)(A + P.norm_ws);
    h->bias_ws = (float *)(A + P.bias_ws);
    h->split_ws = h->split_ws_floats ? (float *)(A + P.split_ws) : nullptr;
    h->rope_cos = (float *)(A + P.rope_cos); h->rope_sin = (float *)(A + P.rope_sin);
    h->tok_dev = (int32_t *)(A + P.tok); h->lab_dev = (int32_t *)(A + P.lab);
    h->rowstart_dev = (int32_t *)(A + P.rowstart); h->order_dev = (int32_t *)(A + P.order);

    CREATE_HIP(hipStreamCreateWithFlags(&h->s_comp, hipStreamNonBlocking));
    CREATE_HIP(hipStreamCreateWithFlags(&h->s_h2d, hipStreamNonBlocking));
    CREATE_HIP(hipStreamCreateWithFlags(&h->s_d2h, hipStreamNonBlocking));
    const int nloads = 3 * D.L + 2, ngrads = D.L + 2;  // at most three passes over the blocks (K > 1)
    auto make_events = [&](std::vector<hipEvent_t> &v, int cnt) -> hipError_t {
        v.assign(cnt, nullptr);
        for (int i = 0; i < cnt; ++i) {
            hipError_t e = hipEventCreate(&v[i]);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    };
    CREATE_HIP(make_events(h->w_ready, nloads));
    CREATE_HIP(make_events(h->w_free, nloads));
    CREATE_HIP(make_events(h->h2d_start, nloads));
    CREATE_HIP(make_events(h->comp_start, nloads + 1));  // + the embedding backward
    CREATE_HIP(make_events(h->g_ready, ngrads));
    CREATE_HIP(make_events(h->g_free, ngrads));
    CREATE_HIP(make_events(h->d2h_start, ngrads));
    CREATE_HIP(make_events(h->gm_ready, ngrads));
    CREATE_HIP(make_events(h->gm_free, ngrads));
    CREATE_HIP(make_events(h->d2hm_start, ngrads));
    CREATE_HIP(hipEventCreate(&h->ev_ref));
    CREATE_HIP(hipEventCreate(&h->ev_inputs));

    // ---- host state
    size_t pinned = 0, pageable = 0;
    {
        // Pin every gradient block when that fits the pinned-memory budget; otherwise use the slab pool.
        size_t want = 0;
        h->staged = (cfg->flags & MT_FLAG_STAGED_WEIGHTS) != 0;
        for (auto &u : h->units) want += (h->staged ? 0 : align_up(u.numel * e2, 4096)) + align_up(u.numel * e4, 4096);
        size_t budget = (size_t)56 << 30;
        if (const char *e = getenv("MT_PINNED_BUDGET_GB")) budget = (size_t)atoll(e) << 30;
        h->grad_slabs = (cfg->flags & MT_FLAG_GRAD_SLABS) || want > budget;
        h->n_slabs = h->grad_slabs ? 4 : 0;
    }
    for (auto &u : h->units) {
        bool ok = true;
        if (!h->staged) {
            ok = hipHostMalloc((void **)&u.h_shadow, align_up(u.numel * e2, 4096), hipHostMallocDefault) == hipSuccess;
            pinned += align_up(u.numel * e2, 4096);
        }
        if (ok) {
            if (h->grad_slabs) {
                void *pg = nullptr;
                ok = posix_memalign(&pg, 4096, align_up(u.numel * e4, 4096)) == 0;
                u.h_grad = (float *)pg;
                pageable += align_up(u.numel * e4, 4096);
            } else {
                ok = hipHostMalloc((void **)&u.h_grad, align_up(u.numel * e4, 4096), hipHostMallocDefault) == hipSuccess;
                pinned += align_up(u.numel * e4, 4096);
            }
        }
        if (!ok) {
            (void)hipGetLastError();
            free_handle(h);
            return fail(MT_ERR_HOST_OOM, "host allocation of a unit's bf16 / gradient block failed (pinned so far: %zu bytes)",
                        pinned);
        }
    }
    if (h->staged) {
        h->wslabs.assign(3, nullptr);
        for (auto &p : h->wslabs) {
            if (hipHostMalloc((void **)&p, align_up(h->pmax * e2, 4096), hipHostMallocDefault) != hipSuccess) {
                (void)hipGetLastError();
                p = nullptr;
                free_handle(h);
                return fail(MT_ERR_HOST_OOM, "pinned weight staging slab allocation failed");
            }
            host_zero(p, align_up(h->pmax * e2, 4096));
            pinned += align_up(h->pmax * e2, 4096);
        }
    }
    h->slabs.assign(h->n_slabs, nullptr);
    for (int i = 0; i < h->n_slabs; ++i) {
        if (hipHostMalloc((void **)&h->slabs[i], align_up(h->pmax * e4, 4096), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            free_handle(h);
            return fail(MT_ERR_HOST_OOM, "pinned gradient slab allocation failed");
        }
        host_zero(h->slabs[i], align_up(h->pmax * e4, 4096));
        pinned += align_up(h->pmax * e4, 4096);
    }
    h->adam_m.assign(h->units.size(), nullptr);
    h->adam_v.assign(h->units.size(), nullptr);
    for (size_t u = 0; u < h->units.size(); ++u) {
        void *pm = nullptr, *pv = nullptr;
        const size_t bytes = align_up(h->units[u].numel * e4, 4096);
        if (posix_memalign(&pm, 4096, bytes) || posix_memalign(&pv, 4096, bytes)) {
            free(pm);
            free_handle(h);
            return fail(MT_ERR_HOST_OOM, "Adam moment allocation failed");
        }
        h->adam_m[u] = (float *)pm;
        h->adam_v[u] = (float *)pv;
        host_zero(pm, bytes);
        host_zero(pv, bytes);
        host_zero(h->units[u].h_grad, bytes);
        pageable += 2 * bytes;
    }
    const size_t stage_ints = (size_t)3 * n + D.V + 1;
    if (hipHostMalloc((void **)&h->tok_host, stage_ints * 4, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc((void **)&h->loss_host, 256, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        free_handle(h);
        return fail(MT_ERR_HOST_OOM, "pinned staging allocation failed");
    }
    pinned += stage_ints * 4 + 256;
    h->pinned_bytes = pinned;
    h->pageable_bytes = pageable;
    h->stats.host_pinned_bytes = pinned;
    h->stats.host_pageable_bytes = pageable;
    build_shadow(h);

    // rotary tables (double precision angles, stored fp32)
    {
        const size_t cnt = (size_t)cfg->max_seq * (D.hd / 2);
        std::vector<float> cs(cnt), sn(cnt);
        rope_table(cs.data(), sn.data(), cfg->max_seq, D.hd, (double)cfg->rope_base);
        CREATE_HIP(hipMemcpy(h->rope_cos, cs.data(), cnt * 4, hipMemcpyHostToDevice));
        CREATE_HIP(hipMemcpy(h->rope_sin, sn.data(), cnt * 4, hipMemcpyHostToDevice));
    }
    CREATE_HIP(hipDeviceSynchronize());
#undef CREATE_HIP
    *out = h;
    return MT_OK;
}

mt_status mt_refresh_shadow(mt_handle *h) {
    if (!h) return fail(MT_ERR_INVALID_ARG, "handle is NULL");
    build_shadow(h);
    h->opt_partial = false;
    return MT_OK;
}

mt_status mt_train_step(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                        float *loss) {
    return train_step_core(h, tokens, labels, batch, seq, loss, nullptr, false);
}

mt_status mt_train_step_accumulate(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch,
                                   int32_t seq, float *loss) {
    if (h && !h->have_grads) return fail(MT_ERR_STATE, "mt_train_step_accumulate before the first mt_train_step");
    return train_step_core(h, tokens, labels, batch, seq, loss, nullptr, true);
}

mt_status mt_train_step_adam(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                             float *loss, float lr, float beta1, float beta2, float eps, float wd, int64_t step) {
    if (step < 1) return fail(MT_ERR_INVALID_ARG, "step must be >= 1");
    if (h && h->opt_partial)
        return fail(MT_ERR_STATE, "an earlier mt_train_step_adam failed part-way: restore the parameters and moments, then call mt_refresh_shadow");
    const AdamHyper hp = {lr, beta1, beta2, eps, wd, step};
    return train_step_core(h, tokens, labels, batch, seq, loss, &hp, false);
}

}  // extern "C"

namespace {

// The pinned slabs of the gradient pool, allocated on first use (at create in slab mode, at the first
// accumulating step otherwise).
mt_status ensure_slabs(mt_handle *h) {
    if (h->n_slabs > 0) return MT_OK;
    const size_t bytes = align_up(h->pmax * sizeof(float), 4096);
    std::vector<float *> v(4, nullptr);
    for (auto &p : v) {
        if (hipHostMalloc((void **)&p, bytes, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            for (auto q : v)
                if (q) (void)hipHostFree(q);
            return fail(MT_ERR_HOST_OOM, "pinned gradient slab allocation failed");
        }
        host_zero(p, bytes);
    }
    h->slabs = v;
    h->n_slabs = 4;
    h->pinned_bytes += 4 * bytes;
    h->stats.host_pinned_bytes = h->pinned_bytes;
    return MT_OK;
}

void progress_line(void *arg) {
    const intptr_t v = (intptr_t)arg;
    fprintf(stderr, "[megatrain] unit slot %d of %d done\n", (int)(v >> 16) + 1, (int)(v & 0xffff));
    fflush(stderr);
}

mt_status train_step_core(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                          float *loss, const AdamHyper *opt, bool accumulate) {
    if (!h || !tokens || !labels || !loss) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (batch <= 0 || seq <= 0) return fail(MT_ERR_SHAPE, "batch and seq must be positive");
    const Dims &D = h->D;
    const int64_t n = (int64_t)batch * seq, nmax = (int64_t)h->cfg.max_batch * h->cfg.max_seq;
    if (seq > h->cfg.max_seq || n > nmax) return fail(MT_ERR_SHAPE, "batch*seq = %lld exceeds the capacity %lld (max_seq %d)", (long long)n, (long long)nmax, h->cfg.max_seq);
    if (seq & 7) return fail(MT_ERR_SHAPE, "seq must be a multiple of 8");
    int64_t n_valid = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (tokens[i] < 0 || tokens[i] >= D.V) return fail(MT_ERR_TOKEN_RANGE, "tokens[%lld] = %d outside [0, %d)", (long long)i, tokens[i], D.V);
        if (labels[i] >= D.V) return fail(MT_ERR_TOKEN_RANGE, "labels[%lld] = %d outside the vocabulary", (long long)i, labels[i]);
        n_valid += labels[i] >= 0;
    }
    const float inv_n = n_valid ? (float)(1.0 / (double)n_valid) : 0.f;
    const double t_begin = now_ms();
    HIPCHK(hipSetDevice(h->cfg.device_id));
    h->spans_used = 0;

    const bool serial = h->cfg.flags & MT_FLAG_SERIAL;
    const bool no_copy = h->cfg.flags & MT_FLAG_COMPUTE_ONLY;
    const bool no_kern = h->cfg.flags & MT_FLAG_COPY_ONLY;
    hipStream_t sc = h->s_comp, sh = h->s_h2d, sd = h->s_d2h;

    // ---- stage inputs: tokens | labels | row_start | order (token -> positions, counting sort)
    int32_t *st_tok = h->tok_host, *st_lab = st_tok + n, *st_rs = st_lab + n, *st_ord = st_rs + (D.V + 1);
    memcpy(st_tok, tokens, n * 4);
    memcpy(st_lab, labels, n * 4);
    memset(st_rs, 0, ((size_t)D.V + 1) * 4);
    for (int64_t i = 0; i < n; ++i) st_rs[tokens[i] + 1]++;
    for (int v = 0; v < D.V; ++v) st_rs[v + 1] += st_rs[v];
    {
        std::vector<int32_t> cursor(st_rs, st_rs + D.V);
        for (int64_t i = 0; i < n; ++i) st_ord[cursor[tokens[i]]++] = (int32_t)i;
    }
    HIPCHK(hipEventRecord(h->ev_ref, sc));
    HIPCHK(hipStreamWaitEvent(sh, h->ev_ref, 0));
    HIPCHK(hipStreamWaitEvent(sd, h->ev_ref, 0));
    HIPCHK(hipMemcpyAsync(h->tok_dev, st_tok, n * 4, hipMemcpyHostToDevice, sh));
    HIPCHK(hipMemcpyAsync(h->lab_dev, st_lab, n * 4, hipMemcpyHostToDevice, sh));
    HIPCHK(hipMemcpyAsync(h->rowstart_dev, st_rs, ((size_t)D.V + 1) * 4, hipMemcpyHostToDevice, sh));
    HIPCHK(hipMemcpyAsync(h->order_dev, st_ord, n * 4, hipMemcpyHostToDevice, sh));
    HIPCHK(hipEventRecord(h->ev_inputs, sh));
    HIPCHK(hipStreamWaitEvent(sc, h->ev_inputs, 0));

    // ---- load schedule: E, 1..L, H, then per block of K layers (last block first) the layers in forward
    // order up to the block's last one (RecomputeBlock) and back down in reverse order (LocalBackward).
    // The block's last layer is recomputed and differentiated in one slot, so a block of m layers costs
    // 2m-1 loads (the last block: m); with K = 1 this is the sequence E, 1..L, H, L..1.
    struct BwdSlot { int layer; bool recompute, backward; };
    std::vector<BwdSlot> bslots;
    const int K = h->K;
    // The last block is the exception: the streaming forward has just left its internals in the activation sets
    // (it runs those layers the way a recomputation would), so its backward starts at once.
    const int last_lo = ((D.L - 1) / K) * K + 1;
    for (int b = (D.L - 1) / K; b >= 0; --b) {
        const int lo = b * K + 1, hi = std::min((b + 1) * K, D.L);
        const bool live = lo == last_lo;
        if (!live)
            for (int l = lo; l < hi; ++l) bslots.push_back({l, true, false});
        bslots.push_back({hi, !live, true});
        for (int l = hi - 1; l >= lo; --l) bslots.push_back({l, false, true});
    }
    const int nloads = D.L + 2 + (int)bslots.size();
    std::vector<int> load_unit(nloads);
    load_unit[0] = 0;
    for (int l = 1; l <= D.L; ++l) load_unit[l] = l;
    load_unit[D.L + 1] = D.L + 1;
    for (size_t i = 0; i < bslots.size(); ++i) load_unit[D.L + 2 + i] = bslots[i].layer;
    std::vector<char> load_issued(nloads, 0);
    h->resident[0] = h->resident[1] = -1;
    uint64_t h2d_bytes = 0, d2h_bytes = 0;
    // What load s copies: (unit, element offset inside the weight buffer).  With tied embeddings the head's
    // image is the embedding unit's table followed by the head unit (the final norm gain).
    auto load_pieces = [&](int s) {
        std::vector<std::pair<int, size_t>> v;
        const int u = load_unit[s];
        if (D.tied && u == D.L + 1) {
            v.push_back({0, 0});
            v.push_back({u, (size_t)D.V * D.d});
        } else {
            v.push_back({u, 0});
        }
        return v;
    };
    static const bool progress = [] {
        const char *e = getenv("MT_PROGRESS");
        return e && atoi(e) != 0;
    }();
    std::unique_ptr<PackWorker> packer;
    if (h->staged) packer.reset(new PackWorker(h));
    std::vector<int> load_slab(nloads, -1);  // staged mode: slab of a requested load
    // staged mode: ask the packer for load s unless its unit will still be resident in the target buffer
    auto request_pack = [&](int s) {
        if (!packer || s >= nloads || load_slab[s] >= 0) return;
        const int resident_then = s >= 2 ? load_unit[s - 2] : -1;  // loads alternate between the two buffers
        if (resident_then == load_unit[s]) return;
        load_slab[s] = packer->request(s, load_pieces(s));
    };
    if (no_copy) {
        // weights of block 1 in both buffers once, so the kernels see finite numbers
        const uint16_t *src = h->units[1].h_shadow;
        if (h->staged) {
            for (int i = 0; i < h->n_tensors; ++i)
                if (h->tref[i].unit == 1) host_f32_to_bf16(h->wslabs[0] + h->tref[i].off, h->params[i], h->tref[i].numel);
            src = h->wslabs[0];
        }
        for (int b = 0; b < 2; ++b)
            HIPCHK(hipMemcpyAsync(h->Wbuf[b], src, h->units[1].numel * 2, hipMemcpyHostToDevice, sc));
        HIPCHK(hipStreamSynchronize(sc));
    }

    auto issue_load = [&](int s) -> mt_status {
        const int u = load_unit[s], b = s & 1;
        if (no_copy || h->resident[b] == u) return MT_OK;
        if (packer) {
            request_pack(s);
            request_pack(s + 1);  // one load of lookahead keeps the packer busy while this copy runs
            if (load_slab[s] < 0 || !packer->wait_packed(s))
                return fail(MT_ERR_HIP, "the weight packing thread failed before load %d", s);
        }
        if (s >= 2) HIPCHK(hipStreamWaitEvent(sh, h->w_free[s - 2], 0));
        HIPCHK(hipEventRecord(h->h2d_start[s], sh));
        for (const auto &pc : load_pieces(s)) {
            const size_t cnt = h->units[pc.first].numel;
            const uint16_t *src = packer ? h->wslabs[load_slab[s]] + pc.second : h->units[pc.first].h_shadow;
            HIPCHK(hipMemcpyAsync(h->Wbuf[b] + pc.second, src, cnt * 2, hipMemcpyHostToDevice, sh));
            h2d_bytes += cnt * 2;
        }
        HIPCHK(hipEventRecord(h->w_ready[s], sh));
        if (packer) packer->copy_enqueued(s);
        h->resident[b] = u;
        load_issued[s] = 1;
        if (serial) HIPCHK(hipDeviceSynchronize());
        return MT_OK;
    };
    std::vector<char> grad_issued(D.L + 2, 0);
    std::unique_ptr<HostWorker> worker;
    const bool apply_opt = opt && !no_copy && !no_kern;
    // accumulation needs a host-side add, so the copies of such a step go through the slab pool too
    const bool use_slabs = (h->grad_slabs || accumulate || D.tied) && !no_copy;
    if (use_slabs) {
        const mt_status es = ensure_slabs(h);
        if (es != MT_OK) return es;
    }
    if (apply_opt || use_slabs) worker.reset(new HostWorker(h, apply_opt ? opt : nullptr));
    if (apply_opt) h->opt_partial = true;  // until every unit's update is known to have been applied
    // Gradient block r lives in Gbuf[r & 1] as the image of unit u.  It normally goes to the host as one piece;
    // with tied embeddings the head's image (table gradient | final norm gradient) goes to two units, and the
    // embedding's scatter-add is added to the table gradient that the head left there.
    // A layer's block leaves in two pieces: the MLP part (two thirds of it) as soon as the MLP backward is done,
    // the rest at the end of the block, so the host update of the step's last block is mostly over when the GPU stops.
    struct GPiece { int unit; size_t dev_off, off, count; bool add, run_adam; };  // offsets in Gbuf and in the unit's block
    size_t slab_seq = 0, sub_used = 0;
    // elements per sub-range: 64 MiB of gradients, about a millisecond on the link (MT_SUBPIECE_ELEMS overrides it, so
    // that a test on a small model can cut its gradient pieces, and tensors, at odd places)
    size_t kSubPiece = (size_t)16 << 20;
    if (const char *e = getenv("MT_SUBPIECE_ELEMS")) {
        const long long v = atoll(e);
        if (v > 0) kSubPiece = (size_t)std::max<long long>(v, 256);  // one event per sub-range: keep their number sane
    }
    std::vector<char> early_issued(D.L + 2, 0);
    // copies the pieces on S_d2h after `ready`, brackets them with `start` / `copied`, hands them to the host worker
    auto offload_pieces = [&](int r, const std::vector<GPiece> &pieces, hipEvent_t ready, hipEvent_t start,
                              hipEvent_t copied) -> mt_status {
        HIPCHK(hipStreamWaitEvent(sd, ready, 0));
        HIPCHK(hipEventRecord(start, sd));
        std::vector<int> slab_of(pieces.size(), -1);
        for (size_t i = 0; i < pieces.size(); ++i) {
            const GPiece &pc = pieces[i];
            float *dst = h->units[pc.unit].h_grad + pc.off;
            if (h->grad_slabs || pc.add) {
                // back-pressure of the slab pool: wait (on the host) until the slab's previous content is folded away
                const int slab = (int)(slab_seq++ % (size_t)h->n_slabs);
                if (!worker->acquire_slab(slab)) return fail(MT_ERR_HIP, "the host worker failed while draining a gradient slab");
                dst = h->slabs[slab];
                slab_of[i] = slab;
            }
            d2h_bytes += pc.count * 4;
            if (apply_opt && slab_of[i] < 0 && pc.run_adam && pc.count > 2 * kSubPiece) {
                // a large piece that lands in place: copied and handed over in sub-ranges, so that the host update of
                // the first one starts while the rest is still on the link (what remains after the GPU's last kernel
                // is one sub-range's copy plus the piece's update, not the piece's copy plus its update)
                for (size_t b = 0; b < pc.count; b += kSubPiece) {
                    const size_t cnt = std::min(kSubPiece, pc.count - b);
                    HIPCHK(hipMemcpyAsync(dst + b, h->Gbuf[r & 1] + pc.dev_off + b, cnt * 4, hipMemcpyDeviceToHost, sd));
                    if (sub_used == h->sub_copied.size()) {
                        hipEvent_t ev = nullptr;
                        HIPCHK(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
                        h->sub_copied.push_back(ev);
                    }
                    hipEvent_t ev = h->sub_copied[sub_used++];
                    HIPCHK(hipEventRecord(ev, sd));
                    worker->push(ev, pc.unit, pc.off + b, cnt, -1, false, true);
                }
                slab_of[i] = -2;  // handed over
                continue;
            }
            HIPCHK(hipMemcpyAsync(dst, h->Gbuf[r & 1] + pc.dev_off, pc.count * 4, hipMemcpyDeviceToHost, sd));
        }
        HIPCHK(hipEventRecord(copied, sd));
        if (worker)
            for (size_t i = 0; i < pieces.size(); ++i)
                if (slab_of[i] != -2)
                    worker->push(copied, pieces[i].unit, pieces[i].off, pieces[i].count, slab_of[i], pieces[i].add, pieces[i].run_adam);
        if (serial) HIPCHK(hipDeviceSynchronize());
        return MT_OK;
    };
    // the MLP part of layer unit u (gradient block r), called from inside the block's backward
    auto issue_offload_early = [&](int r, int u) -> mt_status {
        if (no_copy) return MT_OK;
        HIPCHK(hipEventRecord(h->gm_ready[r], sc));
        early_issued[r] = 1;
        return offload_pieces(r, {{u, h->lo.mlp, h->lo.mlp, h->lo.total - h->lo.mlp, accumulate, true}}, h->gm_ready[r],
                              h->d2hm_start[r], h->gm_free[r]);
    };
    auto issue_offload = [&](int r, int u) -> mt_status {
        HIPCHK(hipEventRecord(h->g_ready[r], sc));
        if (no_copy) return MT_OK;
        std::vector<GPiece> pieces;
        if (D.tied && u == D.L + 1) {
            // head image: table gradient | final norm gradient; they belong to units 0 and L+1
            pieces.push_back({0, 0, 0, (size_t)D.V * D.d, accumulate, false});
            pieces.push_back({u, (size_t)D.V * D.d, 0, (size_t)D.d, accumulate, true});
        } else if (early_issued[r]) {
            pieces.push_back({u, 0, 0, h->lo.mlp, accumulate, true});
        } else {
            pieces.push_back({u, 0, 0, h->units[u].numel, accumulate || (D.tied && u == 0), true});
        }
        grad_issued[r] = 1;
        return offload_pieces(r, pieces, h->g_ready[r], h->d2h_start[r], h->g_free[r]);
    };
    auto begin_unit = [&](int s) -> mt_status {
        if (load_issued[s]) HIPCHK(hipStreamWaitEvent(sc, h->w_ready[s], 0));
        HIPCHK(hipEventRecord(h->comp_start[s], sc));
        return MT_OK;
    };
    auto end_unit = [&](int s) -> mt_status {
        HIPCHK(hipEventRecord(h->w_free[s], sc));
        // MT_PROGRESS=1: one line on stderr when the GPU has finished a unit (steps that take minutes)
        if (progress) HIPCHK(hipLaunchHostFunc(sc, progress_line, (void *)(intptr_t)((s << 16) | (nloads & 0xffff))));
        if (serial) HIPCHK(hipDeviceSynchronize());
        return MT_OK;
    };
    auto wait_gbuf = [&](int r) -> mt_status {
        if (r >= 2 && grad_issued[r - 2]) HIPCHK(hipStreamWaitEvent(sc, h->g_free[r - 2], 0));
        return MT_OK;
    };
#define STEP(expr)                   \
    do {                             \
        mt_status s_ = (expr);       \
        if (s_ != MT_OK) {           \
            (void)hipDeviceSynchronize(); \
            return s_;               \
        }                            \
    } while (0)

    // ---- Phase 1: streaming forward
    STEP(issue_load(0));
    for (int s = 0; s <= D.L; ++s) {
        STEP(issue_load(s + 1));  // prefetch the next unit while this one computes
        STEP(begin_unit(s));
        const uint16_t *W = h->Wbuf[s & 1];
        if (!no_kern) {
            if (s == 0) {
                KCHK(embed_gather(h->boundary(0), W, h->tok_dev, n, D.d, sc));
            } else {
                const bool live = s >= last_lo;  // layers of the last block keep what their backward reads
                if (live) h->select_acts(s - last_lo);
                STEP(layer_forward(h, bind_layer(W, h->lo), h->boundary(s - 1), h->boundary(s), batch, seq, live));
            }
        }
        STEP(end_unit(s));
    }
    // ---- Phase 2: loss anchoring (head unit, load index L+1, gradient block 0)
    uint16_t *gcur = h->gA, *gnext = h->gB;
    {
        const int s = D.L + 1;
        STEP(issue_load(s + 1));
        STEP(begin_unit(s));
        if (!no_kern)
            STEP(head_forward_backward(h, h->Wbuf[s & 1], h->Gbuf[0], h->boundary(D.L), gcur, n, inv_n));
        STEP(end_unit(s));
        STEP(issue_offload(0, D.L + 1));
    }
    // ---- Phase 3: block-wise backward.  Activation set (l - lo) holds layer l of the block in flight.
    for (size_t i = 0; i < bslots.size(); ++i) {
        const int s = D.L + 2 + (int)i, l = bslots[i].layer, r = 1 + (D.L - l);
        const int lo = ((l - 1) / K) * K + 1;
        if (s + 1 < nloads) STEP(issue_load(s + 1));
        // the wait for the gradient buffer comes before the unit's start event, so that a stall on the copy that
        // still drains that buffer is not booked as compute-busy time (it would count that copy as hidden)
        if (bslots[i].backward) STEP(wait_gbuf(r));
        STEP(begin_unit(s));
        if (!no_kern) {
            const LayerW w = bind_layer(h->Wbuf[s & 1], h->lo);
            h->select_acts(l - lo);
            if (bslots[i].recompute)  // RecomputeBlock: the last layer of a block needs no output
                STEP(layer_forward(h, w, h->boundary(l - 1), bslots[i].backward ? nullptr : h->boundary(l), batch, seq, true));
            if (bslots[i].backward) {
                STEP(layer_backward(h, w, h->Gbuf[r & 1], h->boundary(l - 1), gcur, gnext, batch, seq,
                                    [&]() -> mt_status { return issue_offload_early(r, l); }));
                std::swap(gcur, gnext);
            }
        }
        STEP(end_unit(s));
        if (bslots[i].backward) STEP(issue_offload(r, l));
    }
    h->select_acts(0);
    // ---- embedding backward (no weights needed), gradient block L+1
    {
        const int r = D.L + 1;
        STEP(wait_gbuf(r));
        HIPCHK(hipEventRecord(h->comp_start[nloads], sc));
        if (!no_kern) KCHK(embed_scatter(h->Gbuf[r & 1], gcur, h->rowstart_dev, h->order_dev, D.V, D.d, sc));
        STEP(issue_offload(r, 0));
    }
    if (!no_kern) HIPCHK(hipMemcpyAsync(h->loss_host, h->loss_dev, 4, hipMemcpyDeviceToHost, sc));
    HIPCHK(hipStreamSynchronize(sc));
    HIPCHK(hipStreamSynchronize(sh));
    HIPCHK(hipStreamSynchronize(sd));
#undef STEP
    *loss = no_kern ? 0.f : h->loss_host[0];
    h->have_grads = true;
    if (worker) {
        const double busy = worker->finish(false);
        if (apply_opt) h->stats.adam_ms = busy;
        if (worker->failed()) return fail(MT_ERR_HIP, "the host worker thread could not wait for a gradient copy");
    }
    h->opt_partial = false;

    // ---- statistics from event timestamps
    mt_stats &S = h->stats;
    S.step_ms = now_ms() - t_begin;
    S.h2d_bytes = h2d_bytes;
    S.d2h_bytes = d2h_bytes;
    S.steps_done++;
    auto ts = [&](hipEvent_t e, double *out_ms) -> bool {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, h->ev_ref, e) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        *out_ms = ms;
        return true;
    };
    std::vector<Iv> comp, h2d, d2h;
    bool ok = true;
    for (int s = 0; s < nloads && ok; ++s) {
        Iv iv;
        ok = ts(h->comp_start[s], &iv.a) && ts(h->w_free[s], &iv.b);
        if (ok) comp.push_back(iv);
        if (ok && load_issued[s]) {
            Iv c;
            ok = ts(h->h2d_start[s], &c.a) && ts(h->w_ready[s], &c.b);
            if (ok) h2d.push_back(c);
        }
    }
    for (int r = 0; r < D.L + 2 && ok; ++r) {
        if (r == D.L + 1) {
            Iv iv;
            ok = ts(h->comp_start[nloads], &iv.a) && ts(h->g_ready[r], &iv.b);
            if (ok) comp.push_back(iv);
        }
        if (ok && grad_issued[r]) {
            Iv c;
            ok = ts(h->d2h_start[r], &c.a) && ts(h->g_free[r], &c.b);
            if (ok) d2h.push_back(c);
        }
        if (ok && early_issued[r]) {
            Iv c;
            ok = ts(h->d2hm_start[r], &c.a) && ts(h->gm_free[r], &c.b);
            if (ok) d2h.push_back(c);
        }
    }
    for (int c = 0; c < 3; ++c) {
        S.class_ms[c] = 0;
        S.class_flops[c] = 0;
        S.class_bytes[c] = 0;
        S.class_launches[c] = 0;
    }
    for (size_t i = 0; i < h->spans_used; ++i) {
        const mt_handle::Span &sp = h->spans[i];
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.a, sp.b) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        S.class_ms[sp.cls] += ms;
        S.class_flops[sp.cls] += sp.flops;
        S.class_bytes[sp.cls] += sp.bytes;
        S.class_launches[sp.cls] += 1;
    }
    S.compute_busy_ms = S.h2d_busy_ms = S.d2h_busy_ms = S.h2d_hidden_ms = S.d2h_hidden_ms = 0;
    if (ok) {
        for (auto &iv : comp) S.compute_busy_ms += iv.b - iv.a;
        for (auto &iv : h2d) S.h2d_busy_ms += iv.b - iv.a;
        for (auto &iv : d2h) S.d2h_busy_ms += iv.b - iv.a;
        S.h2d_hidden_ms = overlap_with_union(h2d, comp);
        S.d2h_hidden_ms = overlap_with_union(d2h, comp);
    }
    return MT_OK;
}

}  // namespace

extern "C" {

mt_status mt_adam_step(mt_handle *h, float lr, float beta1, float beta2, float eps, float wd, int64_t step) {
    if (!h) return fail(MT_ERR_INVALID_ARG, "handle is NULL");
    if (step < 1) return fail(MT_ERR_INVALID_ARG, "step must be >= 1");
    if (!h->have_grads) return fail(MT_ERR_STATE, "mt_adam_step before any successful mt_train_step");
    if (h->opt_partial)
        return fail(MT_ERR_STATE, "an earlier mt_train_step_adam failed part-way: restore the parameters and moments, then call mt_refresh_shadow");
    const double t0 = now_ms();
    for (int i = 0; i < h->n_tensors; ++i) {
        const TensorRef &t = h->tref[i];
        Unit &u = h->units[t.unit];
        host_adam(h->params[i], u.h_grad + t.off, h->adam_m[t.unit] + t.off, h->adam_v[t.unit] + t.off,
                  u.h_shadow ? u.h_shadow + t.off : nullptr, t.numel, lr, beta1, beta2, eps, wd, step);
    }
    h->resident[0] = h->resident[1] = -1;
    h->stats.adam_ms = now_ms() - t0;
    return MT_OK;
}

mt_status mt_get_tensor(mt_handle *h, int32_t idx, int32_t kind, float **p, size_t *numel) {
    if (!h || !p) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (idx < 0 || idx >= h->n_tensors) return fail(MT_ERR_INVALID_ARG, "tensor index out of range");
    const TensorRef &t = h->tref[idx];
    switch (kind) {
        case MT_KIND_GRAD: *p = h->units[t.unit].h_grad + t.off; break;
        case MT_KIND_ADAM_M: *p = h->adam_m[t.unit] + t.off; break;
        case MT_KIND_ADAM_V: *p = h->adam_v[t.unit] + t.off; break;
        default: return fail(MT_ERR_INVALID_ARG, "unknown tensor kind %d", kind);
    }
    if (numel) *numel = t.numel;
    return MT_OK;
}

mt_status mt_get_stats(mt_handle *h, mt_stats *out) {
    if (!h || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    *out = h->stats;
    return MT_OK;
}

mt_status mt_destroy(mt_handle *h) {
    free_handle(h);
    return MT_OK;
}

int32_t mt_device_count(void) {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return n;
}

mt_status mt_device_synchronize(int32_t device_id) {
    HIPCHK(hipSetDevice(device_id));
    HIPCHK(hipDeviceSynchronize());
    return MT_OK;
}

mt_status mt_link_probe(int32_t device_id, size_t bytes, int32_t reps, double *h2d_gbs, double *d2h_gbs,
                        double *bidir_gbs) {
    if (bytes == 0 || reps <= 0) return fail(MT_ERR_INVALID_ARG, "bytes and reps must be positive");
    HIPCHK(hipSetDevice(device_id));
    void *h1 = nullptr, *h2 = nullptr, *d1 = nullptr, *d2 = nullptr;
    hipStream_t s1 = nullptr, s2 = nullptr;
    mt_status rc = MT_OK;
    auto cleanup = [&]() {
        if (h1) (void)hipHostFree(h1);
        if (h2) (void)hipHostFree(h2);
        if (d1) (void)hipFree(d1);
        if (d2) (void)hipFree(d2);
        if (s1) (void)hipStreamDestroy(s1);
        if (s2) (void)hipStreamDestroy(s2);
    };
#define PCHK(expr)                                                                       \
    do {                                                                                 \
        hipError_t e_ = (expr);                                                          \
        if (e_ != hipSuccess) {                                                          \
            rc = fail(MT_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));        \
            (void)hipGetLastError();                                                     \
            cleanup();                                                                   \
            return rc;                                                                   \
        }                                                                                \
    } while (0)
    PCHK(hipHostMalloc(&h1, bytes, hipHostMallocDefault));
    PCHK(hipHostMalloc(&h2, bytes, hipHostMallocDefault));
    PCHK(hipMalloc(&d1, bytes));
    PCHK(hipMalloc(&d2, bytes));
    host_zero(h1, bytes);
    host_zero(h2, bytes);
    PCHK(hipStreamCreateWithFlags(&s1, hipStreamNonBlocking));
    PCHK(hipStreamCreateWithFlags(&s2, hipStreamNonBlocking));
    PCHK(hipMemcpyAsync(d1, h1, bytes, hipMemcpyHostToDevice, s1));
    PCHK(hipMemcpyAsync(h2, d2, bytes, hipMemcpyDeviceToHost, s2));
    PCHK(hipStreamSynchronize(s1));
    PCHK(hipStreamSynchronize(s2));
    double t0 = now_ms();
    for (int i = 0; i < reps; ++i) PCHK(hipMemcpyAsync(d1, h1, bytes, hipMemcpyHostToDevice, s1));
    PCHK(hipStreamSynchronize(s1));
    double t1 = now_ms();
    if (h2d_gbs) *h2d_gbs = (double)bytes * reps / ((t1 - t0) * 1e6);
    t0 = now_ms();
    for (int i = 0; i < reps; ++i) PCHK(hipMemcpyAsync(h2, d2, bytes, hipMemcpyDeviceToHost, s2));
    PCHK(hipStreamSynchronize(s2));
    t1 = now_ms();
    if (d2h_gbs) *d2h_gbs = (double)bytes * reps / ((t1 - t0) * 1e6);
    t0 = now_ms();
    for (int i = 0; i < reps; ++i) {
        PCHK(hipMemcpyAsync(d1, h1, bytes, hipMemcpyHostToDevice, s1));
        PCHK(hipMemcpyAsync(h2, d2, bytes, hipMemcpyDeviceToHost, s2));
    }
    PCHK(hipStreamSynchronize(s1));
    PCHK(hipStreamSynchronize(s2));
    t1 = now_ms();
    if (bidir_gbs) *bidir_gbs = 2.0 * (double)bytes * reps / ((t1 - t0) * 1e6);
#undef PCHK
    cleanup();
    return MT_OK;
}

}  // extern "C"
