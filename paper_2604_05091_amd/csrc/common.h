// Shared declarations of the gfx950 library: vector types, bf16 helpers, wave
// reductions and the launchers that the engine and the kernel-level C ABI call.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace mt {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ float bflo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bfhi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
// round-to-nearest-even pack of two floats (hardware v_cvt_pk_bf16_f32); a in the low half
__device__ __forceinline__ uint32_t pack2bf(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ bf16_t f2bf(float a) { return __builtin_bit_cast(bf16_t, (__bf16)a); }
// Logistic function with the hardware reciprocal (1 ulp) instead of the IEEE division sequence (about ten
// instructions): the results are rounded to bf16 right after, and inside a GEMM store the arithmetic of a 256 x 256
// tile runs on four waves.  Every SwiGLU path (stand-alone kernels and GEMM stores) uses this one function.
__device__ __forceinline__ float sigmoid_rcp(float v) { return __builtin_amdgcn_rcpf(1.0f + __expf(-v)); }

// SwiGLU backward of one element: s = silu(g) * u, ds given -> dg, du (shared by the stand-alone kernel and the
// GEMM store that applies it, so both round alike)
__device__ __forceinline__ void swiglu_bwd_elem(float d, float g, float u, float *dg, float *du) {
    const float sg = sigmoid_rcp(g);
    *dg = d * u * sg * (1.0f + g * (1.0f - sg));
    *du = d * g * sg;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

#ifdef __HIPCC__
typedef __attribute__((ext_vector_type(4))) short s16x4;

// Transposing fragment read.  `tile` is a natural-layout LDS tile [reduction index][LDP] (e.g. V[kv][hd]).
// The result is the A operand of an MFMA whose output rows are the tile's columns col0 .. col0+31 (lane
// l%32 <-> column) and whose eight reduction slots of lane-half hl are the tile rows
// row0 + 4 hl + {0..3} and row0 + 8 + 4 hl + {0..3}: the order in which a lane holds the matching
// accumulator registers of a 32x32 block.  ds_read_b64_tr_b16 works on groups of 16 lanes: lane r' of a
// group supplies the address of 4 consecutive columns of one row; lane i receives column i of the 4 x 16
// block so formed, rows 0..3.  lane_off is tr_lane_offset(lane, LDP), hoisted out of the loops.
__device__ __forceinline__ int tr_lane_offset(int lane, int ldp) {
    const int g = lane >> 4, i = lane & 15;
    return ((g >> 1) * 4 + (i >> 2)) * ldp + (g & 1) * 16 + (i & 3) * 4;
}
__device__ __forceinline__ bf16x8 read_tr_frag(const bf16_t *tile, int lane_off, int ldp, int row0, int col0) {
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const bf16_t *p = tile + lane_off + row0 * ldp + col0;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * ldp));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

#endif  // __HIPCC__

// ---------------------------------------------------------------- launchers (host side)
// Every launcher validates nothing: callers (engine, C ABI wrappers) check shapes first.

// C[M,N] = A[M,K] . B[N,K]^T (+ R) ; A, B bf16 with the reduction index contiguous.
//   out_fp32 = 0: C bf16, optional residual R bf16 [M,N] added before rounding
//   out_fp32 = 1: C fp32; accumulate = 1 adds to the existing C
//   bias: optional per-column bf16 vector added before the residual and the rounding (bf16 output only)
struct GemmArgs {
    const bf16_t *A; int64_t lda;
    const bf16_t *B; int64_t ldb;
    void *C; int64_t ldc;
    const bf16_t *R; int64_t ldr;
    int32_t M, N, K;
    int32_t out_fp32, accumulate;
    const bf16_t *bias = nullptr;  // optional bf16 [N], added to every row (bf16 output only)
    // optional rotary embedding fused into the store (gemm_nt only, see gemm_nt_fuses_rope): columns
    // [0, rope_cols) are heads of 128 whose pairs (j, j + 64) are rotated by the angle of position
    // row % rope_T; tables cos/sin [rope_T][64] fp32
    const float *rope_cos = nullptr, *rope_sin = nullptr;
    int32_t rope_T = 0, rope_cols = 0;
    // optional SwiGLU fused into the store (gemm_nt only, see gemm_nt_fuses_glu): B is [2 glu_F, K], gate rows
    // then up rows (N = 2 glu_F); a tile computes the gate and the up columns of the same 128 indices and stores
    // glu_out[M, glu_F] = silu(gate) * up (bf16, from the bf16-rounded gate and up, as a separate pass over C would).
    // C may then be NULL (gate | up themselves are not stored).
    int32_t glu_F = 0;
    bf16_t *glu_out = nullptr; int64_t ld_glu = 0;
    // optional SwiGLU backward fused into the store (gemm_nt only, see gemm_nt_fuses_glu_bwd): the product is
    // ds [M, N] (N = F, the gradient of the activation, rounded to bf16 as a stored ds would be); with the forward's
    // gate | up in glu_bwd_gu [M, 2N] the kernel stores C [M, 2N] = dgate | dup instead of ds
    const bf16_t *glu_bwd_gu = nullptr; int64_t ld_glu_bwd = 0;
    // optional split of the reduction (gemm_tn only): the K range is cut into split_k chunks that run as separate
    // workgroups (all tiles of chunk 0, then all tiles of chunk 1, ...), chunk 0 stores to C, chunk s > 0 to
    // split_ws + (s - 1) M N (fp32, pitch N), and a second kernel adds them to C in that order.  For tile counts
    // that fill the last round of workgroups badly (see gemm_tn_pick_split).
    int32_t split_k = 1;
    float *split_ws = nullptr;
    // tile order of the large-grid kernels: tile rows per group (a group is walked column by column); 0 = the
    // launcher chooses (gemm_pick_group_m)
    int32_t group_m = 0;
};
hipError_t gemm_nt(const GemmArgs &g, hipStream_t s);
// true when gemm_nt would apply g.rope_* in its epilogue for this problem (large grid, K % 64 == 0, head-aligned
// columns); otherwise a call with rope_cos set fails with hipErrorNotSupported and the caller rotates separately
bool gemm_nt_fuses_rope(const GemmArgs &g);
// the same for g.glu_*: large grid, K % 64 == 0, glu_F % 128 == 0, bf16 output without residual or bias
bool gemm_nt_fuses_glu(const GemmArgs &g);
// and for g.glu_bwd_*: large grid, K % 64 == 0, N % 8 == 0, bf16 output without residual or bias
bool gemm_nt_fuses_glu_bwd(const GemmArgs &g);
// C[M,N] = A^T . B with A given as [K, M] and B as [K, N] (lda, ldb their row pitches): the weight-gradient
// form dW = dY^T X taken straight from token-major activations.  fp32 output (accumulate optional);
// needs K % 64 == 0, M % 8 == 0, N % 8 == 0; returns hipErrorNotSupported otherwise (callers then transpose
// the operands and use gemm_nt).
hipError_t gemm_tn(const GemmArgs &g, hipStream_t s);
// Reduction split for gemm_tn that minimises the estimated time of an M x N x K weight-gradient product on n_cu
// compute units, 1 = none; the workspace it needs is (split - 1) * M * N floats.
int gemm_tn_pick_split(int64_t M, int64_t N, int64_t K, int n_cu);

// out[b][c][r] = in[b][r][c] for r < rows, c < cols (bf16); leading dimensions in elements.
// Two batch levels (b0 < nb0, b1 < nb1) with independent strides on each side.
struct TransposeArgs {
    const bf16_t *in; bf16_t *out;
    int32_t rows, cols;
    int64_t ld_in, ld_out;
    int32_t nb0, nb1;
    int64_t in_s0, in_s1, out_s0, out_s1;
};
hipError_t transpose_bf16(const TransposeArgs &t, hipStream_t s);

hipError_t rmsnorm_fwd(bf16_t *y, const bf16_t *x, const bf16_t *gain, int64_t n, int32_t d, float eps, hipStream_t s);
// dx_out = dres + rmsnorm_backward(dy; x, gain); dgain[d] fp32 (written, or added to when accumulate_dgain:
// rows processed in several calls). partial: >= rmsnorm_bwd_ws_floats(d) floats.
size_t rmsnorm_bwd_ws_floats(int32_t d);
hipError_t rmsnorm_bwd(bf16_t *dx_out, float *dgain, const bf16_t *dy, const bf16_t *x, const bf16_t *gain,
                       const bf16_t *dres, float *partial, int64_t n, int32_t d, float eps, hipStream_t s,
                       int accumulate_dgain = 0);

// The same with the workspace in a file-scope device array of the library (d <= 8192): no allocation, but calls that
// overlap on one device share that array and race.
hipError_t rmsnorm_bwd_static(bf16_t *dx_out, float *dgain, const bf16_t *dy, const bf16_t *x, const bf16_t *gain,
                              const bf16_t *dres, int64_t n, int32_t d, float eps, hipStream_t s);

// In-place rotation of the first n_heads heads of each row of x [n, ld]; cos/sin tables [T, hd/2] fp32;
// position of row r is r % T; sign +1 forward, -1 inverse.
hipError_t rope_inplace(bf16_t *x, int64_t ld, int64_t n, int32_t T, int32_t n_heads, int32_t hd, const float *cs,
                        const float *sn, int sign, hipStream_t s);

// gu [n, 2F] (gate | up) -> s [n, F]
hipError_t swiglu_fwd(bf16_t *sout, const bf16_t *gu, int64_t n, int32_t F, hipStream_t s);
// dgu [n, 2F] from ds [n, F] and gu
hipError_t swiglu_bwd(bf16_t *dgu, const bf16_t *ds, const bf16_t *gu, int64_t n, int32_t F, hipStream_t s);

hipError_t embed_gather(bf16_t *h, const bf16_t *table, const int32_t *tokens, int64_t n, int32_t d, hipStream_t s);
// dtable[V,d] fp32 fully written: row v = sum of dh rows listed in order[start[v] .. start[v+1])
hipError_t embed_scatter(float *dtable, const bf16_t *dh, const int32_t *row_start, const int32_t *order, int32_t V,
                         int32_t d, hipStream_t s);

// Per row: loss_rows[r] = logsumexp(z_r) - z_r[label] (0 for ignored rows); dlogits bf16 = (softmax - onehot) * inv_n
hipError_t cross_entropy(float *loss_rows, bf16_t *dlogits, const float *logits, const int32_t *labels, int64_t n,
                         int32_t V, float inv_n, hipStream_t s);
// out[0] = (accumulate ? out[0] : 0) + scale * sum(in[0..n)) , one block, fixed order
hipError_t reduce_sum(float *out, const float *in, int64_t n, float scale, int accumulate, hipStream_t s);
// db[cols] fp32 (written) = sum over the n rows of x [n, ld] bf16; ws: >= bias_grad_ws_floats(cols) floats
size_t bias_grad_ws_floats(int32_t cols);
hipError_t bias_grad(float *db, const bf16_t *x, int64_t ld, int64_t n, int32_t cols, float *ws, hipStream_t s);

// Flash attention (causal, grouped KV heads).  q/k/v/o rows are tokens (b*T + t); head h occupies
// columns [h*hd, (h+1)*hd) from the given base pointer with the given leading dimension.
// lse [B, Hq, T] fp32 = log sum_u exp(s_tu) of the scaled scores.
struct AttnArgs {
    int32_t B, T, Hq, Hkv, hd;
    float scale;
    const bf16_t *q; int64_t ldq;
    const bf16_t *k; int64_t ldk;
    const bf16_t *v; int64_t ldv;
    bf16_t *o; int64_t ldo;
    float *lse;
    // backward only
    const bf16_t *dout; int64_t lddo;
    const float *delta;  // [B,Hq,T] rowsum(do * o)
    bf16_t *dq; int64_t lddq;
    bf16_t *dk; int64_t lddk;
    bf16_t *dv; int64_t lddv;
    // optional, backward only: q and k had a rotary embedding applied before the attention (pairs (j, j + hd/2),
    // tables cos/sin [T][hd/2] fp32); dq and dk are then rotated back by the row's angle as they are stored
    const float *rope_cos = nullptr, *rope_sin = nullptr;
};
hipError_t flash_fwd(const AttnArgs &a, hipStream_t s);
// delta[b,h,t] = sum_j do[b,t,h,j] * o[b,t,h,j]
hipError_t attn_delta(float *delta, const bf16_t *dout, int64_t lddo, const bf16_t *o, int64_t ldo, int32_t B, int32_t T,
                      int32_t H, int32_t hd, hipStream_t s);
hipError_t flash_bwd_dkdv(const AttnArgs &a, hipStream_t s);
hipError_t flash_bwd_dq(const AttnArgs &a, hipStream_t s);

hipError_t fill_u32(void *p, uint32_t value, size_t n_words, hipStream_t s);

}  // namespace mt
