// bf16 x bf16 -> fp32-accumulate GEMM on the gfx950 matrix cores.
//
//   C[M,N] = A[M,K] . B[N,K]^T        both operands have the reduction index contiguous
//
// This one kernel serves every projection of a transformer block (Algorithm 1,
// "h_i <- f_i(h_{i-1}; theta_i)" and "LocalBackward"): forward uses the weight as
// stored ([out,in]); the input-gradient and weight-gradient products are brought to
// the same form by transposing one or both operands with transpose_bf16 first.
//
// Tiling: a workgroup of 4 waves (2 x 2) owns a BM x BN tile of C; each wave owns a
// (BM/2) x (BN/2) sub-tile made of 32x32 MFMA blocks (v_mfma_f32_32x32x16_bf16,
// 16 fp32 accumulators per lane per block).  K is walked in steps of 64 through a
// double-buffered LDS stage fed from two register stages: while the matrix cores
// consume step s from LDS, the loads of step s+1 are landing in registers and those of
// step s+2 are being issued; step s+1 is written to the other LDS buffer after the
// MFMAs of step s were issued, so one barrier per step suffices.
// LDS rows are padded to 72 elements (144 B) which makes the 16-byte fragment reads
// of 8 consecutive lanes hit 32 distinct banks.
//
// Workgroup -> tile mapping: consecutive workgroup ids are dealt round-robin to the
// 8 XCDs, each with a private L2.  The id is first re-numbered so that every XCD gets
// a contiguous range of tiles, then walked in column-major groups of 8 tile rows so
// the tiles resident on one XCD share A and B panels.
#include <stdlib.h>

#include "common.h"

namespace mt {

namespace {

constexpr int BK = 64;
constexpr int LDT = BK + 8;
constexpr int kXcd = 8;
constexpr int kGroupM = 8;
#ifndef MT_GX_SETPRIO
#define MT_GX_SETPRIO 0
#endif
#ifndef MT_GX_STAGES
#define MT_GX_STAGES 1
#endif
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_nt_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    constexpr int A_ELEMS = BM * LDT, B_ELEMS = BN * LDT, STAGE = A_ELEMS + B_ELEMS;
    constexpr int RS = NT / 8;                       // rows covered by one pass of the loader
    constexpr int NA = BM / RS, NB = BN / RS;        // 16-byte chunks per thread and operand
    static_assert(BM % RS == 0 && BN % RS == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");

    // ---- tile of this workgroup
    const int nb = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int q = nb / kXcd, r = nb % kXcd, x = pid % kXcd;
        pid = x * q + (x < r ? x : r) + pid / kXcd;
    }
    const int group = kGroupM * tiles_n;
    const int first_m = (pid / group) * kGroupM;
    const int gsz = min(tiles_m - first_m, kGroupM);
    const int tm = first_m + (pid % group) % gsz;
    const int tn = (pid % group) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, hl = lane >> 5;

    // ---- global -> register loader.  Thread owns 16-byte chunk (tid&7) of rows (tid>>3) + RS j.
    // Rows past the matrix edge are clamped to the last row: they only feed C rows/columns that are
    // never stored.  Only the K tail needs real zeros; it is handled in the last step alone.
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const bf16_t *abase = g.A + (int64_t)m0 * g.lda;
    const bf16_t *bbase = g.B + (int64_t)n0 * g.ldb;
    uint32_t aoff[NA], boff[NB];
#pragma unroll
    for (int j = 0; j < NA; ++j) aoff[j] = (uint32_t)(min(lrow + RS * j, g.M - 1 - m0) * (int)g.lda + lkc);
#pragma unroll
    for (int j = 0; j < NB; ++j) boff[j] = (uint32_t)(min(lrow + RS * j, g.N - 1 - n0) * (int)g.ldb + lkc);
    // Two register stages (native vectors, so the selects below stay value selects): while the matrix
    // cores work on k-step t out of LDS, the loads of step t+1 are landing in one stage and the loads of
    // step t+2 are being issued into the other, i.e. every global load has two compute phases to arrive.
    u32x4 ra0[NA], rb0[NB], ra1[NA], rb1[NB];
    bool kok0 = true, kok1 = true;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // K tail: a chunk at or beyond K is read from column 0 of its row instead (always in bounds) and
    // replaced by zeros when it is written to LDS.
#define MT_GEMM_LOAD(RA, RB, KOK, K0)                                                                   \
    {                                                                                                   \
        KOK = ((K0) + lkc) < g.K;                                                                       \
        const bf16_t *ak_ = abase + (KOK ? (K0) : -lkc), *bk_ = bbase + (KOK ? (K0) : -lkc);            \
        _Pragma("unroll") for (int j = 0; j < NA; ++j) RA[j] = *reinterpret_cast<const u32x4 *>(ak_ + aoff[j]); \
        _Pragma("unroll") for (int j = 0; j < NB; ++j) RB[j] = *reinterpret_cast<const u32x4 *>(bk_ + boff[j]); \
    }
#define MT_GEMM_COMMIT(RA, RB, KOK, BUF)                                                                \
    {                                                                                                   \
        bf16_t *ws_ = smem + (BUF) * STAGE + lrow * LDT + lkc;                                          \
        bf16_t *wb_ = ws_ + A_ELEMS;                                                                    \
        _Pragma("unroll") for (int j = 0; j < NA; ++j)                                                  \
            *reinterpret_cast<u32x4 *>(ws_ + RS * j * LDT) = KOK ? RA[j] : zero4;                       \
        _Pragma("unroll") for (int j = 0; j < NB; ++j)                                                  \
            *reinterpret_cast<u32x4 *>(wb_ + RS * j * LDT) = KOK ? RB[j] : zero4;                       \
    }
    // Fragments of k-substep ks+1 are read while the MFMAs of substep ks run (two fragment sets); the
    // scheduling barrier keeps the compiler from sinking the reads back next to their first use.
#define MT_GEMM_READ_FRAGS(SET, KS)                                                                     \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                  \
            af[SET][i] = *reinterpret_cast<const bf16x8 *>(as_ + i * 32 * LDT + (KS) * 16);             \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                  \
            bfr[SET][j] = *reinterpret_cast<const bf16x8 *>(bs_ + j * 32 * LDT + (KS) * 16);            \
    }
#define MT_GEMM_COMPUTE(BUF)                                                                            \
    {                                                                                                   \
        const bf16_t *as_ = smem + (BUF) * STAGE + (wm * WM + l32) * LDT + hl * 8;                      \
        const bf16_t *bs_ = smem + (BUF) * STAGE + A_ELEMS + (wn * WN + l32) * LDT + hl * 8;            \
        bf16x8 af[2][TM], bfr[2][TN];                                                                   \
        MT_GEMM_READ_FRAGS(0, 0);                                                                       \
        _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                        \
            if (ks + 1 < BK / 16) MT_GEMM_READ_FRAGS((ks + 1) & 1, ks + 1);                             \
            __builtin_amdgcn_sched_barrier(0);                                                          \
            if (MT_GX_SETPRIO) __builtin_amdgcn_s_setprio(1);                                           \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
                _Pragma("unroll") for (int j = 0; j < TN; ++j)                                          \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j],  \
                                                                        acc[i][j], 0, 0, 0);            \
            if (MT_GX_SETPRIO) __builtin_amdgcn_s_setprio(0);                                           \
            __builtin_amdgcn_sched_barrier(0);                                                          \
        }                                                                                               \
    }

    const int nk = (g.K + BK - 1) / BK;
#if MT_GX_STAGES == 2
    MT_GEMM_LOAD(ra0, rb0, kok0, 0);
    MT_GEMM_COMMIT(ra0, rb0, kok0, 0);
    if (nk > 1) MT_GEMM_LOAD(ra1, rb1, kok1, BK);
    __syncthreads();

    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        // even step: LDS[0] holds step kt, stage 1 holds step kt+1 (in flight)
        if (kt + 2 < nk) MT_GEMM_LOAD(ra0, rb0, kok0, (kt + 2) * BK);
        MT_GEMM_COMPUTE(0);
        MT_GEMM_COMMIT(ra1, rb1, kok1, 1);
        __syncthreads();
        // odd step: LDS[1] holds step kt+1, stage 0 holds step kt+2 (in flight)
        if (kt + 3 < nk) MT_GEMM_LOAD(ra1, rb1, kok1, (kt + 3) * BK);
        MT_GEMM_COMPUTE(1);
        if (kt + 2 < nk) MT_GEMM_COMMIT(ra0, rb0, kok0, 0);
        __syncthreads();
    }
    if (kt < nk) MT_GEMM_COMPUTE(0);  // odd number of steps: the last one is already in LDS[0]
#else
    (void)ra1; (void)rb1; (void)kok1;
    MT_GEMM_LOAD(ra0, rb0, kok0, 0);
    MT_GEMM_COMMIT(ra0, rb0, kok0, 0);
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        MT_GEMM_LOAD(ra0, rb0, kok0, (kt + 1) * BK);
        MT_GEMM_COMPUTE(0);
        MT_GEMM_COMMIT(ra0, rb0, kok0, 1);
        __syncthreads();
        if (kt + 2 < nk) MT_GEMM_LOAD(ra0, rb0, kok0, (kt + 2) * BK);
        MT_GEMM_COMPUTE(1);
        if (kt + 2 < nk) MT_GEMM_COMMIT(ra0, rb0, kok0, 0);
        __syncthreads();
    }
    if (kt < nk) MT_GEMM_COMPUTE(0);
#endif
#undef MT_GEMM_LOAD
#undef MT_GEMM_COMMIT
#undef MT_GEMM_COMPUTE
#undef MT_GEMM_READ_FRAGS

    // ---- epilogue: lane holds C[row = 8 (r/4) + 4 hl + r%4][col = l32] of each 32x32 block
    const int row_w = m0 + wm * WM + hl * 4, col_w = n0 + wn * WN + l32;
    const bool full = (m0 + BM <= g.M) && (n0 + BN <= g.N);
    if (g.out_fp32) {
        float *cw = reinterpret_cast<float *>(g.C) + (int64_t)row_w * g.ldc + col_w;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = i * 32 + (r >> 2) * 8 + (r & 3);
                if (!full && row_w + dr >= g.M) continue;
                float *cr = cw + (int64_t)dr * g.ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (!full && col_w + j * 32 >= g.N) continue;
                    float v = acc[i][j][r];
                    if (g.accumulate) v += cr[j * 32];
                    cr[j * 32] = v;
                }
            }
    } else {
        bf16_t *cw = reinterpret_cast<bf16_t *>(g.C) + (int64_t)row_w * g.ldc + col_w;
        const bf16_t *rw = g.R ? g.R + (int64_t)row_w * g.ldr + col_w : nullptr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = i * 32 + (r >> 2) * 8 + (r & 3);
                if (!full && row_w + dr >= g.M) continue;
                bf16_t *cr = cw + (int64_t)dr * g.ldc;
                const bf16_t *rr = rw ? rw + (int64_t)dr * g.ldr : nullptr;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (!full && col_w + j * 32 >= g.N) continue;
                    float v = acc[i][j][r];
                    if (rr) v += bf2f(rr[j * 32]);
                    cr[j * 32] = f2bf(v);
                }
            }
    }
}

template <int BM, int BN, int WGM, int WGN>
hipError_t launch(const GemmArgs &g, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * (BM + BN) * LDT * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_kernel<BM, BN, WGM, WGN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    hipLaunchKernelGGL((gemm_nt_kernel<BM, BN, WGM, WGN>), dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WGM * WGN),
                       lds, s, g, tiles_m, tiles_n);
    return hipGetLastError();
}

int variant_override() {
    static int v = [] {
        const char *e = getenv("MT_GEMM_VARIANT");
        return e ? atoi(e) : 0;
    }();
    return v;
}

}  // namespace

hipError_t gemm_nt(const GemmArgs &g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    if ((g.K & 7) || (g.lda & 7) || (g.ldb & 7)) return hipErrorInvalidValue;
    if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
    if (g.lda < g.K || g.ldb < g.K || g.ldc < g.N) return hipErrorInvalidValue;
    if (g.R && (g.out_fp32 || g.ldr < g.N)) return hipErrorInvalidValue;
    // offsets inside one tile are 32-bit: 256 rows of either operand must stay below 2^31 elements
    if (g.lda >= (1 << 22) || g.ldb >= (1 << 22)) return hipErrorInvalidValue;
    const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
    switch (variant_override()) {   // diagnostic override (MT_GEMM_VARIANT), 0 = heuristic
        case 1: return launch<256, 256, 2, 2>(g, s);
        case 2: return launch<256, 256, 2, 4>(g, s);
        case 3: return launch<128, 128, 2, 2>(g, s);
        case 4: return launch<256, 128, 2, 2>(g, s);
        case 5: return launch<256, 128, 4, 2>(g, s);
        default: break;
    }
    if (big_tiles >= 192) return launch<256, 256, 2, 4>(g, s);
    return launch<128, 128, 2, 2>(g, s);
}

}  // namespace mt
