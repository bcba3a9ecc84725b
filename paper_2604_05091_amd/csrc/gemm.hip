// bf16 x bf16 -> fp32-accumulate GEMM on the gfx950 matrix cores.
//
//   C[M,N] = A[M,K] . B[N,K]^T (+ bias) (+ R)      both operands have the reduction index contiguous
//
// This one entry point serves every projection of a transformer block (Algorithm 1,
// "h_i <- f_i(h_{i-1}; theta_i)" and "LocalBackward"): forward uses the weight as
// stored ([out,in]); the input-gradient and weight-gradient products are brought to
// the same form by transposing one or both operands with transpose_bf16 first.
//
// Two kernels share the tile geometry: a workgroup owns a 256 x 256 (or 128 x 128) tile of C made of
// 32x32 MFMA blocks (v_mfma_f32_32x32x16_bf16, 16 fp32 accumulators per lane per block); K is walked in
// steps of 64 through a double-buffered LDS stage; LDS rows are padded to 72 elements (144 B), which
// makes the 16-byte fragment reads of consecutive lanes conflict-free.
//   gemm_nt_w4_kernel  large grids with K % 64 == 0 (every projection of the billion-parameter
//                      workloads): 4 waves x 128x128 quadrants, software-pipelined inside the wave.
//   gemm_nt_kernel     everything else (ragged K, small problems): 8 waves x 128x64 (or 4 x 64x64),
//                      load - compute - commit - barrier per step.
//
// Workgroup -> tile mapping: consecutive workgroup ids are dealt round-robin to the
// 8 XCDs, each with a private L2.  The id is first re-numbered so that every XCD gets
// a contiguous range of tiles, then walked in column-major groups of 8 tile rows so
// the 32 tiles resident on one XCD form an 8 x 4 patch that shares A and B panels.
#include <stdlib.h>

#include "common.h"

namespace mt {

namespace {

constexpr int BK = 64;
constexpr int LDT = BK + 8;
constexpr int kXcd = 8;
constexpr int kGroupM = 8;
// Tile-row group of the large-grid (load-to-LDS) kernels: the 32 workgroups of an XCD then cover 4 x 8 tiles and a
// group's A rows are left after two patches.  Measured inside the step against 8 (8 x 4 patches): 14B GEMM class
// +0.9 %, 1.3B +0.9 %, 7B +0.2 %; 3 and 6 lose at 14B.  (Stand-alone timings of one GEMM repeated on the same
// operands favour small groups far more, up to 7 % at K = 11008, but there the operands are still in the memory-side
// cache from the previous repetition.)
constexpr int kGroupMLarge = 4;
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
    // One register stage (native vectors, so the selects below stay value selects): while the matrix cores
    // work on k-step t out of LDS, the loads of step t+1 are landing in these registers.
    u32x4 ra0[NA], rb0[NB];
    bool kok0 = true;
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
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
                _Pragma("unroll") for (int j = 0; j < TN; ++j)                                          \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j],  \
                                                                        acc[i][j], 0, 0, 0);            \
            __builtin_amdgcn_sched_barrier(0);                                                          \
        }                                                                                               \
    }

    const int nk = (g.K + BK - 1) / BK;
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
                    if (g.bias) v += bf2f(g.bias[col_w + j * 32]);
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

// ---------------------------------------------------------------------------------------------
// 4-wave variant for large problems with K % 64 == 0: the same 256 x 256 x 64 tile and LDS layout,
// but every wave owns a 128 x 128 quadrant (4 x 4 MFMA blocks, 256 accumulators in AGPRs), which
// halves the LDS bytes read per MFMA, and the whole k-step is software-pipelined inside the wave:
//   phase p = 0..2 : MFMAs of k-slice p  ||  LDS reads of slice p+1  ||  a third of the staged
//                    registers of step t+1 written to the other LDS buffer, each register refilled
//                    at once by the global load of step t+2
//   barrier        : all waves have read buffer t%2 and written step t+1
//   phase 3        : MFMAs of slice 3  ||  LDS reads of slice 0 of step t+1
// so neither the LDS writes nor the global loads ever sit between two MFMAs of one wave.  The
// barrier is issued without a memory fence: a fence would also wait for the global loads in flight.
constexpr int W4_BM = 256, W4_BN = 256, W4_NT = 256;
constexpr int W4_A_BYTES = W4_BM * LDT * 2, W4_STAGE_BYTES = 2 * W4_A_BYTES;

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// bf16 results leave through LDS.  Stored straight from the accumulator layout, a store instruction touches 32
// rows with 16 bytes each, and these partial-line writes cost 10-13 us per tile; instead every wave writes its
// 128 x NC block (bf16) into a private LDS region (the k-loop's stages are free after its last barrier) and reads
// it back row-wise, so that a store instruction covers whole 128-byte lines (16 bytes per lane, consecutive lanes
// at consecutive addresses).  Region pitch NC + 8 elements: conflict-free for the 8-byte writes and the 16-byte reads.
constexpr int W4_EP_PITCH = 128 + 8;
__device__ __forceinline__ bf16_t *w4_ep_region(bf16_t *smem, int wave) { return smem + wave * 128 * W4_EP_PITCH; }

// second half: rows of the wave's block from LDS to C, NC columns starting at col0; rows >= M skipped
template <int NC>
__device__ __forceinline__ void w4_flush_rows(bf16_t *C, int64_t ldc, int M, int row0, int col0, const bf16_t *region,
                                              int lane) {
    constexpr int LPR = NC / 8, RPI = 64 / LPR;   // lanes per row, rows per instruction
    const int lr = lane / LPR, lc = (lane % LPR) * 8;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own LDS writes have landed
#pragma unroll 8
    for (int it = 0; it < 128 / RPI; ++it) {
        const int r = it * RPI + lr;
        const int64_t row = row0 + r;
        if (row >= M) continue;
        *reinterpret_cast<uint4 *>(C + row * ldc + col0 + lc) = *reinterpret_cast<const uint4 *>(region + r * W4_EP_PITCH + lc);
    }
}

// Epilogue of the 4-wave kernels.  The MFMAs are issued with the operands swapped (B fragment first), so each
// 32x32 block holds C transposed: the lane owns row l32 of the block and, per group q = r/4, the four
// consecutive columns 8 q + 4 hl + (0..3): one 8-byte (bf16) or 16-byte (fp32) store each.
__device__ __forceinline__ void w4_store(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int wm, int wn,
                                         int l32, int hl) {
    constexpr int BM = W4_BM, BN = W4_BN;
    const int row_l = m0 + wm * 128 + l32, col_l = n0 + wn * 128 + hl * 4;
    const bool full = (m0 + BM <= g.M) && (n0 + BN <= g.N);
    const bool vec = full && !(g.ldc & 3) && !((uintptr_t)g.C & 15) && (!g.R || (!(g.ldr & 3) && !((uintptr_t)g.R & 7))) &&
                     !((uintptr_t)g.bias & 7);
    if (g.out_fp32) {
        float *cw = reinterpret_cast<float *>(g.C);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = row_l + i * 32;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = col_l + j * 32 + q * 8;
                    float *cp = cw + (int64_t)row * g.ldc + col;
                    if (vec) {
                        f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                        if (g.accumulate) v += *reinterpret_cast<const f32x4 *>(cp);
                        *reinterpret_cast<f32x4 *>(cp) = v;
                    } else if (row < g.M) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < g.N) cp[e] = acc[i][j][4 * q + e] + (g.accumulate ? cp[e] : 0.f);
                    }
                }
        }
    } else {
        bf16_t *cw = reinterpret_cast<bf16_t *>(g.C);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = row_l + i * 32;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = col_l + j * 32 + q * 8;
                    bf16_t *cp = cw + (int64_t)row * g.ldc + col;
                    const bf16_t *rp = g.R ? g.R + (int64_t)row * g.ldr + col : nullptr;
                    if (vec) {
                        float v0 = acc[i][j][4 * q], v1 = acc[i][j][4 * q + 1], v2 = acc[i][j][4 * q + 2],
                              v3 = acc[i][j][4 * q + 3];
                        if (g.bias) {
                            const uint2 bv = *reinterpret_cast<const uint2 *>(g.bias + col);
                            v0 += bflo(bv.x); v1 += bfhi(bv.x); v2 += bflo(bv.y); v3 += bfhi(bv.y);
                        }
                        if (rp) {
                            const uint2 rv = *reinterpret_cast<const uint2 *>(rp);
                            v0 += bflo(rv.x); v1 += bfhi(rv.x); v2 += bflo(rv.y); v3 += bfhi(rv.y);
                        }
                        uint2 o;
                        o.x = pack2bf(v0, v1);
                        o.y = pack2bf(v2, v3);
                        *reinterpret_cast<uint2 *>(cp) = o;
                    } else if (row < g.M) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < g.N)
                                cp[e] = f2bf(acc[i][j][4 * q + e] + (g.bias ? bf2f(g.bias[col + e]) : 0.f) +
                                             (rp ? bf2f(rp[e]) : 0.f));
                    }
                }
        }
    }
}

// complete, aligned column tiles (what the host checks before it picks the kernel instantiated with this store;
// a ragged last row tile is handled by row guards).  Bias
// and residual are template parameters as well: tested per element at run time they turned every one of the 64
// loads into a branch with its own wait.  Here a row block's 16 residual loads are in flight together.
template <bool BIAS, bool RES>
__device__ __forceinline__ void w4_store_full_bf16(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int wm,
                                                   int wn, int l32, int hl, bf16_t *region) {
    const int lane = hl * 32 + l32;
    const int col_l = n0 + wn * 128 + hl * 4;
    uint2 bv[16];
    if constexpr (BIAS) {
#pragma unroll
        for (int jq = 0; jq < 16; ++jq) bv[jq] = *reinterpret_cast<const uint2 *>(g.bias + col_l + (jq >> 2) * 32 + (jq & 3) * 8);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16_t *lp = region + (i * 32 + l32) * W4_EP_PITCH + hl * 4;
        // bias and residual are added in fp32, before the one rounding to bf16
        uint2 rv[16];
        if constexpr (RES) {
            // rows past M (a ragged last row tile) re-read the last row; the second half never stores them
            const bf16_t *rp = g.R + (int64_t)min(m0 + wm * 128 + i * 32 + l32, g.M - 1) * g.ldr + col_l;
#pragma unroll
            for (int jq = 0; jq < 16; ++jq) rv[jq] = *reinterpret_cast<const uint2 *>(rp + (jq >> 2) * 32 + (jq & 3) * 8);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int o = j * 32 + q * 8, jq = j * 4 + q;
                float v0 = acc[i][j][4 * q], v1 = acc[i][j][4 * q + 1], v2 = acc[i][j][4 * q + 2], v3 = acc[i][j][4 * q + 3];
                if constexpr (BIAS) {
                    v0 += bflo(bv[jq].x); v1 += bfhi(bv[jq].x); v2 += bflo(bv[jq].y); v3 += bfhi(bv[jq].y);
                }
                if constexpr (RES) {
                    v0 += bflo(rv[jq].x); v1 += bfhi(rv[jq].x); v2 += bflo(rv[jq].y); v3 += bfhi(rv[jq].y);
                }
                uint2 u;
                u.x = pack2bf(v0, v1);
                u.y = pack2bf(v2, v3);
                *reinterpret_cast<uint2 *>(lp + o) = u;
            }
    }
    w4_flush_rows<128>(reinterpret_cast<bf16_t *>(g.C), g.ldc, g.M, m0 + wm * 128, n0 + wn * 128, region, lane);
}

__device__ __forceinline__ void w4_store_full_f32(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int wm,
                                                  int wn, int l32, int hl) {
    const int row_l = m0 + wm * 128 + l32, col_l = n0 + wn * 128 + hl * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (row_l + i * 32 >= g.M) continue;   // ragged last row tile
        float *cp = reinterpret_cast<float *>(g.C) + (int64_t)(row_l + i * 32) * g.ldc + col_l;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int o = j * 32 + q * 8;
                f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                if (g.accumulate) v += *reinterpret_cast<const f32x4 *>(cp + o);
                *reinterpret_cast<f32x4 *>(cp + o) = v;
            }
    }
}

// bf16 store with the rotary embedding applied on the way out (g.rope_*): the wave's 128 columns are one head,
// the lane holds both members (j, j + 64) of every pair of its rows: blocks j4 and j4 + 2 of acc.  Columns are
// complete (N % 128 == 0, checked on the host); rows are guarded.  Heads at or beyond rope_cols (the value
// projection) are stored unrotated.  Bias, if any, is added before the rotation.  The rows leave through LDS.
template <bool BIAS>
__device__ __forceinline__ void w4_store_rope(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int wm, int wn,
                                              int l32, int hl, bf16_t *region) {
    const int row_l = m0 + wm * 128 + l32, col_w = n0 + wn * 128;
    if (col_w >= g.N) return;
    const bool rot = col_w < g.rope_cols;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // rows past M compute values nobody stores; their table row is still a valid one
        const int64_t tpos = (int64_t)((row_l + i * 32) % g.rope_T) * 64;
        bf16_t *lp = region + (i * 32 + l32) * W4_EP_PITCH;
#pragma unroll
        for (int jp = 0; jp < 2; ++jp)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int jc = jp * 32 + q * 8 + hl * 4;  // pair index inside the head, < 64
                float a[4], b[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a[e] = acc[i][jp][4 * q + e];
                    b[e] = acc[i][jp + 2][4 * q + e];
                }
                if constexpr (BIAS) {
                    const uint2 ba = *reinterpret_cast<const uint2 *>(g.bias + col_w + jc);
                    const uint2 bb = *reinterpret_cast<const uint2 *>(g.bias + col_w + jc + 64);
                    a[0] += bflo(ba.x); a[1] += bfhi(ba.x); a[2] += bflo(ba.y); a[3] += bfhi(ba.y);
                    b[0] += bflo(bb.x); b[1] += bfhi(bb.x); b[2] += bflo(bb.y); b[3] += bfhi(bb.y);
                }
                if (rot) {
                    const f32x4 c = *reinterpret_cast<const f32x4 *>(g.rope_cos + tpos + jc);
                    const f32x4 sn = *reinterpret_cast<const f32x4 *>(g.rope_sin + tpos + jc);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float ya = a[e] * c[e] - b[e] * sn[e], yb = b[e] * c[e] + a[e] * sn[e];
                        a[e] = ya;
                        b[e] = yb;
                    }
                }
                uint2 oa, ob;
                oa.x = pack2bf(a[0], a[1]); oa.y = pack2bf(a[2], a[3]);
                ob.x = pack2bf(b[0], b[1]); ob.y = pack2bf(b[2], b[3]);
                *reinterpret_cast<uint2 *>(lp + jc) = oa;
                *reinterpret_cast<uint2 *>(lp + jc + 64) = ob;
            }
    }
    w4_flush_rows<128>(reinterpret_cast<bf16_t *>(g.C), g.ldc, g.M, m0 + wm * 128, col_w, region, hl * 32 + l32);
}

// SwiGLU store (g.glu_*): the tile's 256 B rows are gate columns c .. c+63, up columns c .. c+63, gate c+64 ..,
// up c+64 .. with c = 128 tn, so a wave holds gate (blocks 0, 1) and up (blocks 2, 3) of the same 64 columns.
// Both go through the wave's LDS region; the row-wise second half computes the activation and stores it (and
// gate | up if asked for) as whole lines.  Rows are guarded; columns are complete (glu_F % 128 == 0).
__device__ __forceinline__ void w4_store_glu(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int tn, int wm, int wn,
                                             int l32, int hl, bf16_t *region) {
    const int lane = hl * 32 + l32;
    // first half: gate (blocks 0, 1) to columns 0..63 of the wave's LDS region, up (blocks 2, 3) to 64..127
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16_t *lp = region + (i * 32 + l32) * W4_EP_PITCH + hl * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 u;
                u.x = pack2bf(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                u.y = pack2bf(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                *reinterpret_cast<uint2 *>(lp + j * 32 + q * 8) = u;
            }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    // second half, row-wise: a lane takes 8 consecutive columns of a row, 8 rows per pass
    const int lr = lane >> 3, lc = (lane & 7) * 8;
    const int col = tn * 128 + wn * 64 + lc;
    bf16_t *cw = reinterpret_cast<bf16_t *>(g.C);
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
        const int r = it * 8 + lr;
        const int64_t row = m0 + wm * 128 + r;
        if (row >= g.M) continue;
        const uint4 gv = *reinterpret_cast<const uint4 *>(region + r * W4_EP_PITCH + lc);
        const uint4 uv = *reinterpret_cast<const uint4 *>(region + r * W4_EP_PITCH + 64 + lc);
        if (cw) {
            *reinterpret_cast<uint4 *>(cw + row * g.ldc + col) = gv;
            *reinterpret_cast<uint4 *>(cw + row * g.ldc + g.glu_F + col) = uv;
        }
        const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w}, uw[4] = {uv.x, uv.y, uv.z, uv.w};
        uint32_t sw[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float g0 = bflo(gw[k]), g1 = bfhi(gw[k]);
            sw[k] = pack2bf(g0 * sigmoid_rcp(g0) * bflo(uw[k]), g1 * sigmoid_rcp(g1) * bfhi(uw[k]));
        }
        *reinterpret_cast<uint4 *>(g.glu_out + row * g.ld_glu + col) = uint4{sw[0], sw[1], sw[2], sw[3]};
    }
}

// SwiGLU backward store (g.glu_bwd_*): the accumulators are ds; they go to the wave's LDS region as bf16, and the
// row-wise second half reads 8 consecutive ds per lane, loads the forward's gate and up of the same elements
// (16 bytes each) and stores dgate and dup, all as whole lines.  Rows >= M and column chunks >= N are skipped.
__device__ __forceinline__ void w4_store_glu_bwd(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int wm,
                                                 int wn, int l32, int hl, bf16_t *region) {
    const int lane = hl * 32 + l32;
    const int lr = lane >> 4, lc = (lane & 15) * 8;
    const int col = n0 + wn * 128 + lc;
    const bool col_ok = col < g.N;
    // The forward's gate and up values come from memory, a microsecond or two away.  The loads of the first kDepth
    // row passes are issued before the accumulators are converted (the k-loop's fragment registers are free by now),
    // each later pass is requested when the pass kDepth before it has been consumed, so the second half never waits
    // for a load it has only just issued.  Rows past M re-read row M - 1 (never stored).  Measured at the 7B shape:
    // depth 2: 5.48 ms, 4: 5.43, 6: 5.44, 8: 5.46, 12: 5.51, 16: 5.6, 32: 5.7 (loads issued on demand, 4 at a
    // time: 5.93): beyond a few passes the requests only queue up behind the chip-wide burst of every tile's store.
    constexpr int kDepth = 4;
    uint4 gq[kDepth], uq[kDepth];
    const bf16_t *gu = g.glu_bwd_gu + (col_ok ? col : 0);
    const int64_t row0 = m0 + wm * 128 + lr;
#pragma unroll
    for (int it = 0; it < kDepth; ++it) {
        const int64_t row = min(row0 + it * 4, (int64_t)g.M - 1);
        gq[it] = *reinterpret_cast<const uint4 *>(gu + row * g.ld_glu_bwd);
        uq[it] = *reinterpret_cast<const uint4 *>(gu + row * g.ld_glu_bwd + g.N);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16_t *lp = region + (i * 32 + l32) * W4_EP_PITCH + hl * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 u;
                u.x = pack2bf(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                u.y = pack2bf(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                *reinterpret_cast<uint2 *>(lp + j * 32 + q * 8) = u;
            }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    bf16_t *C = reinterpret_cast<bf16_t *>(g.C);
#pragma unroll
    for (int it = 0; it < 32; ++it) {
        const int r = it * 4 + lr;
        const int64_t row = m0 + wm * 128 + r;
        const uint4 dv = *reinterpret_cast<const uint4 *>(region + r * W4_EP_PITCH + lc);
        const uint4 gv = gq[it % kDepth], uv = uq[it % kDepth];
        if (it + kDepth < 32) {
            const int64_t nrow = min(row0 + (it + kDepth) * 4, (int64_t)g.M - 1);
            gq[it % kDepth] = *reinterpret_cast<const uint4 *>(gu + nrow * g.ld_glu_bwd);
            uq[it % kDepth] = *reinterpret_cast<const uint4 *>(gu + nrow * g.ld_glu_bwd + g.N);
        }
        const uint32_t dw[4] = {dv.x, dv.y, dv.z, dv.w}, gw[4] = {gv.x, gv.y, gv.z, gv.w}, uw[4] = {uv.x, uv.y, uv.z, uv.w};
        uint32_t og[4], ou[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float a0, b0, a1, b1;
            swiglu_bwd_elem(bflo(dw[k]), bflo(gw[k]), bflo(uw[k]), &a0, &b0);
            swiglu_bwd_elem(bfhi(dw[k]), bfhi(gw[k]), bfhi(uw[k]), &a1, &b1);
            og[k] = pack2bf(a0, a1);
            ou[k] = pack2bf(b0, b1);
        }
        if (col_ok && row < g.M) {
            *reinterpret_cast<uint4 *>(C + row * g.ldc + col) = uint4{og[0], og[1], og[2], og[3]};
            *reinterpret_cast<uint4 *>(C + row * g.ldc + g.N + col) = uint4{ou[0], ou[1], ou[2], ou[3]};
        }
    }
}

// The epilogue is a template parameter: one kernel that carries all of them keeps so much guarded store code alive
// that the compiler moves accumulators through scratch memory on the way out (measured: 13-16 us per tile).
enum { EPI_GENERAL = 0, EPI_FULL_BF16 = 1, EPI_FULL_F32 = 2, EPI_ROPE = 3, EPI_GLU = 4, EPI_GLU_BWD = 5, EPI_FULL_BF16_RES = 6,
       EPI_FULL_BF16_BIAS = 7, EPI_ROPE_BIAS = 8 };
// region: the wave's private LDS staging block (128 rows of W4_EP_PITCH bf16), free once the k-loop's last barrier has passed
template <int EPI>
__device__ __forceinline__ void w4_epilogue(const GemmArgs &g, const f32x16 (&acc)[4][4], int m0, int n0, int tn, int wm, int wn,
                                            int l32, int hl, bf16_t *region) {
    if constexpr (EPI == EPI_GLU) w4_store_glu(g, acc, m0, tn, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_ROPE) w4_store_rope<false>(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_ROPE_BIAS) w4_store_rope<true>(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_GLU_BWD) w4_store_glu_bwd(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_FULL_BF16) w4_store_full_bf16<false, false>(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_FULL_BF16_RES) w4_store_full_bf16<false, true>(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_FULL_BF16_BIAS) w4_store_full_bf16<true, false>(g, acc, m0, n0, wm, wn, l32, hl, region);
    else if constexpr (EPI == EPI_FULL_F32) w4_store_full_f32(g, acc, m0, n0, wm, wn, l32, hl);
    else w4_store(g, acc, m0, n0, wm, wn, l32, hl);
}
template <int EPI>
__global__ __launch_bounds__(W4_NT) void gemm_nt_w4_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int BM = W4_BM, BN = W4_BN;
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
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hl = lane >> 5;

    // loader: thread owns 16-byte chunk (tid & 7) of rows (tid >> 3) + 32 j, j < 8, of A and of B
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const bf16_t *abase = g.A + (int64_t)m0 * g.lda;
    constexpr bool glu = EPI == EPI_GLU;
    const bf16_t *bbase = g.B + (glu ? 0 : (int64_t)n0 * g.ldb);
    uint32_t off[16];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        off[j] = (uint32_t)(min(lrow + 32 * j, g.M - 1 - m0) * (int)g.lda + lkc);
        // SwiGLU pairing: tile rows in blocks of 64 = gate c.., up c.., gate c+64.., up c+64.. (c = 128 tn)
        const int brow = glu ? ((j >> 1) & 1) * g.glu_F + tn * 128 + (j >> 2) * 64 + lrow + 32 * (j & 1)
                             : min(lrow + 32 * j, g.N - 1 - n0);
        off[8 + j] = (uint32_t)(brow * (int)g.ldb + lkc);
    }
    u32x4 st[16];
    bf16x8 fr[2][8];   // [set][A block 0..3 | B block 0..3]
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    char *const lds = reinterpret_cast<char *>(smem);
    const uint32_t wr_off = (uint32_t)((lrow * LDT + lkc) * 2);
    const uint32_t rda_off = (uint32_t)(((wm * 128 + l32) * LDT + hl * 8) * 2);
    const uint32_t rdb_off = (uint32_t)(W4_A_BYTES + ((wn * 128 + l32) * LDT + hl * 8) * 2);
    uint32_t cur = 0;   // byte offset of the LDS buffer holding the current step

#define W4_LOAD(J, K0) st[J] = *reinterpret_cast<const u32x4 *>(((J) < 8 ? abase : bbase) + (K0) + off[J]);
#define W4_WRITE(J, BUFOFF)                                                                             \
    *reinterpret_cast<u32x4 *>(lds + (BUFOFF) + wr_off + ((J) < 8 ? 0 : W4_A_BYTES) + ((J) & 7) * 32 * LDT * 2) = st[J];
#define W4_READ(SET, BUFOFF, KS)                                                                        \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
            fr[SET][i] = *reinterpret_cast<const bf16x8 *>(lds + (BUFOFF) + rda_off + i * 32 * LDT * 2 + (KS) * 32); \
            fr[SET][4 + i] = *reinterpret_cast<const bf16x8 *>(lds + (BUFOFF) + rdb_off + i * 32 * LDT * 2 + (KS) * 32); \
        }                                                                                               \
    }
#define W4_MMA(SET)                                                                                     \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                   \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                               \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[SET][4 + j], fr[SET][i], acc[i][j], 0, 0, 0); \
    }
    // phase P of step kt: chunks [C0, C1) of the staged registers move on
#define W4_PHASE(P, SET, C0, C1, COMMIT, LOAD)                                                          \
    {                                                                                                   \
        W4_READ((SET) ^ 1, cur, (P) + 1);                                                               \
        _Pragma("unroll") for (int c = C0; c < C1; ++c) {                                               \
            if (COMMIT) W4_WRITE(c, nxt);                                                               \
            if (LOAD) W4_LOAD(c, (kt + 2) * BK);                                                        \
        }                                                                                               \
        W4_MMA(SET);                                                                                    \
        _Pragma("unroll") for (int c = 0; c < 8; ++c) {                                                 \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        }                                                                                               \
        _Pragma("unroll") for (int c = C0; c < C1; ++c) {                                               \
            if (COMMIT) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                              \
            if (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        }                                                                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 8 - ((C1) - (C0)), 0);                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define W4_MMA_ROWS(SET, I0, I1)                                                                        \
    {                                                                                                   \
        _Pragma("unroll") for (int i = I0; i < I1; ++i)                                                 \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                               \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[SET][4 + j], fr[SET][i], acc[i][j], 0, 0, 0); \
    }
#define W4_STEP(COMMIT, LOAD)                                                                           \
    {                                                                                                   \
        const uint32_t nxt = W4_STAGE_BYTES - cur;                                                      \
        W4_PHASE(0, 0, 0, 4, COMMIT, LOAD);                                                             \
        W4_PHASE(1, 1, 4, 8, COMMIT, LOAD);                                                             \
        W4_PHASE(2, 0, 8, 12, COMMIT, LOAD);                                                            \
        _Pragma("unroll") for (int c = 12; c < 16; ++c) {                                               \
            if (COMMIT) W4_WRITE(c, nxt);                                                               \
            if (LOAD) W4_LOAD(c, (kt + 2) * BK);                                                        \
        }                                                                                               \
        W4_MMA_ROWS(1, 0, 3);                                                                           \
        _Pragma("unroll") for (int c = 12; c < 16; ++c) {                                               \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
            if (COMMIT) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                              \
            if (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
        }                                                                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        lds_barrier();                                                                                  \
        if (COMMIT) W4_READ(0, nxt, 0);                                                                 \
        W4_MMA_ROWS(1, 3, 4);                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        cur = nxt;                                                                                      \
    }

    const int nk = g.K / BK;
    // prologue: step 0 into LDS buffer 0, step 1 into the staged registers
#pragma unroll
    for (int c = 0; c < 16; ++c) W4_LOAD(c, 0);
#pragma unroll
    for (int c = 0; c < 16; ++c) W4_WRITE(c, 0);
    if (nk > 1) {
#pragma unroll
        for (int c = 0; c < 16; ++c) W4_LOAD(c, BK);
    }
    lds_barrier();
    W4_READ(0, 0, 0);
    int kt = 0;
    for (; kt + 2 < nk; ++kt) W4_STEP(true, true);
    if (kt + 1 < nk) {
        W4_STEP(true, false);
        ++kt;
    }
    W4_STEP(false, false);
#undef W4_LOAD
#undef W4_WRITE
#undef W4_READ
#undef W4_MMA
#undef W4_MMA_ROWS
#undef W4_PHASE
#undef W4_STEP

    w4_epilogue<EPI>(g, acc, m0, n0, tn, wm, wn, l32, hl, w4_ep_region(smem, wm * 2 + wn));
}

// ---------------------------------------------------------------------------------------------
// Load-to-LDS variant with full k-steps of 64: a wave-load fills 8 rows of 128 bytes (whole cache lines per request),
// two LDS slots of 64 KB (A 256 x 64 | B 256 x 64 bf16), chunk c of row r stored at position c ^ ((r >> 1) & 7).
//   step t:  k-slice 0: MFMAs  ||  LDS reads of slice 1  ||  the B-row loads of step t + 1
//            k-slices 1, 2: MFMAs, the LDS reads one slice ahead
//            wait for the loads of step t + 1 (all that are in flight) and for the wave's last reads of the slot; barrier
//            k-slice 3: MFMAs  ||  LDS reads of slice 0 of step t + 1  ||  the A-row loads of step t + 2 into the slot just freed
// A load has two to four k-slices (1000-2000 MFMA clocks) to land; loads go out one per two MFMAs (64 clocks): the path
// into LDS takes a wave's 1 KB every 16 clocks and four waves share it.  No staging registers, no LDS store
// instructions, half the LDS instruction traffic of the register-staged kernel; measured 5-8 % faster at the 7B shapes.
constexpr int WE_HALF = 256 * 64 * 2, WE_SLOT = 2 * WE_HALF, WE_ARRAY = 2 * 128 * W4_EP_PITCH * 2;
static_assert(WE_ARRAY >= WE_SLOT, "a slot must fit into two staging blocks");

template <int EPI>
__global__ __launch_bounds__(W4_NT) void gemm_nt_w4e_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(1024))) char sl0[WE_ARRAY];
    __shared__ __attribute__((aligned(1024))) char sl1[WE_ARRAY];
    typedef __attribute__((address_space(3))) void *lptr;
    const int nb = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int q = nb / kXcd, r = nb % kXcd, x = pid % kXcd;
        pid = x * q + (x < r ? x : r) + pid / kXcd;
    }
    const int gm = g.group_m > 0 ? g.group_m : kGroupMLarge;
    const int group = gm * tiles_n;
    const int first_m = (pid / group) * gm;
    const int gsz = min(tiles_m - first_m, gm);
    const int tm = first_m + (pid % group) % gsz;
    const int tn = (pid % group) / gsz;
    const int m0 = tm * W4_BM, n0 = tn * W4_BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hl = lane >> 5;

    // loader: wave w fills rows 64 w .. 64 w + 63 of the A half and of the B half of a slot, 8 rows per load;
    // lane l delivers to chunk position l & 7 of row l >> 3 and fetches the chunk that belongs there
    constexpr bool glu = EPI == EPI_GLU;
    const bf16_t *abase = g.A + (int64_t)m0 * g.lda;
    const bf16_t *bbase = g.B + (glu ? 0 : (int64_t)n0 * g.ldb);
    uint32_t off[16];   // byte offsets from abase (0..7) / bbase (8..15)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int r = wave * 64 + j * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((r >> 1) & 7);
        off[j] = (uint32_t)(min(r, g.M - 1 - m0) * (int)g.lda + chunk * 8) * 2u;
        // SwiGLU pairing: tile rows in blocks of 64 = gate c.., up c.., gate c+64.., up c+64.. (c = 128 tn)
        const int brow = glu ? ((r >> 6) & 1) * g.glu_F + tn * 128 + ((r >> 7) & 1) * 64 + (r & 63) : min(r, g.N - 1 - n0);
        off[8 + j] = (uint32_t)(brow * (int)g.ldb + chunk * 8) * 2u;
    }
    const uint32_t fill_off = (uint32_t)(wave * 64 * 128);
    // fragment reads: k-chunk 2 ks + hl of row l32 + 32 i sits at chunk position (2 ks + hl) ^ ((l32 >> 1) & 7)
    uint32_t rda[4], rdb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const uint32_t pos = (uint32_t)(((2 * ks + hl) ^ ((l32 >> 1) & 7)) * 16);
        rda[ks] = (uint32_t)((wm * 128 + l32) * 128) + pos;
        rdb[ks] = (uint32_t)(WE_HALF + (wn * 128 + l32) * 128) + pos;
    }
    bf16x8 fr[2][8];   // [set][A block 0..3 | B block 0..3]
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // One load-to-LDS, written out as assembly: the compiler orders every later LDS read after all earlier builtin
    // load-to-LDS instructions it cannot tell apart (a full vmcnt(0) in front of reads of the other slot), which undoes
    // the overlap; ordering is done by hand instead (WE_WAIT).  M0 carries the wave-uniform LDS address, lane i lands
    // at M0 + 16 i; the global address is the uniform base plus the lane's 32-bit byte offset.  (M0 is a reserved
    // register: the compiler keeps no value in it and sets it itself before any instruction of its own that reads it.)
#define WE_LOAD1(SLOT, J, T)                                                                            \
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"                       \
                 :                                                                                      \
                 : "v"(off[J]), "s"(((J) < 8 ? abase : bbase) + (T) * 64),                              \
                   "s"((uint32_t)(uintptr_t)(lptr)(SLOT) + ((J) < 8 ? 0u : (uint32_t)WE_HALF) + fill_off + ((J) & 7) * 1024u) \
                 : "memory")
#define WE_FILL(SLOT, T)                                                                                \
    {                                                                                                   \
        WE_LOAD1(SLOT, 0, T); WE_LOAD1(SLOT, 1, T); WE_LOAD1(SLOT, 2, T); WE_LOAD1(SLOT, 3, T);         \
        WE_LOAD1(SLOT, 4, T); WE_LOAD1(SLOT, 5, T); WE_LOAD1(SLOT, 6, T); WE_LOAD1(SLOT, 7, T);         \
        WE_LOAD1(SLOT, 8, T); WE_LOAD1(SLOT, 9, T); WE_LOAD1(SLOT, 10, T); WE_LOAD1(SLOT, 11, T);       \
        WE_LOAD1(SLOT, 12, T); WE_LOAD1(SLOT, 13, T); WE_LOAD1(SLOT, 14, T); WE_LOAD1(SLOT, 15, T);     \
    }
#define WE_READ1(SET, SLOT, KS, IDX)                                                                    \
    fr[SET][IDX] = *reinterpret_cast<const bf16x8 *>((SLOT) + ((IDX) < 4 ? rda[KS] : rdb[KS]) + ((IDX) & 3) * 4096)
#define WE_READ(SET, SLOT, KS)                                                                          \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
            WE_READ1(SET, SLOT, KS, i);                                                                 \
            WE_READ1(SET, SLOT, KS, 4 + i);                                                             \
        }                                                                                               \
    }
#define WE_MMA1(SET, I, J) acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[SET][4 + (J)], fr[SET][I], acc[I][J], 0, 0, 0)
#define WE_MMA(SET)                                                                                     \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                   \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) WE_MMA1(SET, i, j);                           \
    }
    // 16 MFMAs of SET with the 8 fragment reads of (RSET, SLOT, KS) one per MFMA in front
#define WE_SLICE(SET, RSET, SLOT, KS)                                                                   \
    {                                                                                                   \
        WE_READ(RSET, SLOT, KS);                                                                        \
        WE_MMA(SET);                                                                                    \
        _Pragma("unroll") for (int c = 0; c < 8; ++c) {                                                 \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        }                                                                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define WE_WAIT(N) asm volatile("s_waitcnt vmcnt(" #N ") lgkmcnt(0)\n\ts_barrier" ::: "memory")
    // two MFMAs of slice SET (numbers 2 U and 2 U + 1) with one fragment read of (RSET, RSLOT, KS) and, if LD, one load
    // (J of step TL into LSLOT) in front; pinned in this order.  The loads are spaced two MFMAs (64 clocks) apart: the
    // path into LDS takes a wave's 1 KB load every 16 clocks and is shared by four waves.
#define WE_PAIR(SET, RSET, RSLOT, KS, U, LSLOT, J, TL)                                                  \
    {                                                                                                   \
        if ((J) >= 0) WE_LOAD1(LSLOT, ((J) < 0 ? 0 : (J)), TL);                                         \
        WE_READ1(RSET, RSLOT, KS, ((U) >> 1) + ((U) & 1) * 4);                                          \
        WE_MMA1(SET, (U) >> 1, ((U) & 1) * 2);                                                          \
        WE_MMA1(SET, (U) >> 1, ((U) & 1) * 2 + 1);                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
    // a slice whose MFMA pairs 0..7 carry the loads J0..J7 (of step TL into LSLOT; -1 = none)
#define WE_SLICE_LD(SET, RSET, RSLOT, KS, LSLOT, TL, J0, J1, J2, J3, J4, J5, J6, J7)                    \
    {                                                                                                   \
        WE_PAIR(SET, RSET, RSLOT, KS, 0, LSLOT, J0, TL); WE_PAIR(SET, RSET, RSLOT, KS, 1, LSLOT, J1, TL); \
        WE_PAIR(SET, RSET, RSLOT, KS, 2, LSLOT, J2, TL); WE_PAIR(SET, RSET, RSLOT, KS, 3, LSLOT, J3, TL); \
        WE_PAIR(SET, RSET, RSLOT, KS, 4, LSLOT, J4, TL); WE_PAIR(SET, RSET, RSLOT, KS, 5, LSLOT, J5, TL); \
        WE_PAIR(SET, RSET, RSLOT, KS, 6, LSLOT, J6, TL); WE_PAIR(SET, RSET, RSLOT, KS, 7, LSLOT, J7, TL); \
    }
    // step T out of CUR.  The A rows of step T + 1 were requested into NXT during the last slice of step T - 1; its B
    // rows follow during slice 0 here; the A rows of step T + 2 go into CUR during the last slice.  Past the end of K
    // the last step is requested again (kl clamps it): the same instruction stream for every step, no branches around
    // the MFMAs; the extra data lands in a free slot and is never read.
    // step T out of CUR.  Loads 0..7 (the A rows) of step T + 2 go into CUR during the last slice, right after the barrier
    // that frees it; loads 8..15 (the B rows) follow during slice 0 of the next step.  Later than that they miss the
    // next barrier (measured: 5 + 5 + 6 over three slices is 3 % slower), all 16 in one slice back up behind the load
    // path (5 % slower).
#define WE_STEP(CUR, NXT, T)                                                                            \
    {                                                                                                   \
        const int t1_ = min((T) + 1, nk - 1), t2_ = min((T) + 2, nk - 1);                               \
        WE_SLICE_LD(0, 1, CUR, 1, NXT, t1_, 8, 9, 10, 11, 12, 13, 14, 15);                              \
        WE_SLICE(1, 0, CUR, 2);                                                                         \
        WE_SLICE(0, 1, CUR, 3);                                                                         \
        WE_WAIT(0);                                                                                     \
        WE_SLICE_LD(1, 0, NXT, 0, CUR, t2_, 0, 1, 2, 3, 4, 5, 6, 7);                                    \
    }

    const int nk = g.K / BK;
    WE_FILL(sl0, 0);
    {
        // the A rows of step 1, which the schedule would have requested during "step -1"
        const int t1_ = min(1, nk - 1);
        WE_LOAD1(sl1, 0, t1_); WE_LOAD1(sl1, 1, t1_); WE_LOAD1(sl1, 2, t1_); WE_LOAD1(sl1, 3, t1_);
        WE_LOAD1(sl1, 4, t1_); WE_LOAD1(sl1, 5, t1_); WE_LOAD1(sl1, 6, t1_); WE_LOAD1(sl1, 7, t1_);
    }
    WE_WAIT(8);
    WE_READ(0, sl0, 0);
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
        WE_STEP(sl0, sl1, kt);
        WE_STEP(sl1, sl0, kt + 1);
    }
    if (kt < nk) WE_STEP(sl0, sl1, kt);
    WE_WAIT(0);   // the loads requested past the end have landed before the store staging reuses the arrays
#undef WE_LOAD1
#undef WE_FILL
#undef WE_READ1
#undef WE_READ
#undef WE_MMA1
#undef WE_MMA
#undef WE_SLICE
#undef WE_WAIT
#undef WE_PAIR
#undef WE_SLICE_LD
#undef WE_STEP
    // every wave has passed the last step's barrier, i.e. has read its last fragments: the arrays are free
    bf16_t *region = reinterpret_cast<bf16_t *>((wave < 2 ? sl0 : sl1) + (wave & 1) * (128 * W4_EP_PITCH * 2));
    w4_epilogue<EPI>(g, acc, m0, n0, tn, wm, wn, l32, hl, region);
}

// MT_GROUP_M (diagnostics): forces the tile-row group of the large-grid kernels
int group_m_override() {
    static const int v = [] {
        const char *e = getenv("MT_GROUP_M");
        return e ? atoi(e) : 0;
    }();
    return v;
}

template <int EPI>
hipError_t launch_w4e_epi(const GemmArgs &g0, hipStream_t s) {
    GemmArgs g = g0;
    const int tiles_m = (g.M + W4_BM - 1) / W4_BM, tiles_n = EPI == EPI_GLU ? g.glu_F / 128 : (g.N + W4_BN - 1) / W4_BN;
    if (group_m_override() > 0) g.group_m = group_m_override();
    hipLaunchKernelGGL(gemm_nt_w4e_kernel<EPI>, dim3((unsigned)(tiles_m * tiles_n)), dim3(W4_NT), 0, s, g, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_w4_epi(const GemmArgs &g, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * W4_STAGE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_w4_kernel<EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // with the SwiGLU pairing a tile covers 128 gate and the matching 128 up columns
    const int tiles_m = (g.M + W4_BM - 1) / W4_BM, tiles_n = EPI == EPI_GLU ? g.glu_F / 128 : (g.N + W4_BN - 1) / W4_BN;
    hipLaunchKernelGGL(gemm_nt_w4_kernel<EPI>, dim3((unsigned)(tiles_m * tiles_n)), dim3(W4_NT), lds, s, g, tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_w4(const GemmArgs &g, hipStream_t s) {
    if (g.glu_F > 0) return launch_w4_epi<EPI_GLU>(g, s);
    if (g.rope_cos) return g.bias ? launch_w4_epi<EPI_ROPE_BIAS>(g, s) : launch_w4_epi<EPI_ROPE>(g, s);
    if (g.glu_bwd_gu) return launch_w4_epi<EPI_GLU_BWD>(g, s);
    // every column tile complete and every access of the store aligned: the vector stores (rows are guarded)
    const bool full = g.N % W4_BN == 0 && !(g.ldc & 7) && !((uintptr_t)g.C & 15) &&
                      (!g.R || (!(g.ldr & 3) && !((uintptr_t)g.R & 7))) && !((uintptr_t)g.bias & 7);
    if (!full || (g.bias && g.R)) return launch_w4_epi<EPI_GENERAL>(g, s);
    if (g.out_fp32) return launch_w4_epi<EPI_FULL_F32>(g, s);
    if (g.R) return launch_w4_epi<EPI_FULL_BF16_RES>(g, s);
    return g.bias ? launch_w4_epi<EPI_FULL_BF16_BIAS>(g, s) : launch_w4_epi<EPI_FULL_BF16>(g, s);
}

hipError_t launch_w4e(const GemmArgs &g, hipStream_t s) {
    if (g.glu_F > 0) return launch_w4e_epi<EPI_GLU>(g, s);
    if (g.rope_cos) return g.bias ? launch_w4e_epi<EPI_ROPE_BIAS>(g, s) : launch_w4e_epi<EPI_ROPE>(g, s);
    if (g.glu_bwd_gu) return launch_w4e_epi<EPI_GLU_BWD>(g, s);
    const bool full = g.N % W4_BN == 0 && !(g.ldc & 7) && !((uintptr_t)g.C & 15) &&
                      (!g.R || (!(g.ldr & 3) && !((uintptr_t)g.R & 7))) && !((uintptr_t)g.bias & 7);
    if (!full || (g.bias && g.R)) return launch_w4e_epi<EPI_GENERAL>(g, s);
    if (g.out_fp32) return launch_w4e_epi<EPI_FULL_F32>(g, s);
    if (g.R) return launch_w4e_epi<EPI_FULL_BF16_RES>(g, s);
    return g.bias ? launch_w4e_epi<EPI_FULL_BF16_BIAS>(g, s) : launch_w4e_epi<EPI_FULL_BF16>(g, s);
}


// ---------------------------------------------------------------------------------------------
// Weight-gradient form: C[M,N] = sum_k At[k][m] Bt[k][n] with both operands token-major ([K, M] and [K, N]),
// i.e. dW = dY^T X straight from the activations as the other kernels produce them.  Same tile, waves and
// in-wave pipeline as gemm_nt_w4_kernel; the LDS tiles are [64 k][256 m] (pitch 296 elements: rows 20 banks
// apart, the spacing that keeps the transposing reads nearly conflict-free) and the MFMA operands are read
// with ds_read_b64_tr_b16 (read_tr_frag), which hands a lane eight reduction indices of one output row: two
// reads per fragment instead of one.  fp32 output only.
constexpr int TN_LDT = 256 + 40;
constexpr int TN_TILE_BYTES = BK * TN_LDT * 2, TN_STAGE_BYTES = 2 * TN_TILE_BYTES;

template <int EPI>
__global__ __launch_bounds__(W4_NT) void gemm_tn_w4_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int BM = W4_BM, BN = W4_BN;
    const int n_tiles = tiles_m * tiles_n, nb = n_tiles * g.split_k;
    int pid = blockIdx.x;
    {
        const int q = nb / kXcd, r = nb % kXcd, x = pid % kXcd;
        pid = x * q + (x < r ? x : r) + pid / kXcd;
    }
    // split reduction: units are ordered chunk-major, so the workgroups running together still form tile patches
    // that walk the same K range; chunk 0 owns C, the others a slice of the workspace
    const int chunk = pid / n_tiles;
    pid -= chunk * n_tiles;
    const int nk_all = g.K / BK;
    const int kb = (int)((int64_t)chunk * nk_all / g.split_k), ke = (int)((int64_t)(chunk + 1) * nk_all / g.split_k);
    if (chunk > 0) {
        g.C = g.split_ws + (int64_t)(chunk - 1) * g.M * g.N;
        g.ldc = g.N;
        g.accumulate = 0;
    }
    const int group = kGroupM * tiles_n;
    const int first_m = (pid / group) * kGroupM;
    const int gsz = min(tiles_m - first_m, kGroupM);
    const int tm = first_m + (pid % group) % gsz;
    const int tn = (pid % group) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hl = lane >> 5;
    const int tr_off = tr_lane_offset(lane, TN_LDT);

    // loader: thread owns the 16-byte chunk (tid & 31) (8 consecutive m or n) of the k rows (tid >> 5) + 8 j.
    // Chunks past the matrix edge re-read the last chunk; they only feed outputs that are never stored.
    const int lk = tid >> 5, lc = (tid & 31) * 8;
    const bf16_t *abase = g.A + min(m0 + lc, g.M - 8) + (int64_t)kb * BK * g.lda;
    const bf16_t *bbase = g.B + min(n0 + lc, g.N - 8) + (int64_t)kb * BK * g.ldb;
    u32x4 st[16];
    bf16x8 fr[2][8];
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    char *const lds = reinterpret_cast<char *>(smem);
    const uint32_t wr_off = (uint32_t)((lk * TN_LDT + lc) * 2);
    uint32_t cur = 0;

#define TN_LOAD(J, K0)                                                                                  \
    st[J] = *reinterpret_cast<const u32x4 *>(                                                           \
        ((J) < 8 ? abase + (int64_t)((K0) + lk + 8 * ((J) & 7)) * g.lda : bbase + (int64_t)((K0) + lk + 8 * ((J) & 7)) * g.ldb));
#define TN_WRITE(J, BUFOFF)                                                                             \
    *reinterpret_cast<u32x4 *>(lds + (BUFOFF) + wr_off + ((J) < 8 ? 0 : TN_TILE_BYTES) + ((J) & 7) * 8 * TN_LDT * 2) = st[J];
#define TN_READ(SET, BUFOFF, KS)                                                                        \
    {                                                                                                   \
        const bf16_t *ta_ = reinterpret_cast<const bf16_t *>(lds + (BUFOFF));                           \
        const bf16_t *tb_ = reinterpret_cast<const bf16_t *>(lds + (BUFOFF) + TN_TILE_BYTES);           \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
            fr[SET][i] = read_tr_frag(ta_, tr_off, TN_LDT, (KS) * 16, wm * 128 + i * 32);               \
            fr[SET][4 + i] = read_tr_frag(tb_, tr_off, TN_LDT, (KS) * 16, wn * 128 + i * 32);           \
        }                                                                                               \
    }
#define TN_MMA_ROWS(SET, I0, I1)                                                                        \
    {                                                                                                   \
        _Pragma("unroll") for (int i = I0; i < I1; ++i)                                                 \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                               \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[SET][4 + j], fr[SET][i], acc[i][j], 0, 0, 0); \
    }
#define TN_PHASE(P, SET, C0, C1, COMMIT, LOAD)                                                          \
    {                                                                                                   \
        TN_READ((SET) ^ 1, cur, (P) + 1);                                                               \
        _Pragma("unroll") for (int c = C0; c < C1; ++c) {                                               \
            if (COMMIT) TN_WRITE(c, nxt);                                                               \
            if (LOAD) TN_LOAD(c, (kt + 2) * BK);                                                        \
        }                                                                                               \
        TN_MMA_ROWS(SET, 0, 4);                                                                         \
        _Pragma("unroll") for (int c = 0; c < 8; ++c) {                                                 \
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                          \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        }                                                                                               \
        _Pragma("unroll") for (int c = C0; c < C1; ++c) {                                               \
            if (COMMIT) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                              \
            if (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        }                                                                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 8 - ((C1) - (C0)), 0);                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define TN_STEP(COMMIT, LOAD)                                                                           \
    {                                                                                                   \
        const uint32_t nxt = TN_STAGE_BYTES - cur;                                                      \
        TN_PHASE(0, 0, 0, 4, COMMIT, LOAD);                                                             \
        TN_PHASE(1, 1, 4, 8, COMMIT, LOAD);                                                             \
        TN_PHASE(2, 0, 8, 12, COMMIT, LOAD);                                                            \
        _Pragma("unroll") for (int c = 12; c < 16; ++c) {                                               \
            if (COMMIT) TN_WRITE(c, nxt);                                                               \
            if (LOAD) TN_LOAD(c, (kt + 2) * BK);                                                        \
        }                                                                                               \
        TN_MMA_ROWS(1, 0, 3);                                                                           \
        _Pragma("unroll") for (int c = 12; c < 16; ++c) {                                               \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
            if (COMMIT) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                              \
            if (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
        }                                                                                               \
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        lds_barrier();                                                                                  \
        if (COMMIT) TN_READ(0, nxt, 0);                                                                 \
        TN_MMA_ROWS(1, 3, 4);                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        cur = nxt;                                                                                      \
    }

    const int nk = ke - kb;
#pragma unroll
    for (int c = 0; c < 16; ++c) TN_LOAD(c, 0);
#pragma unroll
    for (int c = 0; c < 16; ++c) TN_WRITE(c, 0);
    if (nk > 1) {
#pragma unroll
        for (int c = 0; c < 16; ++c) TN_LOAD(c, BK);
    }
    lds_barrier();
    TN_READ(0, 0, 0);
    int kt = 0;
    for (; kt + 2 < nk; ++kt) TN_STEP(true, true);
    if (kt + 1 < nk) {
        TN_STEP(true, false);
        ++kt;
    }
    TN_STEP(false, false);
#undef TN_LOAD
#undef TN_WRITE
#undef TN_READ
#undef TN_MMA_ROWS
#undef TN_PHASE
#undef TN_STEP
    if constexpr (EPI == EPI_FULL_F32) w4_store_full_f32(g, acc, m0, n0, wm, wn, l32, hl);
    else w4_store(g, acc, m0, n0, wm, wn, l32, hl);
}

// The same product with the loads written straight into LDS, as in gemm_nt_w4e_kernel: two slots of 64 KB
// (A [64 k][256 m] | B [64 k][256 n] bf16, rows of 512 bytes, unpadded), a wave-load fills two k rows, loads spaced two
// MFMAs apart, one barrier per k-step.  The transposing reads touch 8 k rows x 64 bytes per instruction; the 64-byte
// column group cg of k row r is stored at group position cg ^ (r & 7), which puts the four rows that half a wave reads
// together on disjoint banks (unswizzled they would all sit on the same 16).
constexpr int WT_HALF = 64 * 256 * 2, WT_SLOT = 2 * WT_HALF;

template <int EPI>
__global__ __launch_bounds__(W4_NT) void gemm_tn_w4e_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(1024))) char sl0[WT_SLOT];
    __shared__ __attribute__((aligned(1024))) char sl1[WT_SLOT];
    typedef __attribute__((address_space(3))) void *lptr;
    typedef __attribute__((address_space(3))) s16x4 *trptr;
    constexpr int BM = W4_BM, BN = W4_BN;
    const int n_tiles = tiles_m * tiles_n, nb = n_tiles * g.split_k;
    int pid = blockIdx.x;
    {
        const int q = nb / kXcd, r = nb % kXcd, x = pid % kXcd;
        pid = x * q + (x < r ? x : r) + pid / kXcd;
    }
    // split reduction: units are ordered chunk-major, so the workgroups running together still form tile patches
    // that walk the same K range; chunk 0 owns C, the others a slice of the workspace
    const int chunk = pid / n_tiles;
    pid -= chunk * n_tiles;
    const int nk_all = g.K / BK;
    const int kb = (int)((int64_t)chunk * nk_all / g.split_k), ke = (int)((int64_t)(chunk + 1) * nk_all / g.split_k);
    if (chunk > 0) {
        g.C = g.split_ws + (int64_t)(chunk - 1) * g.M * g.N;
        g.ldc = g.N;
        g.accumulate = 0;
    }
    const int gm = g.group_m > 0 ? g.group_m : kGroupMLarge;
    const int group = gm * tiles_n;
    const int first_m = (pid / group) * gm;
    const int gsz = min(tiles_m - first_m, gm);
    const int tm = first_m + (pid % group) % gsz;
    const int tn = (pid % group) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hl = lane >> 5;

    // loader: wave w fills k rows 16 w .. 16 w + 15 of the A half and of the B half of a slot, two rows per load;
    // lane l delivers to the 16-byte position l & 31 of row l >> 5 and fetches the chunk that belongs there.
    // Chunks past the matrix edge re-read the last chunk; they only feed outputs that are never stored.
    const bf16_t *abase = g.A + (int64_t)kb * BK * g.lda;
    const bf16_t *bbase = g.B + (int64_t)kb * BK * g.ldb;
    uint32_t off[16];   // byte offsets from abase (0..7) / bbase (8..15)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int r = wave * 16 + j * 2 + (lane >> 5);
        const int c16 = ((((lane & 31) >> 2) ^ (r & 7)) << 2) | (lane & 3);
        off[j] = (uint32_t)(r * (int)g.lda + min(m0 + c16 * 8, g.M - 8)) * 2u;
        off[8 + j] = (uint32_t)(r * (int)g.ldb + min(n0 + c16 * 8, g.N - 8)) * 2u;
    }
    const uint32_t fill_off = (uint32_t)(wave * 16 * 512);
    // transposing fragment reads (see read_tr_frag): lane (g, i) of a wave supplies k row (g >> 1) * 4 + (i >> 2) of the
    // slice (and that row + 8), columns (g & 1) * 16 + (i & 3) * 4 .. + 3 of the block's 32; block b of the wave's
    // quadrant is column group cg = 4 wm + b (A) or 4 wn + b (B), stored at group position cg ^ (row & 7)
    uint32_t rd[8];
    {
        const int gq = lane >> 4, ii = lane & 15;
        const int row = (gq >> 1) * 4 + (ii >> 2), inner = (gq & 1) * 16 + (ii & 3) * 4;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            rd[b] = (uint32_t)((row * 256 + (((wm * 4 + b) ^ (row & 7)) * 32) + inner) * 2);
            rd[4 + b] = (uint32_t)(WT_HALF + (row * 256 + (((wn * 4 + b) ^ (row & 7)) * 32) + inner) * 2);
        }
    }
    bf16x8 fr[2][8];
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // one load-to-LDS as assembly, ordered by hand (see gemm_nt_w4e_kernel); a k-step advances both operands by 64 rows
#define WT_LOAD1(SLOT, J, T)                                                                            \
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"                       \
                 :                                                                                      \
                 : "v"(off[J]), "s"((J) < 8 ? abase + (int64_t)(T) * BK * g.lda : bbase + (int64_t)(T) * BK * g.ldb), \
                   "s"((uint32_t)(uintptr_t)(lptr)(SLOT) + ((J) < 8 ? 0u : (uint32_t)WT_HALF) + fill_off + ((J) & 7) * 1024u) \
                 : "memory")
#define WT_READ1(SET, SLOT, KS, IDX)                                                                    \
    {                                                                                                   \
        const s16x4 lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((trptr)((SLOT) + rd[IDX] + (KS) * 8192));        \
        const s16x4 hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((trptr)((SLOT) + rd[IDX] + (KS) * 8192 + 4096)); \
        typedef __attribute__((ext_vector_type(8))) short s16x8_;                                       \
        const s16x8_ v_ = {lo_[0], lo_[1], lo_[2], lo_[3], hi_[0], hi_[1], hi_[2], hi_[3]};             \
        fr[SET][IDX] = __builtin_bit_cast(bf16x8, v_);                                                  \
    }
#define WT_READ(SET, SLOT, KS)                                                                          \
    {                                                                                                   \
        WT_READ1(SET, SLOT, KS, 0); WT_READ1(SET, SLOT, KS, 4); WT_READ1(SET, SLOT, KS, 1); WT_READ1(SET, SLOT, KS, 5); \
        WT_READ1(SET, SLOT, KS, 2); WT_READ1(SET, SLOT, KS, 6); WT_READ1(SET, SLOT, KS, 3); WT_READ1(SET, SLOT, KS, 7); \
    }
#define WT_MMA1(SET, I, J) acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[SET][4 + (J)], fr[SET][I], acc[I][J], 0, 0, 0)
#define WT_WAIT(N) asm volatile("s_waitcnt vmcnt(" #N ") lgkmcnt(0)\n\ts_barrier" ::: "memory")
    // two MFMAs of slice SET with one fragment (two reads) of (RSET, RSLOT, KS) and, if J >= 0, load J of step TL into
    // LSLOT in front; pinned in this order
#define WT_PAIR(SET, RSET, RSLOT, KS, U, LSLOT, J, TL)                                                  \
    {                                                                                                   \
        if ((J) >= 0) WT_LOAD1(LSLOT, ((J) < 0 ? 0 : (J)), TL);                                         \
        WT_READ1(RSET, RSLOT, KS, ((U) >> 1) + ((U) & 1) * 4);                                          \
        WT_MMA1(SET, (U) >> 1, ((U) & 1) * 2);                                                          \
        WT_MMA1(SET, (U) >> 1, ((U) & 1) * 2 + 1);                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define WT_SLICE(SET, RSET, RSLOT, KS, LSLOT, TL, J0, J1, J2, J3, J4, J5, J6, J7)                       \
    {                                                                                                   \
        WT_PAIR(SET, RSET, RSLOT, KS, 0, LSLOT, J0, TL); WT_PAIR(SET, RSET, RSLOT, KS, 1, LSLOT, J1, TL); \
        WT_PAIR(SET, RSET, RSLOT, KS, 2, LSLOT, J2, TL); WT_PAIR(SET, RSET, RSLOT, KS, 3, LSLOT, J3, TL); \
        WT_PAIR(SET, RSET, RSLOT, KS, 4, LSLOT, J4, TL); WT_PAIR(SET, RSET, RSLOT, KS, 5, LSLOT, J5, TL); \
        WT_PAIR(SET, RSET, RSLOT, KS, 6, LSLOT, J6, TL); WT_PAIR(SET, RSET, RSLOT, KS, 7, LSLOT, J7, TL); \
    }
    // step T out of CUR: the schedule of gemm_nt_w4e_kernel
#define WT_STEP(CUR, NXT, T)                                                                            \
    {                                                                                                   \
        const int t1_ = min((T) + 1, nk - 1), t2_ = min((T) + 2, nk - 1);                               \
        WT_SLICE(0, 1, CUR, 1, NXT, t1_, 8, 9, 10, 11, 12, 13, 14, 15);                                 \
        WT_SLICE(1, 0, CUR, 2, NXT, t1_, -1, -1, -1, -1, -1, -1, -1, -1);                               \
        WT_SLICE(0, 1, CUR, 3, NXT, t1_, -1, -1, -1, -1, -1, -1, -1, -1);                               \
        WT_WAIT(0);                                                                                     \
        WT_SLICE(1, 0, NXT, 0, CUR, t2_, 0, 1, 2, 3, 4, 5, 6, 7);                                       \
    }

    const int nk = ke - kb;
    {
        WT_LOAD1(sl0, 0, 0); WT_LOAD1(sl0, 1, 0); WT_LOAD1(sl0, 2, 0); WT_LOAD1(sl0, 3, 0);
        WT_LOAD1(sl0, 4, 0); WT_LOAD1(sl0, 5, 0); WT_LOAD1(sl0, 6, 0); WT_LOAD1(sl0, 7, 0);
        WT_LOAD1(sl0, 8, 0); WT_LOAD1(sl0, 9, 0); WT_LOAD1(sl0, 10, 0); WT_LOAD1(sl0, 11, 0);
        WT_LOAD1(sl0, 12, 0); WT_LOAD1(sl0, 13, 0); WT_LOAD1(sl0, 14, 0); WT_LOAD1(sl0, 15, 0);
        const int t1_ = min(1, nk - 1);
        WT_LOAD1(sl1, 0, t1_); WT_LOAD1(sl1, 1, t1_); WT_LOAD1(sl1, 2, t1_); WT_LOAD1(sl1, 3, t1_);
        WT_LOAD1(sl1, 4, t1_); WT_LOAD1(sl1, 5, t1_); WT_LOAD1(sl1, 6, t1_); WT_LOAD1(sl1, 7, t1_);
    }
    WT_WAIT(8);
    WT_READ(0, sl0, 0);
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
        WT_STEP(sl0, sl1, kt);
        WT_STEP(sl1, sl0, kt + 1);
    }
    if (kt < nk) WT_STEP(sl0, sl1, kt);
    WT_WAIT(0);
#undef WT_LOAD1
#undef WT_READ1
#undef WT_READ
#undef WT_MMA1
#undef WT_WAIT
#undef WT_PAIR
#undef WT_SLICE
#undef WT_STEP
    if constexpr (EPI == EPI_FULL_F32) w4_store_full_f32(g, acc, m0, n0, wm, wn, l32, hl);
    else w4_store(g, acc, m0, n0, wm, wn, l32, hl);
}

// C (pitch ldc) += ws[0] + ws[1] + ... (n_ws slices of M x N floats, pitch N), added in that order
__global__ __launch_bounds__(256) void split_reduce_kernel(float *C, int64_t ldc, const float *ws, int n_ws, int M, int N) {
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4, total = (int64_t)M * N;
    if (idx >= total) return;
    const int64_t row = idx / N;
    const int col = (int)(idx % N);
    f32x4 v = *reinterpret_cast<const f32x4 *>(C + row * ldc + col);
    for (int k = 0; k < n_ws; ++k) v += *reinterpret_cast<const f32x4 *>(ws + (int64_t)k * total + idx);
    *reinterpret_cast<f32x4 *>(C + row * ldc + col) = v;
}

int variant_override();

template <int EPI>
hipError_t launch_tn_epi(const GemmArgs &g0, hipStream_t s) {
    GemmArgs g = g0;
    if (group_m_override() > 0) g.group_m = group_m_override();
    const int tiles_m = (g.M + W4_BM - 1) / W4_BM, tiles_n = (g.N + W4_BN - 1) / W4_BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n * g.split_k));
    if (variant_override() == 5) {   // diagnostic: the register-staged kernel
        constexpr size_t lds = (size_t)2 * TN_STAGE_BYTES;
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tn_w4_kernel<EPI>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        hipLaunchKernelGGL(gemm_tn_w4_kernel<EPI>, grid, dim3(W4_NT), lds, s, g, tiles_m, tiles_n);
    } else {
        hipLaunchKernelGGL(gemm_tn_w4e_kernel<EPI>, grid, dim3(W4_NT), 0, s, g, tiles_m, tiles_n);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || g.split_k == 1) return e;
    const int64_t quads = ((int64_t)g.M * g.N + 3) / 4;
    hipLaunchKernelGGL(split_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, reinterpret_cast<float *>(g.C),
                       g.ldc, g.split_ws, g.split_k - 1, g.M, g.N);
    return hipGetLastError();
}

hipError_t launch_tn(const GemmArgs &g, hipStream_t s) {
    const bool full = g.N % W4_BN == 0 && !(g.ldc & 3) && !((uintptr_t)g.C & 15);
    return full ? launch_tn_epi<EPI_FULL_F32>(g, s) : launch_tn_epi<EPI_GENERAL>(g, s);
}

int variant_override() {
    static int v = [] {
        const char *e = getenv("MT_GEMM_VARIANT");
        return e ? atoi(e) : 0;
    }();
    return v;
}

}  // namespace

static bool takes_w4(const GemmArgs &g) {
    const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
    const int v = variant_override();
    return g.K % BK == 0 && (v == 6 || ((v == 0 || v == 5) && big_tiles >= 192));
}

bool gemm_nt_fuses_rope(const GemmArgs &g) {
    return g.M > 0 && g.N > 0 && g.K > 0 && takes_w4(g) && !g.out_fp32 && !g.R && g.rope_T > 0 && (g.N % 128) == 0 &&
           (g.rope_cols % 128) == 0 && g.rope_cols <= g.N && !(g.ldc & 7) && !((uintptr_t)g.C & 15) &&
           !((uintptr_t)g.bias & 7) && g.rope_cos && g.rope_sin && !((uintptr_t)g.rope_cos & 15) &&
           !((uintptr_t)g.rope_sin & 15);
}

bool gemm_nt_fuses_glu(const GemmArgs &g) {
    return g.M > 0 && g.K > 0 && g.glu_F > 0 && g.N == 2 * g.glu_F && (g.glu_F % 128) == 0 && takes_w4(g) && !g.out_fp32 &&
           !g.R && !g.bias && !g.rope_cos && !g.rope_sin && g.glu_out && !(g.ld_glu & 7) && g.ld_glu >= g.glu_F &&
           !((uintptr_t)g.glu_out & 15) && (!g.C || (!(g.ldc & 7) && !((uintptr_t)g.C & 15))) &&
           (int64_t)g.N * g.ldb < ((int64_t)1 << 31);
}

bool gemm_nt_fuses_glu_bwd(const GemmArgs &g) {
    return g.M > 0 && g.N > 0 && g.K > 0 && (g.N & 7) == 0 && takes_w4(g) && !g.out_fp32 && !g.R && !g.bias && !g.rope_cos &&
           !g.rope_sin && !g.glu_F && !g.glu_out && g.glu_bwd_gu && g.C && !(g.ldc & 7) && g.ldc >= 2 * (int64_t)g.N &&
           !((uintptr_t)g.C & 15) && !(g.ld_glu_bwd & 7) && g.ld_glu_bwd >= 2 * (int64_t)g.N &&
           !((uintptr_t)g.glu_bwd_gu & 15);
}

hipError_t gemm_nt(const GemmArgs &g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    if (g.glu_bwd_gu && !gemm_nt_fuses_glu_bwd(g)) return hipErrorNotSupported;
    if ((g.rope_cos || g.rope_sin) && !gemm_nt_fuses_rope(g)) return hipErrorNotSupported;
    if ((g.glu_F || g.glu_out) && !gemm_nt_fuses_glu(g)) return hipErrorNotSupported;
    if (!g.C && !g.glu_F) return hipErrorInvalidValue;
    if ((g.K & 7) || (g.lda & 7) || (g.ldb & 7)) return hipErrorInvalidValue;
    if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
    if (g.lda < g.K || g.ldb < g.K || (g.C && g.ldc < g.N)) return hipErrorInvalidValue;
    if (g.R && (g.out_fp32 || g.ldr < g.N)) return hipErrorInvalidValue;
    if (g.bias && g.out_fp32) return hipErrorInvalidValue;
    // offsets inside one tile are 32-bit: 256 rows of either operand must stay below 2^31 elements
    if (g.lda >= (1 << 22) || g.ldb >= (1 << 22)) return hipErrorInvalidValue;
    const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
    switch (variant_override()) {   // diagnostic override (MT_GEMM_VARIANT), 0 = heuristic
        case 2: return launch<256, 256, 2, 4>(g, s);
        case 3: return launch<128, 128, 2, 2>(g, s);
        case 5: if (g.K % BK == 0 && big_tiles >= 192) return launch_w4(g, s); break;   // register-staged 4-wave kernel
        case 6: if (g.K % BK == 0) return launch_w4e(g, s); break;                      // 4-wave kernel on any grid
        default: break;
    }
    if (big_tiles >= 192) return (g.K % BK == 0) ? launch_w4e(g, s) : launch<256, 256, 2, 4>(g, s);
    return launch<128, 128, 2, 2>(g, s);
}

int gemm_tn_pick_split(int64_t M, int64_t N, int64_t K, int n_cu) {
    if (M <= 0 || N <= 0 || K < BK || n_cu <= 0) return 1;
    const int64_t tiles = ((M + W4_BM - 1) / W4_BM) * ((N + W4_BN - 1) / W4_BN);
    const int64_t nk = K / BK;
    // one 64-deep k-step of a 256 x 256 tile takes about 1.65 us; the reduction moves (split + 1) M N floats at
    // about 3.5 TB/s; a round of workgroups costs the same whether it is full or not
    const double t_step = 1.65e-6, bw = 3.5e12;
    int best = 1;
    double best_t = 0.0, t_unsplit = 0.0;
    for (int sp = 1; sp <= 6 && nk / sp >= 32; ++sp) {
        const double rounds = (double)((tiles * sp + n_cu - 1) / n_cu);
        const double t = rounds * (double)nk / sp * t_step + (sp > 1 ? (sp + 1) * 4.0 * (double)M * (double)N / bw : 0.0);
        if (sp == 1) {
            best_t = t_unsplit = t;
            continue;
        }
        // a split has to win by 4 % in this estimate: measured, a partly filled last round costs less than a full one
        // (fewer busy compute units clock higher), e.g. 7B down-projection gradient 2.69 rounds: 5.05 ms unsplit, 5.11 split
        if (t < 0.96 * t_unsplit && t < best_t) {
            best_t = t;
            best = sp;
        }
    }
    return best;
}

hipError_t gemm_tn(const GemmArgs &g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    if ((g.lda & 7) || (g.ldb & 7) || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
    if (g.lda < g.M || g.ldb < g.N || g.ldc < g.N || !g.out_fp32 || g.R || g.bias || g.rope_cos || g.rope_sin || g.glu_F ||
        g.glu_out || g.glu_bwd_gu)
        return hipErrorInvalidValue;
    if ((g.K % BK) || (g.M & 7) || (g.N & 7)) return hipErrorNotSupported;
    if (g.split_k < 1 || g.split_k > g.K / BK) return hipErrorInvalidValue;
    // the reduction of a split reads and writes C four floats at a time
    if (g.split_k > 1 && (!g.split_ws || ((uintptr_t)g.split_ws & 15) || (g.ldc & 3) || (g.N & 3) || ((uintptr_t)g.C & 15)))
        return hipErrorInvalidValue;
    return launch_tn(g, s);
}

}  // namespace mt
