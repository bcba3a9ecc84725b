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
// double-buffered LDS stage: while the matrix cores consume stage s, the global
// loads of stage s+1 are already in flight in registers and are written to the other
// LDS buffer after the MFMAs were issued, so one barrier per step suffices.
// LDS rows are padded to 72 elements (144 B) which makes the 16-byte fragment reads
// of 8 consecutive lanes hit 32 distinct banks.
//
// Workgroup -> tile mapping: consecutive workgroup ids are dealt round-robin to the
// 8 XCDs, each with a private L2.  The id is first re-numbered so that every XCD gets
// a contiguous range of tiles, then walked in column-major groups of 8 tile rows so
// the tiles resident on one XCD share A and B panels.
#include "common.h"

namespace mt {

namespace {

constexpr int BK = 64;
constexpr int LDT = BK + 8;
constexpr int kXcd = 8;
constexpr int kGroupM = 8;

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int A_ELEMS = BM * LDT, B_ELEMS = BN * LDT, STAGE = A_ELEMS + B_ELEMS;
    constexpr int NA = BM / 32, NB = BN / 32;  // 16-byte chunks per thread and operand

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
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hl = lane >> 5;

    // ---- global -> register loader: thread owns chunk column (tid&7) of rows (tid>>3) + 32 j
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const bf16_t *ap = g.A + (int64_t)(m0 + lrow) * g.lda + lkc;
    const bf16_t *bp = g.B + (int64_t)(n0 + lrow) * g.ldb + lkc;
    uint4 ra[NA], rb[NB];
    const uint4 zero = {0u, 0u, 0u, 0u};

    auto load_global = [&](int k0) {
        const bool kok = (k0 + lkc) < g.K;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const bool ok = kok && (m0 + lrow + 32 * j) < g.M;
            ra[j] = ok ? *reinterpret_cast<const uint4 *>(ap + (int64_t)(32 * j) * g.lda + k0) : zero;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const bool ok = kok && (n0 + lrow + 32 * j) < g.N;
            rb[j] = ok ? *reinterpret_cast<const uint4 *>(bp + (int64_t)(32 * j) * g.ldb + k0) : zero;
        }
    };
    auto store_lds = [&](int buf) {
        bf16_t *as = smem + buf * STAGE + lrow * LDT + lkc;
        bf16_t *bs = as + A_ELEMS;
#pragma unroll
        for (int j = 0; j < NA; ++j) *reinterpret_cast<uint4 *>(as + 32 * j * LDT) = ra[j];
#pragma unroll
        for (int j = 0; j < NB; ++j) *reinterpret_cast<uint4 *>(bs + 32 * j * LDT) = rb[j];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (g.K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) load_global((kt + 1) * BK);
        const bf16_t *as = smem + cur * STAGE + (wm * WM + l32) * LDT + hl * 8;
        const bf16_t *bs = smem + cur * STAGE + A_ELEMS + (wn * WN + l32) * LDT + hl * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(as + i * 32 * LDT + ks * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(bs + j * 32 * LDT + ks * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds C[row = 8 (r/4) + 4 hl + r%4][col = l32] of each 32x32 block
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * WN + j * 32 + l32;
            if (col >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * WM + i * 32 + (r >> 2) * 8 + hl * 4 + (r & 3);
                if (row >= g.M) continue;
                float v = acc[i][j][r];
                if (g.out_fp32) {
                    float *c = reinterpret_cast<float *>(g.C) + (int64_t)row * g.ldc + col;
                    if (g.accumulate) v += *c;
                    *c = v;
                } else {
                    if (g.R) v += bf2f(g.R[(int64_t)row * g.ldr + col]);
                    reinterpret_cast<bf16_t *>(g.C)[(int64_t)row * g.ldc + col] = f2bf(v);
                }
            }
        }
}

template <int BM, int BN>
hipError_t launch(const GemmArgs &g, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * (BM + BN) * LDT * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_kernel<BM, BN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    hipLaunchKernelGGL((gemm_nt_kernel<BM, BN>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), lds, s, g, tiles_m,
                       tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t gemm_nt(const GemmArgs &g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    if ((g.K & 7) || (g.lda & 7) || (g.ldb & 7)) return hipErrorInvalidValue;
    if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
    if (g.lda < g.K || g.ldb < g.K || g.ldc < g.N) return hipErrorInvalidValue;
    if (g.R && (g.out_fp32 || g.ldr < g.N)) return hipErrorInvalidValue;
    const int64_t big_tiles = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big_tiles >= 192) return launch<256, 256>(g, s);
    return launch<128, 128>(g, s);
}

}  // namespace mt
