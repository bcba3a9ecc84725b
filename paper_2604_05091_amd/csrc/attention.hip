// Causal flash attention for gfx950, forward and backward, grouped KV heads.
//
// The attention inside f_i and LocalBackward (Algorithm 1) never materialises the
// T x T score matrix: scores are produced tile by tile on the matrix cores, the
// softmax is carried online (running maximum and sum per query), and the backward
// recomputes the probabilities from the saved log-sum-exp.
//
// Register layout.  v_mfma_f32_32x32x16_bf16 leaves, in lane l, the column l%32 of
// the 32x32 result with rows 8(r/4) + 4(l/32) + r%4 for r = 0..15.  The kernels are
// arranged so that the "column" is always the index a wave owns:
//
//   forward, dQ kernel:  S^T = K Q^T, so a lane owns one query.  Row statistics
//       (max, sum, lse, delta) are per-lane scalars; the only cross-lane step is one
//       exchange with lane l^32.  P^T in registers is already a valid B operand for
//       O^T = V^T P^T and dQ^T = K^T dS^T (the reduction index of an MFMA may be
//       permuted freely as long as both operands use the same permutation).
//   dK/dV kernel:        S = Q K^T, so a lane owns one key; dV^T = dO^T P and
//       dK^T = Q^T dS take P and dS from registers in the same way.
//
// The A operands of those second products (V^T, K^T, dO^T, Q^T) are never built in memory:
// they are read from the natural row-major LDS tiles with the gfx950 transposing LDS read
// (ds_read_b64_tr_b16), which hands each lane four consecutive rows of one column; two such
// reads give exactly the eight reduction indices of the accumulator permutation.
// dQ and dK/dV are separate kernels: no atomics, results are bit-reproducible.
//
// LDS rows have a pitch of head_dim + 40 elements: consecutive rows then start 20 banks apart, which keeps
// the 16-byte row reads conflict-free and lets the four rows touched by one transposing read overlap in 12
// of the 64 banks only (a pitch of head_dim + 8 piles them onto the same 28 banks and halves the LDS rate).
#include <stdlib.h>

#include "common.h"

namespace mt {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazyMax = 8.0f;  // forward: the running maximum may lag the true one by this much (log2 units)

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Register-staged cooperative copy of a [ROWS x COLS] bf16 tile (row-major source, leading dimension ld)
// into LDS with pitch LDP, by NT threads.  fetch() issues all global loads back to back (out-of-range
// chunks are redirected to the tile origin, which is always readable, and remembered in a bit mask);
// commit() writes the registers to LDS, zeros for the out-of-range chunks.  Splitting the two lets the
// loads of tile t+1 fly while tile t is being multiplied.
template <int ROWS, int COLS, int LDP, int NT>
struct TileStage {
    static constexpr int CPR = COLS / 8, CHUNKS = ROWS * CPR, N = CHUNKS / NT;
    static_assert(CHUNKS % NT == 0, "tile must split evenly over the threads");
    u32x4 v[N];
    uint32_t okmask;
    __device__ __forceinline__ void fetch(const bf16_t *src, int64_t ld, int rows_valid, int cols_valid) {
        okmask = 0;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int chunk = threadIdx.x + NT * j, r = chunk / CPR, c = (chunk % CPR) * 8;
            const bool ok = r < rows_valid && c < cols_valid;
            const bf16_t *p = src + (ok ? (int64_t)r * ld + c : 0);
            v[j] = *reinterpret_cast<const u32x4 *>(p);
            okmask |= (ok ? 1u : 0u) << j;
        }
    }
    // Rows past rows_valid re-read the last valid row instead of becoming zeros (callers that mask those
    // rows anyway); no select on the way to LDS, so the values never have to pass through the VALU.
    __device__ __forceinline__ void fetch_clamped(const bf16_t *src, int64_t ld, int rows_valid) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int chunk = threadIdx.x + NT * j, r = min(chunk / CPR, rows_valid - 1), c = (chunk % CPR) * 8;
            v[j] = *reinterpret_cast<const u32x4 *>(src + (int64_t)r * ld + c);
        }
    }
    __device__ __forceinline__ void commit_plain(bf16_t *dst) const {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int chunk = threadIdx.x + NT * j, r = chunk / CPR, c = (chunk % CPR) * 8;
            *reinterpret_cast<u32x4 *>(dst + r * LDP + c) = v[j];
        }
    }
    __device__ __forceinline__ void commit(bf16_t *dst) const {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int chunk = threadIdx.x + NT * j, r = chunk / CPR, c = (chunk % CPR) * 8;
            *reinterpret_cast<u32x4 *>(dst + r * LDP + c) = ((okmask >> j) & 1u) ? v[j] : zero;
        }
    }
};

__device__ __forceinline__ bf16x8 pack_frag(const f32x16 &v, int cch) {
    const int o = cch * 8;
    const uint4 u = {pack2bf(v[o + 0], v[o + 1]), pack2bf(v[o + 2], v[o + 3]), pack2bf(v[o + 4], v[o + 5]),
                     pack2bf(v[o + 6], v[o + 7])};
    return __builtin_bit_cast(bf16x8, u);
}

// Unconditional 16-byte load (callers clamp the row to the last valid one, so the loads of a fragment set
// are issued back to back instead of one branch per load; rows past the end are never stored).
__device__ __forceinline__ bf16x8 load_frag_global(const bf16_t *p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

// lane-owned O^T / dQ^T style accumulator [HD rows][32 owned columns] -> out[owned][HD], scaled
template <int HD>
__device__ __forceinline__ void store_owned_rows(bf16_t *out_row, const f32x16 *acc, float mul, int hl) {
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int j = hb * 32 + r4 * 8 + hl * 4;
            const uint2 u = {pack2bf(acc[hb][r4 * 4 + 0] * mul, acc[hb][r4 * 4 + 1] * mul),
                             pack2bf(acc[hb][r4 * 4 + 2] * mul, acc[hb][r4 * 4 + 3] * mul)};
            *reinterpret_cast<uint2 *>(out_row + j) = u;
        }
}

// The same store with the backward of the rotary embedding: the pair (j, j + HD/2) of the row is rotated by minus
// the row's angle; cs / sn point at the row's HD/2 table entries.
template <int HD>
__device__ __forceinline__ void store_owned_rows_unrotated(bf16_t *out_row, const f32x16 *acc, float mul, int hl,
                                                           const float *cs, const float *sn) {
    constexpr int HB2 = HD / 64;
#pragma unroll
    for (int hb = 0; hb < HB2; ++hb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int j = hb * 32 + r4 * 8 + hl * 4;
            const float4 c4 = *reinterpret_cast<const float4 *>(cs + j), s4 = *reinterpret_cast<const float4 *>(sn + j);
            const float c[4] = {c4.x, c4.y, c4.z, c4.w}, sv[4] = {s4.x, s4.y, s4.z, s4.w};
            float xa[4], xb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ya = acc[hb][r4 * 4 + e] * mul, yb = acc[hb + HB2][r4 * 4 + e] * mul;
                xa[e] = ya * c[e] + yb * sv[e];
                xb[e] = yb * c[e] - ya * sv[e];
            }
            const uint2 ua = {pack2bf(xa[0], xa[1]), pack2bf(xa[2], xa[3])};
            const uint2 ub = {pack2bf(xb[0], xb[1]), pack2bf(xb[2], xb[3])};
            *reinterpret_cast<uint2 *>(out_row + j) = ua;
            *reinterpret_cast<uint2 *>(out_row + j + HD / 2) = ub;
        }
}

// Results leave through LDS: stored from the accumulator layout (a lane owns a row) one store instruction would
// touch 64 rows with 8 bytes each.  Every wave writes its 32 x HD block into a private LDS region (free after the
// main loop's last barrier) with the two functions above and copies it out row-wise, 16 bytes per lane, whole lines.
// Falls back to the direct stores when the destination rows are not 16-byte aligned.
template <int HD>
__device__ __forceinline__ bf16_t *out_region(bf16_t *smem, int wave) { return smem + wave * 32 * (HD + 8); }

template <int HD>
__device__ __forceinline__ void flush_owned_rows(bf16_t *out_row0, int64_t ld, const bf16_t *region, int lane, int n_valid) {
    constexpr int LPR = HD / 8, RPI = 64 / LPR;
    const int lr = lane / LPR, lc = (lane % LPR) * 8;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + lr;
        if (r < n_valid)
            *reinterpret_cast<uint4 *>(out_row0 + r * ld + lc) = *reinterpret_cast<const uint4 *>(region + r * (HD + 8) + lc);
    }
}

// out_row0: row of the wave's first query / key; cs, sn: rotary tables at that row, or NULL
template <int HD>
__device__ __forceinline__ void write_owned_rows(bf16_t *out_row0, int64_t ld, const f32x16 *acc, float mul, int l32, int hl,
                                                 int n_valid, const float *cs, const float *sn, bf16_t *region) {
    const bool wide = !(ld & 7) && !((uintptr_t)out_row0 & 15);
    bf16_t *dst = wide ? region + l32 * (HD + 8) : out_row0 + l32 * ld;
    if (wide || l32 < n_valid) {
        const int tr = min(l32, n_valid - 1);  // rows past the end are never stored; keep their table reads in range
        if (cs) store_owned_rows_unrotated<HD>(dst, acc, mul, hl, cs + tr * (HD / 2), sn + tr * (HD / 2));
        else store_owned_rows<HD>(dst, acc, mul, hl);
    }
    if (wide) flush_owned_rows<HD>(out_row0, ld, region, hl * 32 + l32, n_valid);
}

// acc[hb] += X^T (columns hb*32.. of the natural tile X, reduction rows rb*32 + cch*16 ..) * frag, for all hb
template <int HD, int LDP>
__device__ __forceinline__ void mfma_tr_accumulate(f32x16 *acc, const bf16_t *tile, int tr_off, int rb, int cch,
                                                   const bf16x8 &frag) {
    bf16x8 a[HD / 32];
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb) a[hb] = read_tr_frag(tile, tr_off, LDP, rb * 32 + cch * 16, hb * 32);
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb) acc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[hb], frag, acc[hb], 0, 0, 0);
}

// Workgroup -> (batch, KV head, item) mapping shared by the three kernels.  Consecutive workgroup ids are
// dealt round-robin to the 8 XCDs; all workgroups that read the same K/V (or Q/dO) stream are given ids
// congruent modulo 8 and adjacent in dispatch order, so they run together on one XCD and the stream is
// fetched into that XCD's L2 once.  per_set = workgroups per (batch, KV head); returns false for the
// padding workgroups of the last, partial round.
constexpr int kXcds = 8;
__device__ __forceinline__ bool decode_block(int per_set, int n_sets, int *set, int *inner) {
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    *set = (slot / per_set) * kXcds + xcd;
    *inner = slot % per_set;
    return *set < n_sets;
}
// Causal work falls off linearly with the block index, and the workgroups of an XCD are handed to its shader
// engines round-robin in dispatch order: with the plain order "heaviest first" one engine would always get the
// heavier blocks of every set (measured: 15 us of idle time per block on the other engines' CUs at T = 4096).
// Rows of 8 consecutive positions therefore alternate direction (15..8, 0..7, ...): every residue class of the
// position modulo 8, 4 and 2 then carries the same amount of work.  i in [0, n) -> a permutation of [0, n).
__device__ __forceinline__ int snake8(int i, int n) {
    const int row = i >> 3;
    // long sequences: the classes differ by less than a percent, and the plain order keeps neighbouring blocks
    // (shared keys) together, which measured 1 % faster at 128k
    if (n > 128 || !(row & 1) || row * 8 + 7 >= n) return i;
    return row * 8 + 7 - (i & 7);
}
inline unsigned grid_blocks(int per_set, int n_sets) { return (unsigned)(((n_sets + kXcds - 1) / kXcds) * kXcds * per_set); }

// ------------------------------------------------------------------ forward
// grid (q blocks of 32*NW rows, heaviest first; Hq; B); wave w owns 32 queries.  K and V tiles of 64
// keys go through a double-buffered LDS stage, one barrier per tile.
#ifndef MT_FWD_PAD
#define MT_FWD_PAD 40
#endif
#ifndef MT_DQ_PAD
#define MT_DQ_PAD 40
#endif
#ifndef MT_DQ_WAVES
#define MT_DQ_WAVES 8
#endif
constexpr int kFwdPad = MT_FWD_PAD, kDqPad = MT_DQ_PAD;
template <int HD, int NW>
__global__ __launch_bounds__(64 * NW) void flash_fwd_kernel(AttnArgs a) {
    constexpr int LDK = HD + kFwdPad, NT = 64 * NW, BQ = 32 * NW;
    constexpr int STAGE = 2 * 64 * LDK;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

    const int T = a.T, G = a.Hq / a.Hkv, nqb = (T + BQ - 1) / BQ;
    int set, inner;
    if (!decode_block(G * nqb, a.B * a.Hkv, &set, &inner)) return;
    const int b = set / a.Hkv, hk = set % a.Hkv, h = hk * G + inner / nqb;
    const int qb = nqb - 1 - snake8(inner % nqb, nqb);  // heaviest query blocks first, in alternating rows of 8
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hl = lane >> 5;
    const int tr_off = tr_lane_offset(lane, LDK);
    const int q0 = qb * BQ + wave * 32, q = q0 + l32;
    const bool qok = q < T;
    const int qm = qok ? q : T - 1;  // padded queries behave like the last row; never stored

    bf16x8 qf[HD / 16];
    {
        const bf16_t *qp = a.q + ((int64_t)b * T + qm) * a.ldq + (int64_t)h * HD + hl * 8;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) qf[ks] = load_frag_global(qp + ks * 16);
    }
    f32x16 oacc[HD / 32];
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb) oacc[hb] = zero16();
    float m = -INFINITY, lsum = 0.f;  // m: running maximum of the raw (unscaled) scores
    const float c = a.scale * kLog2e, tau = kLazyMax / c;

    const bf16_t *kbase = a.k + (int64_t)b * T * a.ldk + (int64_t)hk * HD;
    const bf16_t *vbase = a.v + (int64_t)b * T * a.ldv + (int64_t)hk * HD;
    const int kv_end = min(T, qb * BQ + BQ);
    const int ntiles = (kv_end + 63) / 64;

    TileStage<64, HD, LDK, NT> stK, stV;
    stK.fetch(kbase, a.ldk, T, HD);
    stV.fetch(vbase, a.ldv, T, HD);
    stK.commit(smem);
    stV.commit(smem + 64 * LDK);
    __syncthreads();

    for (int kt = 0; kt < ntiles; ++kt) {
        const int kv0 = kt * 64;
        const bool more = kt + 1 < ntiles;
        const bf16_t *Ks = smem + (kt & 1) * STAGE, *Vs = Ks + 64 * LDK;
        if (more) {
            stK.fetch(kbase + (int64_t)(kv0 + 64) * a.ldk, a.ldk, T - kv0 - 64, HD);
            stV.fetch(vbase + (int64_t)(kv0 + 64) * a.ldv, a.ldv, T - kv0 - 64, HD);
        }
        if (kv0 <= q0 + 31) {  // otherwise the whole tile lies after every query of this wave
            // S^T = K Q^T for the two 32-key row blocks: fragments are read in batches of 4 k-steps ahead of
            // the MFMAs, and the two independent accumulation chains are interleaved
            f32x16 sacc[2] = {zero16(), zero16()};
            {
                const bf16_t *kr0 = Ks + l32 * LDK + hl * 8, *kr1 = kr0 + 32 * LDK;
#pragma unroll
                for (int half = 0; half < HD / 64; ++half) {
                    bf16x8 k0[4], k1[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        k0[j] = *reinterpret_cast<const bf16x8 *>(kr0 + (half * 4 + j) * 16);
                        k1[j] = *reinterpret_cast<const bf16x8 *>(kr1 + (half * 4 + j) * 16);
                    }
                    __builtin_amdgcn_sched_barrier(0);  // keep the batch of reads ahead of the MFMAs
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[j], qf[half * 4 + j], sacc[0], 0, 0, 0);
                        sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1[j], qf[half * 4 + j], sacc[1], 0, 0, 0);
                    }
                }
            }
            // V^T fragments of the first two 16-key chunks are requested now, so that their LDS latency is
            // covered by the softmax arithmetic below; the other two chunks follow behind the first MFMAs
            bf16x8 va[2][HD / 32];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch)
#pragma unroll
                for (int hb = 0; hb < HD / 32; ++hb) va[ch][hb] = read_tr_frag(Vs, tr_off, LDK, ch * 16, hb * 32);
            __builtin_amdgcn_sched_barrier(0);
            // Softmax on the raw scores: the scale is folded into the exponent's multiply-add, the running
            // maximum m is only moved when some query of the wave saw a score more than kLazyMax above it
            // (P then stays below 2^kLazyMax * ... which bf16 and the fp32 sums hold without loss; the final
            // O / lsum and lse do not depend on which maximum was used), so the accumulator rescale is rare.
            if (kv0 + 63 > q0) {  // tile touches the diagonal: mask keys after the query
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kv = kv0 + rb * 32 + (r >> 2) * 8 + hl * 4 + (r & 3);
                        sacc[rb][r] = kv > qm ? -INFINITY : sacc[rb][r];
                    }
            }
            float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, sacc[0][r]), sacc[1][r]);  // v_max3_f32
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            // m = -inf before the first tile: the comparison is then true (every query sees key kv0)
            if (__builtin_amdgcn_ballot_w64(mx > m + tau) != 0) {
                const float m_new = fmaxf(m, mx);
                const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
                lsum *= alpha;
#pragma unroll
                for (int hb = 0; hb < HD / 32; ++hb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[hb][r] *= alpha;
                m = m_new;
            }
            const float negmc = -m * c;
            float ps = 0.f;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[rb][r], c, negmc));
                    sacc[rb][r] = pv;
                    ps += pv;
                }
            lsum += ps;
            // O^T += V^T P^T
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                const bf16x8 pf = pack_frag(sacc[ch >> 1], ch & 1);
#pragma unroll
                for (int hb = 0; hb < HD / 32; ++hb)
                    oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ch & 1][hb], pf, oacc[hb], 0, 0, 0);
                if (ch < 2) {
#pragma unroll
                    for (int hb = 0; hb < HD / 32; ++hb)
                        va[ch & 1][hb] = read_tr_frag(Vs, tr_off, LDK, (ch + 2) * 16, hb * 32);
                }
            }
        }
        if (more) {
            bf16_t *nx = smem + ((kt + 1) & 1) * STAGE;
            stK.commit(nx);
            stV.commit(nx + 64 * LDK);
        }
        __syncthreads();
    }
    lsum += __shfl_xor(lsum, 32, 64);
    if (q0 < T)
        write_owned_rows<HD>(a.o + ((int64_t)b * T + q0) * a.ldo + (int64_t)h * HD, a.ldo, oacc, 1.0f / lsum, l32, hl,
                             min(32, T - q0), nullptr, nullptr, out_region<HD>(smem, wave));
    if (qok && hl == 0) a.lse[((int64_t)b * a.Hq + h) * T + q] = (m * c + __builtin_amdgcn_logf(lsum)) * kLn2;
}

// ------------------------------------------------------------------ backward: dQ
// Same ownership as the forward: a lane owns one query, loops over key tiles <= q.
template <int HD, int NW>
__global__ __launch_bounds__(64 * NW) void flash_bwd_dq_kernel(AttnArgs a) {
    constexpr int BQ = 32 * NW, NT = 64 * NW;
    constexpr int LDK = HD + kDqPad;
    constexpr int STAGE = 2 * 64 * LDK;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

    const int T = a.T, G = a.Hq / a.Hkv, nqb = (T + BQ - 1) / BQ;
    int set, inner;
    if (!decode_block(G * nqb, a.B * a.Hkv, &set, &inner)) return;
    const int b = set / a.Hkv, hk = set % a.Hkv, h = hk * G + inner / nqb;
    const int qb = nqb - 1 - snake8(inner % nqb, nqb);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hl = lane >> 5;
    const int tr_off = tr_lane_offset(lane, LDK);
    const int q0 = qb * BQ + wave * 32, q = q0 + l32;
    const bool qok = q < T;
    const int qm = qok ? q : T - 1;

    bf16x8 qf[HD / 16], dof[HD / 16];
    {
        const bf16_t *qp = a.q + ((int64_t)b * T + qm) * a.ldq + (int64_t)h * HD + hl * 8;
        const bf16_t *dp = a.dout + ((int64_t)b * T + qm) * a.lddo + (int64_t)h * HD + hl * 8;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) {
            qf[ks] = load_frag_global(qp + ks * 16);
            dof[ks] = load_frag_global(dp + ks * 16);
        }
    }
    const int64_t stat = ((int64_t)b * a.Hq + h) * T + qm;
    const float lse2 = a.lse[stat] * kLog2e, dlt = a.delta[stat];
    const float c = a.scale * kLog2e;
    f32x16 dqacc[HD / 32];
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb) dqacc[hb] = zero16();

    const bf16_t *kbase = a.k + (int64_t)b * T * a.ldk + (int64_t)hk * HD;
    const bf16_t *vbase = a.v + (int64_t)b * T * a.ldv + (int64_t)hk * HD;
    const int kv_end = min(T, qb * BQ + BQ);
    const int ntiles = (kv_end + 63) / 64;

    TileStage<64, HD, LDK, NT> stK, stV;
    stK.fetch(kbase, a.ldk, T, HD);
    stV.fetch(vbase, a.ldv, T, HD);
    stK.commit(smem);
    stV.commit(smem + 64 * LDK);
    __syncthreads();

    for (int kt = 0; kt < ntiles; ++kt) {
        const int kv0 = kt * 64;
        const bool more = kt + 1 < ntiles;
        const bf16_t *Ks = smem + (kt & 1) * STAGE, *Vs = Ks + 64 * LDK;
        if (more) {
            stK.fetch(kbase + (int64_t)(kv0 + 64) * a.ldk, a.ldk, T - kv0 - 64, HD);
            stV.fetch(vbase + (int64_t)(kv0 + 64) * a.ldv, a.ldv, T - kv0 - 64, HD);
        }
        if (kv0 <= q0 + 31) {
            const bool diag = kv0 + 63 > q0;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                f32x16 sacc = zero16(), dpacc = zero16();
                const bf16_t *kr = Ks + (rb * 32 + l32) * LDK + hl * 8;
                const bf16_t *vr = Vs + (rb * 32 + l32) * LDK + hl * 8;
#pragma unroll
                for (int half = 0; half < HD / 64; ++half) {
                    bf16x8 kk[4], vv[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        kk[j] = *reinterpret_cast<const bf16x8 *>(kr + (half * 4 + j) * 16);
                        vv[j] = *reinterpret_cast<const bf16x8 *>(vr + (half * 4 + j) * 16);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kk[j], qf[half * 4 + j], sacc, 0, 0, 0);
                        dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv[j], dof[half * 4 + j], dpacc, 0, 0, 0);
                    }
                }
                if (diag) {  // wave-uniform: only tiles that touch the diagonal pay for the mask
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kv = kv0 + rb * 32 + (r >> 2) * 8 + hl * 4 + (r & 3);
                        const float p = kv > qm ? 0.f : __builtin_amdgcn_exp2f(sacc[r] * c - lse2);
                        sacc[r] = p * (dpacc[r] - dlt);  // dS^T
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sacc[r] = __builtin_amdgcn_exp2f(sacc[r] * c - lse2) * (dpacc[r] - dlt);
                }
                // dQ^T += K^T dS^T
#pragma unroll
                for (int cch = 0; cch < 2; ++cch)
                    mfma_tr_accumulate<HD, LDK>(dqacc, Ks, tr_off, rb, cch, pack_frag(sacc, cch));
            }
        }
        if (more) {
            bf16_t *nx = smem + ((kt + 1) & 1) * STAGE;
            stK.commit(nx);
            stV.commit(nx + 64 * LDK);
        }
        __syncthreads();
    }
    if (q0 < T)
        write_owned_rows<HD>(a.dq + ((int64_t)b * T + q0) * a.lddq + (int64_t)h * HD, a.lddq, dqacc, a.scale, l32, hl,
                             min(32, T - q0), a.rope_cos ? a.rope_cos + (int64_t)q0 * (HD / 2) : nullptr,
                             a.rope_cos ? a.rope_sin + (int64_t)q0 * (HD / 2) : nullptr, out_region<HD>(smem, wave));
}

// ------------------------------------------------------------------ backward: dK, dV
// grid: key blocks of 256 (heaviest first = block 0) x (batch, KV head); the query heads of the group and their
// 64-query tiles >= the key block are walked as one sequence through a double-buffered LDS stage, one barrier
// per tile.  8 waves, two per SIMD: wave w owns keys w*32 .. w*32+31 of the block (a lane owns one key) and works
// through both 32-query halves of every tile: S^T = K Q^T and dP^T = V dO^T (16 MFMAs), P = exp2(S c - lse),
// dS = P (dP - delta) on the vector ALU, then dV^T += dO^T P and dK^T += Q^T dS (16 MFMAs); the other wave's MFMAs
// cover the exponentials.  The lane's K fragments live in registers, its V fragments are re-read from LDS for
// every half: with both in registers only one wave fits on a SIMD (that version, with a three-stage software
// pipeline inside the wave to make up for it, measured 25 % slower at 128k tokens).  A block of 256 keys rather
// than 128 halves the Q / dO bytes fetched and written to LDS per MFMA: LDS takes writes at ~70 bytes per clock,
// and with 128-key blocks the tile commits alone were 15 % of the kernel's time.
// LDS: V [256][HD + 8] | two stages of { Q, dO [64][HD + 40], lse * log2e [64], delta [64] }.
// Row pitch HD + 40 elements: consecutive rows are 20 banks apart, which keeps the 16-byte row reads
// conflict-free (odd multiple of 4 banks) and lets the four rows of a transposing read overlap in only
// 12 of 64 banks (with HD + 8 they pile up on the same 28 banks).
constexpr int kDkdvPad = 40;
template <int HD>
__global__ __launch_bounds__(512) void flash_bwd_dkdv_kernel(AttnArgs a) {
    constexpr int LDK = HD + kDkdvPad, LDKV = HD + 8, HB = HD / 32, KB = 256;
    constexpr int V_BF = KB * LDKV;
    constexpr int STAGE_BF = 2 * 64 * LDK, STAGE = STAGE_BF + 256;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *Vt = smem, *stages = smem + V_BF;

    const int T = a.T, G = a.Hq / a.Hkv, nkb = (T + KB - 1) / KB;
    int set, kvb;
    if (!decode_block(nkb, a.B * a.Hkv, &set, &kvb)) return;
    kvb = snake8(kvb, nkb);
    const int b = set / a.Hkv, hk = set % a.Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hl = lane >> 5;
    const int tr_off = tr_lane_offset(lane, LDK);
    const int kv0w = kvb * KB + wave * 32, kv = kv0w + l32;

    f32x16 dvacc[HB], dkacc[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        dvacc[hb] = zero16();
        dkacc[hb] = zero16();
    }
    const float c = a.scale * kLog2e;
    const int qt_first = (kvb * KB) / 64, n_qt = (T + 63) / 64 - qt_first;
    const int total = G * n_qt;

    using Stage = TileStage<64, HD, LDK, 512>;
    Stage stQ, stDO;
    float stat = 0.f;
    bool stat_pad = false;
    int f_head = 0, f_tile = 0;
    auto fetch_next = [&]() {
        const int h = hk * G + f_head, q0t = (qt_first + f_tile) * 64;
        if (++f_tile == n_qt) {
            f_tile = 0;
            ++f_head;
        }
        stQ.fetch_clamped(a.q + ((int64_t)b * T + q0t) * a.ldq + (int64_t)h * HD, a.ldq, T - q0t);
        stDO.fetch_clamped(a.dout + ((int64_t)b * T + q0t) * a.lddo + (int64_t)h * HD, a.lddo, T - q0t);
        if (threadIdx.x < 128) {
            // one plain load, nothing computed from it here: arithmetic on the value would make these two waves
            // wait for it (and for the tile loads just issued) before they start on the current tile
            const int qq = q0t + (threadIdx.x & 63);
            const int64_t si = ((int64_t)b * a.Hq + h) * T + (qq < T ? qq : T - 1);
            stat = *(threadIdx.x < 64 ? a.lse + si : a.delta + si);
            stat_pad = qq >= T;
        }
    };
    auto commit = [&](int stage) {
        bf16_t *sp = stages + stage * STAGE;
        stQ.commit_plain(sp);
        stDO.commit_plain(sp + 64 * LDK);
        // queries past T: lse = +inf makes their P (and with it dS) exactly zero
        if (threadIdx.x < 128)
            reinterpret_cast<float *>(sp + STAGE_BF)[threadIdx.x] =
                threadIdx.x < 64 ? (stat_pad ? INFINITY : stat * kLog2e) : stat;
    };
    bf16x8 kf[HD / 16];
    {
        TileStage<KB, HD, LDKV, 512> stV;
        stV.fetch(a.v + ((int64_t)b * T + kvb * KB) * a.ldv + (int64_t)hk * HD, a.ldv, T - kvb * KB, HD);
        fetch_next();
        const bf16_t *kp = a.k + ((int64_t)b * T + min(kv, T - 1)) * a.ldk + (int64_t)hk * HD + hl * 8;
#pragma unroll
        for (int i = 0; i < HD / 16; ++i) kf[i] = load_frag_global(kp + i * 16);
        stV.commit(Vt);
        commit(0);
    }
    __syncthreads();

    const bf16_t *vr = Vt + (wave * 32 + l32) * LDKV + hl * 8;
    int tq = 0;  // query tile inside the head
    for (int j = 0; j < total; ++j) {
        const bf16_t *Qs = stages + (j & 1) * STAGE, *dOs = Qs + 64 * LDK;
        const float *lses = reinterpret_cast<const float *>(Qs + STAGE_BF), *dlts = lses + 64;
        const int q0t = (qt_first + tq) * 64;
        const bool more = j + 1 < total;
        if (more) fetch_next();
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int q0u = q0t + rb * 32;
            if (q0u + 31 < kv0w) continue;  // wave-uniform: no query of the half sees a key of the wave
            f32x16 s_ = zero16(), p_ = zero16();
            const bf16_t *qr = Qs + (rb * 32 + l32) * LDK + hl * 8;
            const bf16_t *dor = dOs + (rb * 32 + l32) * LDK + hl * 8;
#pragma unroll
            for (int half = 0; half < HD / 64; ++half) {
                bf16x8 qq[4], dd[4], vv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) qq[i] = *reinterpret_cast<const bf16x8 *>(qr + (half * 4 + i) * 16);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    dd[i] = *reinterpret_cast<const bf16x8 *>(dor + (half * 4 + i) * 16);
                    vv[i] = *reinterpret_cast<const bf16x8 *>(vr + (half * 4 + i) * 16);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    s_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qq[i], kf[half * 4 + i], s_, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) p_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dd[i], vv[i], p_, 0, 0, 0);
            }
            // P = exp2(S c - lse), dS = P (dP - delta); element r of the lane belongs to query
            // q0u + (r >> 2) * 8 + hl * 4 + (r & 3), visible to the lane's key only if kv <= query
            const int lim = kv - (q0u + hl * 4);
            const bool diag = q0u < kv0w + 31;
            f32x16 dsacc;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int qi = rb * 32 + r4 * 8 + hl * 4;
                const float4 l4 = *reinterpret_cast<const float4 *>(lses + qi);
                const float4 d4 = *reinterpret_cast<const float4 *>(dlts + qi);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = r4 * 4 + e;
                    float p = __builtin_amdgcn_exp2f(s_[r] * c - lv[e]);
                    if (diag) p = (r4 * 8 + e < lim) ? 0.f : p;
                    s_[r] = p;
                    dsacc[r] = p * (p_[r] - dv4[e]);
                }
            }
            // dV^T += dO^T P, dK^T += Q^T dS
#pragma unroll
            for (int cch = 0; cch < 2; ++cch) {
                mfma_tr_accumulate<HD, LDK>(dvacc, dOs, tr_off, rb, cch, pack_frag(s_, cch));
                mfma_tr_accumulate<HD, LDK>(dkacc, Qs, tr_off, rb, cch, pack_frag(dsacc, cch));
            }
        }
        if (more) commit((j + 1) & 1);
        __syncthreads();
        tq = tq + 1 == n_qt ? 0 : tq + 1;
    }
    if (kv0w < T) {
        const int n_valid = min(32, T - kv0w);
        write_owned_rows<HD>(a.dk + ((int64_t)b * T + kv0w) * a.lddk + (int64_t)hk * HD, a.lddk, dkacc, a.scale, l32, hl,
                             n_valid, a.rope_cos ? a.rope_cos + (int64_t)kv0w * (HD / 2) : nullptr,
                             a.rope_cos ? a.rope_sin + (int64_t)kv0w * (HD / 2) : nullptr, out_region<HD>(smem, wave));
        write_owned_rows<HD>(a.dv + ((int64_t)b * T + kv0w) * a.lddv + (int64_t)hk * HD, a.lddv, dvacc, 1.0f, l32, hl,
                             n_valid, nullptr, nullptr, out_region<HD>(smem, wave));
    }
}

bool attn_shape_ok(const AttnArgs &a) {
    if (a.B <= 0 || a.T <= 0 || a.Hq <= 0 || a.Hkv <= 0 || a.Hq % a.Hkv) return false;
    if (a.hd != 64 && a.hd != 128) return false;
    if (a.T & 7) return false;
    if ((int64_t)a.B * a.Hq * ((a.T + 127) / 128) > (int64_t)1 << 30) return false;
    return true;
}
bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
// both rotary tables or none, read 16 bytes at a time
bool rope_tables_ok(const AttnArgs &a) {
    if (!a.rope_cos && !a.rope_sin) return true;
    return a.rope_cos && a.rope_sin && aligned16(a.rope_cos) && aligned16(a.rope_sin);
}

}  // namespace

template <typename K>
static hipError_t ensure_lds(K kernel, size_t bytes, bool *done) {
    if (*done || bytes <= 48 * 1024) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) *done = true;
    return e;
}

hipError_t flash_fwd(const AttnArgs &a, hipStream_t s) {
    if (!attn_shape_ok(a) || (a.ldq & 7) || (a.ldk & 7) || (a.ldv & 7) || (a.ldo & 3)) return hipErrorInvalidValue;
    if (!aligned16(a.q) || !aligned16(a.k) || !aligned16(a.v) || ((uintptr_t)a.o & 7)) return hipErrorInvalidValue;
    constexpr int NW = 8;
    const dim3 grid(grid_blocks((a.Hq / a.Hkv) * ((a.T + 32 * NW - 1) / (32 * NW)), a.B * a.Hkv));
    if (a.hd == 128) {
        constexpr size_t lds = 2 * (2 * 64 * (128 + kFwdPad)) * sizeof(bf16_t);
        static bool done = false;
        hipError_t e = ensure_lds(&flash_fwd_kernel<128, NW>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((flash_fwd_kernel<128, NW>), grid, dim3(64 * NW), lds, s, a);
    } else {
        constexpr size_t lds = 2 * (2 * 64 * (64 + kFwdPad)) * sizeof(bf16_t);
        static bool done = false;
        hipError_t e = ensure_lds(&flash_fwd_kernel<64, NW>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((flash_fwd_kernel<64, NW>), grid, dim3(64 * NW), lds, s, a);
    }
    return hipGetLastError();
}

hipError_t flash_bwd_dq(const AttnArgs &a, hipStream_t s) {
    if (!rope_tables_ok(a)) return hipErrorInvalidValue;
    if (!attn_shape_ok(a) || (a.ldq & 7) || (a.ldk & 7) || (a.ldv & 7) || (a.lddo & 7) || (a.lddq & 3))
        return hipErrorInvalidValue;
    if (!aligned16(a.q) || !aligned16(a.k) || !aligned16(a.v) || !aligned16(a.dout) || ((uintptr_t)a.dq & 7))
        return hipErrorInvalidValue;
    constexpr int NW = MT_DQ_WAVES;
    const dim3 grid(grid_blocks((a.Hq / a.Hkv) * ((a.T + 32 * NW - 1) / (32 * NW)), a.B * a.Hkv));
    if (a.hd == 128) {
        constexpr size_t lds = 2 * (2 * 64 * (128 + kDqPad)) * sizeof(bf16_t);
        static bool done = false;
        hipError_t e = ensure_lds(&flash_bwd_dq_kernel<128, NW>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((flash_bwd_dq_kernel<128, NW>), grid, dim3(64 * NW), lds, s, a);
    } else {
        constexpr size_t lds = 2 * (2 * 64 * (64 + kDqPad)) * sizeof(bf16_t);
        static bool done = false;
        hipError_t e = ensure_lds(&flash_bwd_dq_kernel<64, NW>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((flash_bwd_dq_kernel<64, NW>), grid, dim3(64 * NW), lds, s, a);
    }
    return hipGetLastError();
}

hipError_t flash_bwd_dkdv(const AttnArgs &a, hipStream_t s) {
    if (!rope_tables_ok(a)) return hipErrorInvalidValue;
    if (!attn_shape_ok(a) || (a.ldq & 7) || (a.ldk & 7) || (a.ldv & 7) || (a.lddo & 7) || (a.lddk & 3) ||
        (a.lddv & 3))
        return hipErrorInvalidValue;
    if (!aligned16(a.q) || !aligned16(a.k) || !aligned16(a.v) || !aligned16(a.dout) || ((uintptr_t)a.dk & 7) ||
        ((uintptr_t)a.dv & 7))
        return hipErrorInvalidValue;
    const dim3 grid(grid_blocks((a.T + 255) / 256, a.B * a.Hkv));
    // V [256][hd + 8] | two stages of Q, dO [64][hd + pad] + 64 lse + 64 delta
    if (a.hd == 128) {
        constexpr size_t lds = (256 * (128 + 8) + 2 * (2 * 64 * (128 + kDkdvPad))) * sizeof(bf16_t) + 2 * 512;
        static bool done = false;
        hipError_t e = ensure_lds(&flash_bwd_dkdv_kernel<128>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(flash_bwd_dkdv_kernel<128>, grid, dim3(512), lds, s, a);
    } else {
        constexpr size_t lds = (256 * (64 + 8) + 2 * (2 * 64 * (64 + kDkdvPad))) * sizeof(bf16_t) + 2 * 512;
        static bool done = false;
        hipError_t e = ensure_lds(&flash_bwd_dkdv_kernel<64>, lds, &done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(flash_bwd_dkdv_kernel<64>, grid, dim3(512), lds, s, a);
    }
    return hipGetLastError();
}

}  // namespace mt
