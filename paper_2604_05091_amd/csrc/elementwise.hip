// HBM-bound kernels of the transformer block: transpose, RMSNorm, rotary embedding,
// SwiGLU, embedding gather / scatter, cross-entropy and a fixed-order sum.
//
// All of them move 16 bytes per lane per access (8 bf16 or 4 fp32), do their
// arithmetic in fp32 and reduce inside a 64-lane wave with cross-lane shuffles.
// None uses atomics, so every result is bit-reproducible from run to run.
#include <atomic>

#include "common.h"

namespace mt {

namespace {

__device__ __forceinline__ void unpack8(const uint4 &u, float *f) {
    f[0] = bflo(u.x); f[1] = bfhi(u.x); f[2] = bflo(u.y); f[3] = bfhi(u.y);
    f[4] = bflo(u.z); f[5] = bfhi(u.z); f[6] = bflo(u.w); f[7] = bfhi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float *f) {
    uint4 u;
    u.x = pack2bf(f[0], f[1]); u.y = pack2bf(f[2], f[3]); u.z = pack2bf(f[4], f[5]); u.w = pack2bf(f[6], f[7]);
    return u;
}

// ------------------------------------------------------------------ transpose
// 64 x 64 tile through LDS; 256 threads; 16-byte global accesses on both sides.
__global__ __launch_bounds__(256) void transpose_kernel(TransposeArgs t) {
    __shared__ bf16_t tile[64][64 + 2];
    const int b0 = blockIdx.z / t.nb1, b1 = blockIdx.z % t.nb1;
    const bf16_t *in = t.in + b0 * t.in_s0 + b1 * t.in_s1;
    bf16_t *out = t.out + b0 * t.out_s0 + b1 * t.out_s1;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int chunk = tid + 256 * j, r = chunk >> 3, c = (chunk & 7) * 8;
        uint4 v = {0u, 0u, 0u, 0u};
        if (r0 + r < t.rows && c0 + c < t.cols)
            v = *reinterpret_cast<const uint4 *>(in + (int64_t)(r0 + r) * t.ld_in + c0 + c);
        uint32_t *dst = reinterpret_cast<uint32_t *>(&tile[r][c]);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int chunk = tid + 256 * j, c = chunk & 63, r = (chunk >> 6) * 8;  // out row c, out cols r..r+7
        if (c0 + c < t.cols && r0 + r < t.rows) {
            uint4 v;
            v.x = (uint32_t)tile[r + 0][c] | ((uint32_t)tile[r + 1][c] << 16);
            v.y = (uint32_t)tile[r + 2][c] | ((uint32_t)tile[r + 3][c] << 16);
            v.z = (uint32_t)tile[r + 4][c] | ((uint32_t)tile[r + 5][c] << 16);
            v.w = (uint32_t)tile[r + 6][c] | ((uint32_t)tile[r + 7][c] << 16);
            *reinterpret_cast<uint4 *>(out + (int64_t)(c0 + c) * t.ld_out + r0 + r) = v;
        }
    }
}

// ------------------------------------------------------------------ RMSNorm forward
// One wave per row; the row is held in registers (NCH chunks of 8 per lane).
template <int NCH>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(bf16_t *y, const bf16_t *x, const bf16_t *gain, int64_t n,
                                                          int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const int nch = d >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + row * d);
    uint4 xv[NCH];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
            xv[i] = xr[c];
            float f[8];
            unpack8(xv[i], f);
#pragma unroll
            for (int k = 0; k < 8; ++k) ss += f[k] * f[k];
        }
    }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
    const uint4 *gr = reinterpret_cast<const uint4 *>(gain);
    uint4 *yr = reinterpret_cast<uint4 *>(y + row * d);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
            float f[8], gf[8];
            unpack8(xv[i], f);
            unpack8(gr[c], gf);
#pragma unroll
            for (int k = 0; k < 8; ++k) f[k] = f[k] * r * gf[k];
            yr[c] = pack8(f);
        }
    }
}

// ------------------------------------------------------------------ RMSNorm backward
// Wave w walks rows w, w + W, ...  Per row: r and dot = sum_j g_j dy_j x_j, then
// dx = r g dy - x r^3 dot / d (+ dres).  The gain gradient sum_t dy x r is kept in
// registers per lane and column, summed over the 4 waves of the block through LDS and
// written as one partial row per block; a second kernel adds the partial rows in order.
constexpr int kNormBwdBlocks = 512;

template <int NCH>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(bf16_t *dx, float *partial, const bf16_t *dy,
                                                          const bf16_t *x, const bf16_t *gain, const bf16_t *dres,
                                                          int64_t n, int d, float eps) {
    extern __shared__ float red[];  // [d]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nch = d >> 3;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    float dg[NCH][8];
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int k = 0; k < 8; ++k) dg[i][k] = 0.f;
    const uint4 *gr = reinterpret_cast<const uint4 *>(gain);

    // up to 8 chunks per lane (d <= 4096) the row stays in registers between the two passes; wider rows are read again
    constexpr bool kKeep = NCH <= 8;
    for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < n; row += nwaves) {
        const uint4 *xr = reinterpret_cast<const uint4 *>(x + row * d);
        const uint4 *dyr = reinterpret_cast<const uint4 *>(dy + row * d);
        uint4 xk[kKeep ? NCH : 1], yk[kKeep ? NCH : 1];
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) {
                float xf[8], yf[8], gf[8];
                const uint4 xu = xr[c], yu = dyr[c];
                if (kKeep) {
                    xk[i] = xu;
                    yk[i] = yu;
                }
                unpack8(xu, xf);
                unpack8(yu, yf);
                unpack8(gr[c], gf);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    ss += xf[k] * xf[k];
                    dot += gf[k] * yf[k] * xf[k];
                }
            }
        }
        ss = wave_sum(ss);
        dot = wave_sum(dot);
        const float r = 1.0f / sqrtf(ss / (float)d + eps);
        const float cc = r * r * r * dot / (float)d;
        uint4 *dxr = reinterpret_cast<uint4 *>(dx + row * d);
        const uint4 *rr = dres ? reinterpret_cast<const uint4 *>(dres + row * d) : nullptr;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) {
                float xf[8], yf[8], gf[8], of[8];
                unpack8(kKeep ? xk[i] : xr[c], xf);
                unpack8(kKeep ? yk[i] : dyr[c], yf);
                unpack8(gr[c], gf);
                if (rr) {
                    unpack8(rr[c], of);
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) of[k] = 0.f;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    of[k] += r * gf[k] * yf[k] - xf[k] * cc;
                    dg[i][k] += yf[k] * xf[k] * r;
                }
                dxr[c] = pack8(of);
            }
        }
    }
    // block reduction of the gain-gradient partials in the fixed order ((w0 + w1) + w2) + w3
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int c = lane + 64 * i;
                if (c < nch)
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        if (w == 0) red[c * 8 + k] = dg[i][k];
                        else red[c * 8 + k] += dg[i][k];
                    }
            }
        }
        __syncthreads();
    }
    for (int j = threadIdx.x; j < d; j += 256) partial[(int64_t)blockIdx.x * d + j] = red[j];
}

// out[j] (+)= sum over rows of partial[r][j].  A block owns 32 columns; its 8 row groups each add every 8th row in
// order and the 8 group sums are added in order, so the result does not depend on the launch.
__global__ __launch_bounds__(256) void colsum_kernel(float *out, const float *partial, int nrows, int d, int accumulate) {
    __shared__ float red[8][32];
    const int cl = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int j = blockIdx.x * 32 + cl;
    float s = 0.f;
    if (j < d)
        for (int r = rg; r < nrows; r += 8) s += partial[(int64_t)r * d + j];
    red[rg][cl] = s;
    __syncthreads();
    if (rg == 0 && j < d) {
        float t = red[0][cl];
#pragma unroll
        for (int g = 1; g < 8; ++g) t += red[g][cl];
        out[j] = accumulate ? out[j] + t : t;
    }
}

// ------------------------------------------------------------------ bias gradient (column sums of a bf16 matrix)
// block (bx, by): 16-byte column chunk bx*256 + thread of the rows [by*rpb, (by+1)*rpb) -> partial[by][cols]
constexpr int kBiasGradRowBlocks = 128;
__global__ __launch_bounds__(256) void bias_grad_partial_kernel(float *partial, const bf16_t *x, int64_t ld, int64_t n,
                                                                int cols, int64_t rpb) {
    const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (c >= cols) return;
    const int64_t r0 = (int64_t)blockIdx.y * rpb, r1 = min(n, r0 + rpb);
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t r = r0; r < r1; ++r) {
        const uint4 u = *reinterpret_cast<const uint4 *>(x + r * ld + c);
        a[0] += bflo(u.x); a[1] += bfhi(u.x); a[2] += bflo(u.y); a[3] += bfhi(u.y);
        a[4] += bflo(u.z); a[5] += bfhi(u.z); a[6] += bflo(u.w); a[7] += bfhi(u.w);
    }
    float *p = partial + (int64_t)blockIdx.y * cols + c;
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = a[e];
}

// ------------------------------------------------------------------ rotary embedding
// thread = (row, head, group of 8 pair indices j); pairs (j, j + hd/2)
__global__ __launch_bounds__(256) void rope_kernel(bf16_t *x, int64_t ld, int64_t n, int T, int n_heads, int hd,
                                                   const float *cs, const float *sn, float sign) {
    const int half = hd >> 1, gpr = half >> 3;  // groups per head
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = n * n_heads * gpr;
    if (idx >= total) return;
    const int gi = (int)(idx % gpr);
    const int h = (int)((idx / gpr) % n_heads);
    const int64_t row = idx / ((int64_t)gpr * n_heads);
    const int t = (int)(row % T);
    bf16_t *p = x + row * ld + (int64_t)h * hd + gi * 8;
    uint4 *pa = reinterpret_cast<uint4 *>(p), *pb = reinterpret_cast<uint4 *>(p + half);
    float a[8], b[8];
    unpack8(*pa, a);
    unpack8(*pb, b);
    const float4 *cp = reinterpret_cast<const float4 *>(cs + (int64_t)t * half + gi * 8);
    const float4 *sp = reinterpret_cast<const float4 *>(sn + (int64_t)t * half + gi * 8);
    const float4 c0 = cp[0], c1 = cp[1], s0 = sp[0], s1 = sp[1];
    const float c[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    float oa[8], ob[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float sk = sign * s[k];
        oa[k] = a[k] * c[k] - b[k] * sk;
        ob[k] = b[k] * c[k] + a[k] * sk;
    }
    *pa = pack8(oa);
    *pb = pack8(ob);
}

// ------------------------------------------------------------------ SwiGLU
__device__ __forceinline__ float sigmoidf_(float v) { return sigmoid_rcp(v); }

__global__ __launch_bounds__(256) void swiglu_fwd_kernel(bf16_t *sout, const bf16_t *gu, int64_t n, int F) {
    const int cpr = F >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * cpr) return;
    const int64_t row = idx / cpr;
    const int c = (int)(idx % cpr) * 8;
    float g[8], u[8], o[8];
    unpack8(*reinterpret_cast<const uint4 *>(gu + row * 2 * F + c), g);
    unpack8(*reinterpret_cast<const uint4 *>(gu + row * 2 * F + F + c), u);
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = g[k] * sigmoidf_(g[k]) * u[k];
    *reinterpret_cast<uint4 *>(sout + row * F + c) = pack8(o);
}

__global__ __launch_bounds__(256) void swiglu_bwd_kernel(bf16_t *dgu, const bf16_t *ds, const bf16_t *gu, int64_t n,
                                                         int F) {
    const int cpr = F >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * cpr) return;
    const int64_t row = idx / cpr;
    const int c = (int)(idx % cpr) * 8;
    float g[8], u[8], d[8], og[8], ou[8];
    unpack8(*reinterpret_cast<const uint4 *>(gu + row * 2 * F + c), g);
    unpack8(*reinterpret_cast<const uint4 *>(gu + row * 2 * F + F + c), u);
    unpack8(*reinterpret_cast<const uint4 *>(ds + row * F + c), d);
#pragma unroll
    for (int k = 0; k < 8; ++k) swiglu_bwd_elem(d[k], g[k], u[k], &og[k], &ou[k]);
    *reinterpret_cast<uint4 *>(dgu + row * 2 * F + c) = pack8(og);
    *reinterpret_cast<uint4 *>(dgu + row * 2 * F + F + c) = pack8(ou);
}

// ------------------------------------------------------------------ embedding
__global__ __launch_bounds__(256) void embed_gather_kernel(bf16_t *h, const bf16_t *table, const int32_t *tokens,
                                                           int64_t n, int d) {
    const int cpr = d >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * cpr) return;
    const int64_t row = idx / cpr;
    const int c = (int)(idx % cpr);
    reinterpret_cast<uint4 *>(h + row * d)[c] = reinterpret_cast<const uint4 *>(table + (int64_t)tokens[row] * d)[c];
}

// one block per vocabulary row; positions of that token are summed in list order
__global__ __launch_bounds__(256) void embed_scatter_kernel(float *dtable, const bf16_t *dh, const int32_t *row_start,
                                                            const int32_t *order, int d) {
    const int v = blockIdx.x;
    const int beg = row_start[v], end = row_start[v + 1];
    const int cpr = d >> 3;
    for (int c = threadIdx.x; c < cpr; c += 256) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int i = beg; i < end; ++i) {
            float f[8];
            unpack8(reinterpret_cast<const uint4 *>(dh + (int64_t)order[i] * d)[c], f);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] += f[k];
        }
        float4 *o = reinterpret_cast<float4 *>(dtable + (int64_t)v * d + c * 8);
        o[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        o[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// ------------------------------------------------------------------ cross-entropy
// One block per row.  Pass 1: online (max, sum exp).  Pass 2: gradient.
__global__ __launch_bounds__(256) void cross_entropy_kernel(float *loss_rows, bf16_t *dlogits, const float *logits,
                                                            const int32_t *labels, int V, float inv_n) {
    __shared__ float sm[4], ssum[4];
    const int64_t row = blockIdx.x;
    const int label = labels[row];
    const float4 *z = reinterpret_cast<const float4 *>(logits + row * V);
    uint2 *dz = reinterpret_cast<uint2 *>(dlogits + row * V);
    const int nq = V >> 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (label < 0) {
        if (threadIdx.x == 0) loss_rows[row] = 0.f;
        for (int i = threadIdx.x; i < nq; i += 256) dz[i] = make_uint2(0u, 0u);
        return;
    }
    float mx = -INFINITY, sum = 0.f;
    for (int i = threadIdx.x; i < nq; i += 256) {
        const float4 v = z[i];
        const float m4 = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
        if (m4 > mx) {
            sum *= __expf(mx - m4);
            mx = m4;
        }
        sum += __expf(v.x - mx) + __expf(v.y - mx) + __expf(v.z - mx) + __expf(v.w - mx);
    }
    // combine (mx, sum) pairs: wave, then the 4 waves
    const float wmx = wave_max(mx);
    sum = wave_sum(mx == -INFINITY ? 0.f : sum * __expf(mx - wmx));
    if (lane == 0) {
        sm[wave] = wmx;
        ssum[wave] = sum;
    }
    __syncthreads();
    const float bmx = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float bsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (sm[w] != -INFINITY) bsum += ssum[w] * __expf(sm[w] - bmx);
    const float lse = bmx + __logf(bsum);
    if (threadIdx.x == 0) loss_rows[row] = lse - logits[row * V + label];
    for (int i = threadIdx.x; i < nq; i += 256) {
        const float4 v = z[i];
        float p0 = __expf(v.x - lse), p1 = __expf(v.y - lse), p2 = __expf(v.z - lse), p3 = __expf(v.w - lse);
        const int c = i * 4;
        if (label == c) p0 -= 1.f;
        if (label == c + 1) p1 -= 1.f;
        if (label == c + 2) p2 -= 1.f;
        if (label == c + 3) p3 -= 1.f;
        dz[i] = make_uint2(pack2bf(p0 * inv_n, p1 * inv_n), pack2bf(p2 * inv_n, p3 * inv_n));
    }
}

// fixed-order sum with one block of 1024 threads
__global__ __launch_bounds__(1024) void reduce_sum_kernel(float *out, const float *in, int64_t n, float scale,
                                                          int accumulate) {
    __shared__ float part[16];
    float s = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) s += in[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int i = 0; i < 16; ++i) t += part[i];
        out[0] = (accumulate ? out[0] : 0.f) + scale * t;
    }
}

// delta[b,h,t] = sum_j do[b,t,h,j] o[b,t,h,j]; hd/8 lanes per (token, head)
__global__ __launch_bounds__(256) void attn_delta_kernel(float *delta, const bf16_t *dout, int64_t lddo,
                                                         const bf16_t *o, int64_t ldo, int B, int T, int H, int hd) {
    const int lpg = hd >> 3;  // lanes per group: 8 or 16
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t grp = idx / lpg;
    const int li = (int)(idx % lpg);
    const int64_t total = (int64_t)B * T * H;
    float s = 0.f;
    int64_t row = 0;
    int h = 0;
    if (grp < total) {
        row = grp / H;
        h = (int)(grp % H);
        float a[8], b[8];
        unpack8(*reinterpret_cast<const uint4 *>(dout + row * lddo + (int64_t)h * hd + li * 8), a);
        unpack8(*reinterpret_cast<const uint4 *>(o + row * ldo + (int64_t)h * hd + li * 8), b);
#pragma unroll
        for (int k = 0; k < 8; ++k) s += a[k] * b[k];
    }
    for (int off = lpg >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (grp < total && li == 0) {
        const int64_t b = row / T, t = row % T;
        delta[(b * H + h) * T + t] = s;
    }
}

__global__ __launch_bounds__(256) void fill_kernel(uint32_t *p, uint32_t v, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t st = (size_t)gridDim.x * 256;
    for (; i < n; i += st) p[i] = v;
}

inline unsigned blocks_for(int64_t work, int per_block) { return (unsigned)((work + per_block - 1) / per_block); }

}  // namespace

hipError_t transpose_bf16(const TransposeArgs &t, hipStream_t s) {
    if (t.rows <= 0 || t.cols <= 0 || t.nb0 <= 0 || t.nb1 <= 0) return hipErrorInvalidValue;
    if ((t.rows & 7) || (t.cols & 7) || (t.ld_in & 7) || (t.ld_out & 7)) return hipErrorInvalidValue;
    if ((t.in_s0 & 7) || (t.in_s1 & 7) || (t.out_s0 & 7) || (t.out_s1 & 7)) return hipErrorInvalidValue;
    if (((uintptr_t)t.in & 15) || ((uintptr_t)t.out & 15)) return hipErrorInvalidValue;
    if (t.ld_in < t.cols || t.ld_out < t.rows) return hipErrorInvalidValue;
    const int64_t nz = (int64_t)t.nb0 * t.nb1;
    if (nz > 65535) return hipErrorInvalidValue;
    dim3 grid((t.cols + 63) / 64, (t.rows + 63) / 64, (unsigned)nz);
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, s, t);
    return hipGetLastError();
}

hipError_t rmsnorm_fwd(bf16_t *y, const bf16_t *x, const bf16_t *gain, int64_t n, int32_t d, float eps,
                       hipStream_t s) {
    if (n <= 0 || d <= 0 || (d & 7) || d > 8192) return hipErrorInvalidValue;
    const unsigned grid = blocks_for(n, 4);
    if (d <= 2048) hipLaunchKernelGGL(rmsnorm_fwd_kernel<4>, dim3(grid), dim3(256), 0, s, y, x, gain, n, d, eps);
    else if (d <= 4096) hipLaunchKernelGGL(rmsnorm_fwd_kernel<8>, dim3(grid), dim3(256), 0, s, y, x, gain, n, d, eps);
    else hipLaunchKernelGGL(rmsnorm_fwd_kernel<16>, dim3(grid), dim3(256), 0, s, y, x, gain, n, d, eps);
    return hipGetLastError();
}

size_t rmsnorm_bwd_ws_floats(int32_t d) { return (size_t)kNormBwdBlocks * (size_t)d; }

hipError_t rmsnorm_bwd(bf16_t *dx_out, float *dgain, const bf16_t *dy, const bf16_t *x, const bf16_t *gain,
                       const bf16_t *dres, float *partial, int64_t n, int32_t d, float eps, hipStream_t s,
                       int accumulate_dgain) {
    if (n <= 0 || d <= 0 || (d & 7) || d > 8192) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((n + 3) / 4 < kNormBwdBlocks ? (n + 3) / 4 : kNormBwdBlocks);
    const size_t lds = (size_t)d * sizeof(float);
    if (d <= 2048)
        hipLaunchKernelGGL(rmsnorm_bwd_kernel<4>, dim3(grid), dim3(256), lds, s, dx_out, partial, dy, x, gain, dres, n,
                           d, eps);
    else if (d <= 4096)
        hipLaunchKernelGGL(rmsnorm_bwd_kernel<8>, dim3(grid), dim3(256), lds, s, dx_out, partial, dy, x, gain, dres, n,
                           d, eps);
    else
        hipLaunchKernelGGL(rmsnorm_bwd_kernel<16>, dim3(grid), dim3(256), lds, s, dx_out, partial, dy, x, gain, dres,
                           n, d, eps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(colsum_kernel, dim3(blocks_for(d, 32)), dim3(256), 0, s, dgain, partial, (int)grid, d,
                       accumulate_dgain);
    return hipGetLastError();
}

// ---- RMSNorm backward for callers that may not allocate: the partial-gain-gradient workspace is a file-scope
// device array instead of a caller buffer.  Its name is only a host-side handle; the device address is looked up
// once per device (each device holds its own copy) and passed to the kernels like any other workspace.
constexpr int kStaticNormMaxD = 8192;
static __device__ __align__(256) float scratch[(size_t)kNormBwdBlocks * kStaticNormMaxD];  // 16 MiB per device
constexpr int kMaxDevices = 64;

hipError_t rmsnorm_bwd_static(bf16_t *dx_out, float *dgain, const bf16_t *dy, const bf16_t *x, const bf16_t *gain,
                              const bf16_t *dres, int64_t n, int32_t d, float eps, hipStream_t s) {
    static std::atomic<float *> scratch_of_device[kMaxDevices];
    if (d <= 0 || d > kStaticNormMaxD) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    float *ptr = scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_of_device[dev].store(ptr, std::memory_order_release);  // same value from every thread
    }
    // every partial row that the column sum reads is written by the first kernel of this call: nothing to clear
    return rmsnorm_bwd(dx_out, dgain, dy, x, gain, dres, ptr, n, d, eps, s, 0);
}

size_t bias_grad_ws_floats(int32_t cols) { return (size_t)kBiasGradRowBlocks * (size_t)cols; }

hipError_t bias_grad(float *db, const bf16_t *x, int64_t ld, int64_t n, int32_t cols, float *ws, hipStream_t s) {
    if (n <= 0 || cols <= 0 || (cols & 7) || (ld & 7)) return hipErrorInvalidValue;
    const int64_t rpb = (n + kBiasGradRowBlocks - 1) / kBiasGradRowBlocks;
    hipLaunchKernelGGL(bias_grad_partial_kernel, dim3(blocks_for(cols / 8, 256), kBiasGradRowBlocks), dim3(256), 0, s, ws, x,
                       ld, n, cols, rpb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(colsum_kernel, dim3(blocks_for(cols, 32)), dim3(256), 0, s, db, ws, kBiasGradRowBlocks, cols, 0);
    return hipGetLastError();
}

hipError_t rope_inplace(bf16_t *x, int64_t ld, int64_t n, int32_t T, int32_t n_heads, int32_t hd, const float *cs,
                        const float *sn, int sign, hipStream_t s) {
    if (n <= 0 || T <= 0 || n_heads <= 0 || (hd & 15) || (ld & 7)) return hipErrorInvalidValue;
    const int64_t total = n * n_heads * (hd >> 4);
    hipLaunchKernelGGL(rope_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, x, ld, n, T, n_heads, hd, cs, sn,
                       sign >= 0 ? 1.0f : -1.0f);
    return hipGetLastError();
}

hipError_t swiglu_fwd(bf16_t *sout, const bf16_t *gu, int64_t n, int32_t F, hipStream_t s) {
    if (n <= 0 || F <= 0 || (F & 7)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(swiglu_fwd_kernel, dim3(blocks_for(n * (F >> 3), 256)), dim3(256), 0, s, sout, gu, n, F);
    return hipGetLastError();
}

hipError_t swiglu_bwd(bf16_t *dgu, const bf16_t *ds, const bf16_t *gu, int64_t n, int32_t F, hipStream_t s) {
    if (n <= 0 || F <= 0 || (F & 7)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(blocks_for(n * (F >> 3), 256)), dim3(256), 0, s, dgu, ds, gu, n, F);
    return hipGetLastError();
}

hipError_t embed_gather(bf16_t *h, const bf16_t *table, const int32_t *tokens, int64_t n, int32_t d, hipStream_t s) {
    if (n <= 0 || d <= 0 || (d & 7)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(embed_gather_kernel, dim3(blocks_for(n * (d >> 3), 256)), dim3(256), 0, s, h, table, tokens, n,
                       d);
    return hipGetLastError();
}

hipError_t embed_scatter(float *dtable, const bf16_t *dh, const int32_t *row_start, const int32_t *order, int32_t V,
                         int32_t d, hipStream_t s) {
    if (V <= 0 || d <= 0 || (d & 7)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(embed_scatter_kernel, dim3((unsigned)V), dim3(256), 0, s, dtable, dh, row_start, order, d);
    return hipGetLastError();
}

hipError_t cross_entropy(float *loss_rows, bf16_t *dlogits, const float *logits, const int32_t *labels, int64_t n,
                         int32_t V, float inv_n, hipStream_t s) {
    if (n <= 0 || V <= 0 || (V & 3)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(cross_entropy_kernel, dim3((unsigned)n), dim3(256), 0, s, loss_rows, dlogits, logits, labels, V,
                       inv_n);
    return hipGetLastError();
}

hipError_t reduce_sum(float *out, const float *in, int64_t n, float scale, int accumulate, hipStream_t s) {
    if (n < 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(reduce_sum_kernel, dim3(1), dim3(1024), 0, s, out, in, n, scale, accumulate);
    return hipGetLastError();
}

hipError_t attn_delta(float *delta, const bf16_t *dout, int64_t lddo, const bf16_t *o, int64_t ldo, int32_t B,
                      int32_t T, int32_t H, int32_t hd, hipStream_t s) {
    if (hd != 64 && hd != 128) return hipErrorInvalidValue;
    const int64_t total = (int64_t)B * T * H * (hd >> 3);
    hipLaunchKernelGGL(attn_delta_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, delta, dout, lddo, o, ldo, B, T,
                       H, hd);
    return hipGetLastError();
}

hipError_t fill_u32(void *p, uint32_t value, size_t n_words, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    size_t blocks = (n_words + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint32_t *>(p), value,
                       n_words);
    return hipGetLastError();
}

}  // namespace mt
