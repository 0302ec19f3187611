// Layer normalisation over the channel axis, forward and backward: the per-token normalisation in front
// of the attention and of the MLP of every encoder layer (Sec. 3, "Video Transformer"), one of the
// three entries of the paper's memory profile (Sec. 4.1).  Per token row x in R^D:
//     mu = mean(x), var = mean((x - mu)^2), rstd = 1/sqrt(var + eps), xhat = (x - mu) rstd,
//     y = xhat gamma + beta
//     dbeta = sum_rows dy, dgamma = sum_rows dy xhat, g = dy gamma,
//     dx = rstd (g - mean(g) - xhat mean(g xhat))
// What the backward needs from the forward is x itself and two fp32 per row (mu, rstd).
//
// Bound by memory bandwidth (forward: one read and one write of 2 bytes per element; backward: two
// reads and one write), so the kernels are organised around keeping loads in flight:
// one wavefront owns a row at a time (lane j holds the 16-byte chunks j, j+64, ... of the row, all of
// it in registers, so the mean and the variance about it are taken in two passes over registers, not
// over memory), walks the rows with a stride, and requests the next row before it works on the
// current one.  Statistics and all sums are fp32; outputs are rounded once (nearest even).
// The parameter gradients are summed over each wavefront's rows in registers, over the workgroup's
// wavefronts through LDS, and over the workgroups by a second small kernel in a fixed order -- no
// atomics, so results are bit-reproducible.
#pragma once
#include "avion_common.h"

constexpr int kLnWaves = 4;          // wavefronts per workgroup
constexpr int kLnMaxChunks = 4;      // 16-byte chunks per lane: D <= 64 * 4 * 8 = 2048 (ViT-B/L/H: 768, 1024, 1280)
constexpr int kLnMaxGrid = 1024;     // workgroups of a launch; also the number of partial sums of dgamma, dbeta

DEVINL float wave_sum(float x)
{
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) x += __shfl_xor(x, off, 64);
    return both_halves_sum(x);
}

// one row's share of a lane: NCH chunks of 8 elements
template <int NCH>
struct LnRow {
    u32x4 c[NCH];
    DEVINL void load(const raw16* row, int nchunks, int lane)
    {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = lane + 64 * j;
            c[j] = ch < nchunks ? *reinterpret_cast<const u32x4*>(row + ch * 8) : zero;
        }
    }
    template <typename E>
    DEVINL float get(int j, int e) const
    {
        return E::widen(as_frag8(c[j]), e);
    }
};

template <int NCH, typename E>
__global__ void __launch_bounds__(kLnWaves * 64)
avion_ln_fwd_kernel(const raw16* __restrict__ x, const float* __restrict__ gamma, const float* __restrict__ beta,
                    raw16* __restrict__ y, float* __restrict__ mean, float* __restrict__ rstd, long M, int D, float eps)
{
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int nchunks = D / 8;
    const float inv_d = 1.0f / (float)D;
    const long stride = (long)gridDim.x * kLnWaves;
    long row = (long)blockIdx.x * kLnWaves + wave;
    if (row >= M) return;
    float gam[NCH][8], bet[NCH][8];
#pragma unroll
    for (int j = 0; j < NCH; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int ch = lane + 64 * j;
            gam[j][e] = ch < nchunks ? gamma[ch * 8 + e] : 0.f;
            bet[j][e] = ch < nchunks ? beta[ch * 8 + e] : 0.f;
        }

    auto finish = [&](const LnRow<NCH>& r, long at) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += r.template get<E>(j, e);  // chunks past the row are zeros
        const float mu = wave_sum(s) * inv_d;
        float v = 0.f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
            if (lane + 64 * j < nchunks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = r.template get<E>(j, e) - mu;
                    v = fmaf(d, d, v);
                }
        const float rs = __builtin_amdgcn_rsqf(wave_sum(v) * inv_d + eps);
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = lane + 64 * j;
            if (ch < nchunks) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf((r.template get<E>(j, e) - mu) * rs, gam[j][e], bet[j][e]);
                u32x4 w;
#pragma unroll
                for (int p = 0; p < 4; ++p) w[p] = E::pack(o[2 * p], o[2 * p + 1]);
                *reinterpret_cast<u32x4*>(y + at * D + ch * 8) = w;
            }
        }
        if (lane == 0) {
            mean[at] = mu;
            rstd[at] = rs;
        }
    };

    // two rows in registers: the next one is in flight while the current one is worked on
    LnRow<NCH> a, b;
    a.load(x + row * D, nchunks, lane);
    while (true) {
        const long n1 = row + stride;
        if (n1 < M) b.load(x + n1 * D, nchunks, lane);
        finish(a, row);
        if (n1 >= M) break;
        const long n2 = n1 + stride;
        if (n2 < M) a.load(x + n2 * D, nchunks, lane);
        finish(b, n1);
        if (n2 >= M) break;
        row = n2;
    }
}

// dx, and this workgroup's partial sums of dgamma and dbeta into part[blockIdx.x][2][D]
template <int NCH, typename E>
__global__ void __launch_bounds__(kLnWaves * 64)
avion_ln_bwd_kernel(const raw16* __restrict__ x, const float* __restrict__ gamma, const float* __restrict__ mean,
                    const float* __restrict__ rstd, const raw16* __restrict__ dy, raw16* __restrict__ dx,
                    float* __restrict__ part, long M, int D)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];  // (kLnWaves - 1) x 2 x D floats
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int nchunks = D / 8;
    const float inv_d = 1.0f / (float)D;
    const long stride = (long)gridDim.x * kLnWaves;

    float gam[NCH][8], dg[NCH][8], db[NCH][8];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int ch = lane + 64 * j;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            gam[j][e] = ch < nchunks ? gamma[ch * 8 + e] : 0.f;
            dg[j][e] = 0.f;
            db[j][e] = 0.f;
        }
    }

    auto finish = [&](const LnRow<NCH>& rx, const LnRow<NCH>& ry, long at) {
        const float mu = mean[at], rs = rstd[at];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xh = (rx.template get<E>(j, e) - mu) * rs, gy = ry.template get<E>(j, e);
                const float g = gy * gam[j][e];                 // zero in chunks past the row
                s1 += g;
                s2 = fmaf(g, xh, s2);
                dg[j][e] = fmaf(gy, xh, dg[j][e]);
                db[j][e] += gy;
            }
        const float c1 = wave_sum(s1) * inv_d, c2 = wave_sum(s2) * inv_d;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = lane + 64 * j;
            if (ch < nchunks) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float xh = (rx.template get<E>(j, e) - mu) * rs;
                    o[e] = rs * (ry.template get<E>(j, e) * gam[j][e] - c1 - xh * c2);
                }
                u32x4 w;
#pragma unroll
                for (int p = 0; p < 4; ++p) w[p] = E::pack(o[2 * p], o[2 * p + 1]);
                *reinterpret_cast<u32x4*>(dx + at * D + ch * 8) = w;
            }
        }
    };

    long row = (long)blockIdx.x * kLnWaves + wave;
    if (row < M) {
        LnRow<NCH> ax, ay, bx, by;
        ax.load(x + row * D, nchunks, lane);
        ay.load(dy + row * D, nchunks, lane);
        while (true) {
            const long n1 = row + stride;
            if (n1 < M) {
                bx.load(x + n1 * D, nchunks, lane);
                by.load(dy + n1 * D, nchunks, lane);
            }
            finish(ax, ay, row);
            if (n1 >= M) break;
            const long n2 = n1 + stride;
            if (n2 < M) {
                ax.load(x + n2 * D, nchunks, lane);
                ay.load(dy + n2 * D, nchunks, lane);
            }
            finish(bx, by, n1);
            if (n2 >= M) break;
            row = n2;
        }
    }
    // workgroup sum in wavefront order (0 + 1 + 2 + 3), then one partial per workgroup
    float* sh = reinterpret_cast<float*>(smem);
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = lane + 64 * j;
            if (ch < nchunks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    sh[((wave - 1) * 2 + 0) * D + ch * 8 + e] = dg[j][e];
                    sh[((wave - 1) * 2 + 1) * D + ch * 8 + e] = db[j][e];
                }
        }
    }
    __syncthreads();
    if (wave == 0) {
        float* out = part + (long)blockIdx.x * 2 * D;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = lane + 64 * j;
            if (ch < nchunks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float a = dg[j][e], b = db[j][e];
                    for (int w = 0; w < kLnWaves - 1; ++w) {
                        a += sh[(w * 2 + 0) * D + ch * 8 + e];
                        b += sh[(w * 2 + 1) * D + ch * 8 + e];
                    }
                    out[ch * 8 + e] = a;
                    out[D + ch * 8 + e] = b;
                }
        }
    }
}

// dgamma, dbeta = sum over the workgroups' partials in a fixed order: a workgroup takes 64 of the 2*D
// columns, 16 threads per column each sum every 16th partial (independent loads, many in flight), and
// the 16 sums are added in order.
constexpr int kLnReduceCols = 64, kLnReduceGroups = 16;
__global__ void __launch_bounds__(kLnReduceCols * kLnReduceGroups)
avion_ln_param_reduce_kernel(const float* __restrict__ part, float* __restrict__ dgamma, float* __restrict__ dbeta,
                             int nparts, int D)
{
    __shared__ float sh[kLnReduceGroups][kLnReduceCols];
    const int col = threadIdx.x % kLnReduceCols, grp = threadIdx.x / kLnReduceCols;
    const int c = blockIdx.x * kLnReduceCols + col;
    float s = 0.f;
    if (c < 2 * D) {
        int p = grp;
        for (; p + 3 * kLnReduceGroups < nparts; p += 4 * kLnReduceGroups) {
            const float a0 = part[(long)p * 2 * D + c], a1 = part[(long)(p + kLnReduceGroups) * 2 * D + c],
                        a2 = part[(long)(p + 2 * kLnReduceGroups) * 2 * D + c], a3 = part[(long)(p + 3 * kLnReduceGroups) * 2 * D + c];
            s += a0;
            s += a1;
            s += a2;
            s += a3;
        }
        for (; p < nparts; p += kLnReduceGroups) s += part[(long)p * 2 * D + c];
    }
    sh[grp][col] = s;
    __syncthreads();
    if (grp == 0 && c < 2 * D) {
        float t = sh[0][col];
        for (int g = 1; g < kLnReduceGroups; ++g) t += sh[g][col];
        if (c < D) dgamma[c] = t;
        else dbeta[c - D] = t;
    }
}
