// Bias + GELU, forward and backward: the elementwise step between the two matrix products of the
// encoder's MLP (Sec. 3, "Video Transformer": every layer holds a 2-layer MLP), the third entry of the
// paper's memory profile (Sec. 4.1).  The paper names no activation; this is the exact (erf) form of
// the plain ViT.  Per element, with h = x + bias_c:
//     y  = h Phi(h),                    Phi(h) = (1 + erf(h / sqrt 2)) / 2
//     dx = dy (Phi(h) + h phi(h)),      phi(h) = exp(-h^2 / 2) / sqrt(2 pi)
//     dbias_c = sum_rows dx_c           (summed from the unrounded fp32 dx)
// The backward rebuilds Phi and phi from x: the activation's output need not be kept for it.
//
// Bound by memory bandwidth (forward one read and one write of 2 bytes per element, backward two reads
// and one write).  A workgroup of 128 threads owns 1024 consecutive columns (thread = one 16-byte
// chunk, so its 8 bias values and its 8 partial sums of dbias live in registers for the whole kernel)
// and walks the rows of its row group with a stride, four rows in flight.  The partial sums of the row
// groups are added by avion_ln_param_reduce_kernel in a fixed order: no atomics, bit-reproducible.
//
// Tensors much larger than the chip's last-level cache (256 MB) are read and written with
// nontemporal accesses (STREAM): nothing of them will be found there again, and keeping them out of it
// is worth 4 % (forward) and 7 % (backward) on [50176, 3072]; smaller tensors take ordinary accesses,
// so that a consumer right after finds them cached.
//
// erf: 1 - erf(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1 / (1 + p z), z >= 0
// (Abramowitz and Stegun 7.1.26, absolute error < 1.5e-7, far below the rounding of the outputs);
// its exponential exp(-z^2) = exp(-h^2 / 2) is the one phi(h) needs, so each element costs one
// exponential and one reciprocal.
#pragma once
#include "avion_common.h"

constexpr int kGeluThreads = 128;     // threads per workgroup = 16-byte column chunks per workgroup
constexpr int kGeluRows = 4;          // rows in flight per thread
constexpr int kGeluMaxGrid = 4096;    // workgroups of a launch (column blocks x row groups)

template <bool STREAM>
DEVINL u32x4 gelu_load(const raw16* p)
{
    const u32x4* q = reinterpret_cast<const u32x4*>(p);
    return STREAM ? __builtin_nontemporal_load(q) : *q;
}
template <bool STREAM>
DEVINL void gelu_store(raw16* p, u32x4 v)
{
    u32x4* q = reinterpret_cast<u32x4*>(p);
    if (STREAM) __builtin_nontemporal_store(v, q);
    else *q = v;
}

// Phi(h) and h * phi(h)
DEVINL void gelu_terms(float h, float& cdf, float& hpdf)
{
    const float e = fast_exp2(h * h * (-0.5f * kLog2e));  // exp(-h^2 / 2)
    const float z = fabsf(h) * 0.70710678f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float tail = 0.5f * poly * t * e;  // (1 - erf(|h| / sqrt 2)) / 2
    cdf = h >= 0.f ? 1.0f - tail : tail;
    hpdf = h * e * 0.3989422804f;
}

// ncb = column blocks; gridDim.x = ncb * (row groups)
template <typename E, bool STREAM>
__global__ void __launch_bounds__(kGeluThreads)
avion_bias_gelu_fwd_kernel(const raw16* __restrict__ x, const float* __restrict__ bias, raw16* __restrict__ y, long M, int F,
                           int ncb)
{
    const int cb = blockIdx.x % ncb;
    const long rg = blockIdx.x / ncb, nrg = gridDim.x / ncb;
    const int col = (cb * kGeluThreads + threadIdx.x) * 8;
    if (col >= F) return;
    float b[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = bias[col + e];
    for (long r = rg; r < M; r += nrg * kGeluRows) {
        u32x4 in[kGeluRows];
#pragma unroll
        for (int k = 0; k < kGeluRows; ++k) {
            const long row = r + k * nrg;
            if (row < M) in[k] = gelu_load<STREAM>(x + row * F + col);
        }
#pragma unroll
        for (int k = 0; k < kGeluRows; ++k) {
            const long row = r + k * nrg;
            if (row < M) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float h = E::widen(as_frag8(in[k]), e) + b[e];
                    float cdf, hpdf;
                    gelu_terms(h, cdf, hpdf);
                    o[e] = h * cdf;
                }
                u32x4 w;
#pragma unroll
                for (int p = 0; p < 4; ++p) w[p] = E::pack(o[2 * p], o[2 * p + 1]);
                gelu_store<STREAM>(y + row * F + col, w);
            }
        }
    }
}

// dx, and this row group's partial sums of dbias into part[row group][F]
template <typename E, bool STREAM>
__global__ void __launch_bounds__(kGeluThreads)
avion_bias_gelu_bwd_kernel(const raw16* __restrict__ x, const float* __restrict__ bias, const raw16* __restrict__ dy,
                           raw16* __restrict__ dx, float* __restrict__ part, long M, int F, int ncb)
{
    const int cb = blockIdx.x % ncb;
    const long rg = blockIdx.x / ncb, nrg = gridDim.x / ncb;
    const int col = (cb * kGeluThreads + threadIdx.x) * 8;
    if (col >= F) return;
    float b[8], acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = bias[col + e];
        acc[e] = 0.f;
    }
    for (long r = rg; r < M; r += nrg * kGeluRows) {
        u32x4 in[kGeluRows], gin[kGeluRows];
#pragma unroll
        for (int k = 0; k < kGeluRows; ++k) {
            const long row = r + k * nrg;
            if (row < M) {
                in[k] = gelu_load<STREAM>(x + row * F + col);
                gin[k] = gelu_load<STREAM>(dy + row * F + col);
            }
        }
#pragma unroll
        for (int k = 0; k < kGeluRows; ++k) {
            const long row = r + k * nrg;
            if (row < M) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float h = E::widen(as_frag8(in[k]), e) + b[e];
                    float cdf, hpdf;
                    gelu_terms(h, cdf, hpdf);
                    o[e] = E::widen(as_frag8(gin[k]), e) * (cdf + hpdf);
                    acc[e] += o[e];
                }
                u32x4 w;
#pragma unroll
                for (int p = 0; p < 4; ++p) w[p] = E::pack(o[2 * p], o[2 * p + 1]);
                gelu_store<STREAM>(dx + row * F + col, w);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[rg * F + col + e] = acc[e];
}
