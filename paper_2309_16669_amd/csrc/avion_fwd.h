// Forward kernel: O = softmax(scale * Q K^T) V and LSE, one pass over the keys, nothing N x N stored
// (Sec. 3, "Flash Attention": implicit softmax weights, block-wise work out of on-chip memory;
// Sec. 1: block results combined into the exact output).
//
// Work split: one workgroup = NW wavefronts = 32*QT*NW consecutive queries of one (batch, head).
// Each wavefront owns 32*QT queries and keeps, per query tile of 32:
//   Q as MFMA B-operand fragments (lane = query, 8 channels per 16-deep step),
//   O^T accumulators (lane = query, registers = channels), the running maximum and row sums.
// Keys and values come in tiles of BN = 64 tokens through triple-buffered LDS in their natural row
// layout: K rows are the A operand of S^T = K Q^T, and V is read through transposing LDS loads as
// the A operand of O^T = V^T P^T.
// Computing the transposed products keeps every score of a query inside one lane pair, so the
// accumulator of the first contraction is, after rounding to bf16, directly the B operand of the
// second one (no LDS round trip), and the row maximum needs a single exchange between the two
// halves of the wavefront.
//
// Software pipeline: while the softmax arithmetic of tile t runs on the vector ALUs, the matrix
// cores already work on S^T of tile t+1 (issued first, into a second set of accumulators) and then
// on the P V product of tile t.  Tile t+2 is in flight from global memory meanwhile and is written
// to the third LDS buffer at the end of the step; one workgroup barrier per tile.
#pragma once
#include "avion_common.h"

// The stored maximum is only raised when the true maximum exceeds it by more than this many
// binades; until then the weights are exp2 of at most kLazyBinades, well inside fp32/bf16 range,
// and the final division by the row sum cancels the stale factor exactly.
constexpr float kLazyBinades = 8.0f;

template <int D, int QT, int NW>
struct FwdCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * QT * NW;
    using Stage = TileStage<D, BN, NT>;
    static constexpr int LDS_BYTES = 6 * Stage::BYTES;  // K0 K1 K2 V0 V1 V2
};

template <int D, int QT, int NW>
__global__ void __launch_bounds__(NW * 64)
avion_fwd_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                 bf16* __restrict__ o, float* __restrict__ lse, int H, int N, int nqb, int nblocks, float cs)
{
    using Cfg = FwdCfg<D, QT, NW>;
    using Stage = typename Cfg::Stage;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Stage::STRIDE;
    constexpr int KS = D / 16;         // 16-deep steps over the channels
    constexpr int CT = (D + 31) / 32;  // 32-channel tiles of O^T
    constexpr int KT = BN / 32;        // 32-key sub-tiles of an LDS tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    auto kbuf = [&](int i) { return smem + i * Stage::BYTES; };
    auto vbuf = [&](int i) { return smem + (3 + i) * Stage::BYTES; };

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nqb, qb = logical % nqb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const bf16* qh = q + head_off;
    const SliceView kh(k + head_off, rs, N, D);
    const SliceView vh(v + head_off, rs, N, D);
    bf16* oh = o + head_off;
    const int q0 = qb * BM + wave * 32 * QT;  // first query of this wavefront
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // Q fragments stay in registers for the whole kernel
    bf16x8 qf[QT][KS];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = min(q0 + 32 * qt + l32, N - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[qt][ks] = *reinterpret_cast<const bf16x8*>(qh + (long)row * rs + ks * 16 + g * 8);
    }

    f32x16 oacc[CT][QT];
    float m_used[QT], lsum[QT], rsum[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_used[qt] = -INFINITY;
        lsum[qt] = 0.f;
        rsum[qt] = 0.f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) oacc[ct][qt] = f32x16_zero();
    }

    const int ntiles = (N + BN - 1) / BN;
    Stage kst, vst;
    if constexpr (D % 32 != 0) {
        for (int i = 0; i < 3; ++i) Stage::zero_pad(vbuf(i), tid);
    }
    kst.load(kh, 0, tid);
    vst.load(vh, 0, tid);
    kst.store(kbuf(0), tid);
    vst.store(vbuf(0), tid);
    if (ntiles > 1) {
        kst.load(kh, BN, tid);
        vst.load(vh, BN, tid);
        kst.store(kbuf(1), tid);
        vst.store(vbuf(1), tid);
    }
    __syncthreads();

    // S^T of one LDS tile: [sub-tile of 32 keys][query tile], rows = keys, cols = queries
    auto scores = [&](const char* kc, f32x16 (&s)[KT][QT]) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = nat_frag(kc, STRIDE, 32 * kt + l32, ks, g);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    s[kt][qt] = mfma32(a, qf[qt][ks], ks == 0 ? f32x16_zero() : s[kt][qt]);
            }
    };

    // one pipeline step on tile t: `cur` holds S^T of tile t, `nxt` receives S^T of tile t+1
    auto step = [&](int t, f32x16 (&cur)[KT][QT], f32x16 (&nxt)[KT][QT]) {
        const bool have1 = t + 1 < ntiles, have2 = t + 2 < ntiles;
        if (have2) {
            kst.load(kh, (t + 2) * BN, tid);
            vst.load(vh, (t + 2) * BN, tid);
        }
        if (wave_active) {
            if (have1) scores(kbuf((t + 1) % 3), nxt);
            const char* vc = vbuf(t % 3);
            if ((t + 1) * BN > N) {  // ragged last tile: keys at or beyond N get weight 0
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    const int key0 = t * BN + 32 * kt + 4 * g;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (key0 + 8 * (i / 4) + (i % 4) >= N) {
#pragma unroll
                            for (int qt = 0; qt < QT; ++qt) cur[kt][qt][i] = -INFINITY;
                        }
                }
            }
            // online softmax in base 2: weights are exp2(cs*s - m_used)
            bf16x8 pf[KT][QT][2];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                float mx = max16(cur[0][qt]);
#pragma unroll
                for (int kt = 1; kt < KT; ++kt) mx = max3(mx, max16(cur[kt][qt]), mx);
                const float m2 = both_halves_max(mx) * cs;
                if (__builtin_amdgcn_ballot_w64(m2 > m_used[qt] + kLazyBinades) != 0ull) {
                    const float mn = fmaxf(m_used[qt], m2);
                    const float alpha = fast_exp2(m_used[qt] - mn);
                    m_used[qt] = mn;
                    lsum[qt] *= alpha;
                    rsum[qt] *= alpha;
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[ct][qt][i] *= alpha;
                }
                const float nm = -m_used[qt];
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    float rowsum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = fast_exp2(fmaf(cur[kt][qt][i], cs, nm));
                        cur[kt][qt][i] = p;
                        rowsum += p;
                    }
                    lsum[qt] += rowsum;
                    pf[kt][qt][0] = acc_to_frag(cur[kt][qt], 0);
                    pf[kt][qt][1] = acc_to_frag(cur[kt][qt], 1);
                    // Second row sum, over the weights as rounded to bf16, i.e. exactly the numbers
                    // the second contraction multiplies V with.  O is divided by this one, which
                    // makes it a true convex combination of value rows (the rounding of a dominant
                    // weight cancels); LSE uses the unrounded sum.
                    rsum[qt] = frag_sum(pf[kt][qt][1], frag_sum(pf[kt][qt][0], rsum[qt]));
                }
            }
            // O^T += V^T P^T
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 a = tr_frag(vc, STRIDE, tr_off, ct, 2 * kt + half);
#pragma unroll
                        for (int qt = 0; qt < QT; ++qt) oacc[ct][qt] = mfma32(a, pf[kt][qt][half], oacc[ct][qt]);
                    }
        }
        if (have2) {
            kst.store(kbuf((t + 2) % 3), tid);
            vst.store(vbuf((t + 2) % 3), tid);
        }
        __syncthreads();
    };

    f32x16 sa[KT][QT], sb[KT][QT];
    if (wave_active) scores(kbuf(0), sa);
    wait_all_loads();
    for (int t = 0; t < ntiles; t += 2) {
        step(t, sa, sb);
        if (t + 1 < ntiles) step(t + 1, sb, sa);
    }

    if (!wave_active) return;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float l = both_halves_sum(lsum[qt]);
        const float inv = 1.0f / both_halves_sum(rsum[qt]);
        const int row = q0 + 32 * qt + l32;
        if (row < N) {
            bf16* orow = oh + (long)row * rs;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const int c0 = 32 * ct + 8 * a4 + 4 * g;
                    if (c0 < D)
                        store_bf16x4(orow + c0, oacc[ct][qt][4 * a4 + 0] * inv, oacc[ct][qt][4 * a4 + 1] * inv,
                                     oacc[ct][qt][4 * a4 + 2] * inv, oacc[ct][qt][4 * a4 + 3] * inv);
                }
            if (g == 0) lse[(long)bh * N + row] = (m_used[qt] + __builtin_amdgcn_logf(l)) * kLn2;
        }
    }
}
