// Backward kernels.  P is rebuilt tile by tile from Q, K and the saved LSE, so no N x N matrix is
// read or written (Sec. 3, "Flash Attention": the weights stay implicit; Sec. 4.1: the attention
// activation memory disappears).  With s = scale*<q_i,k_j>, P = exp(s - LSE_i),
// delta_i = sum_c dO_ic O_ic:
//     dV = P^T dO ,  dP = dO V^T ,  dS = P o (dP - delta) ,  dQ = scale dS K ,  dK = scale dS^T Q.
//
// Two kernels, both free of atomics (results are bit-reproducible):
//   avion_dq_kernel   : query-stationary.  Also computes delta from O and dO and saves it for the
//                       second kernel.  Same shape as the forward: S^T = K Q^T and dP^T = V dO^T
//                       land with lane = query, so LSE and delta are per-lane scalars and dS^T
//                       feeds dQ^T = K^T dS^T as a B operand straight from registers; K^T comes
//                       from the same LDS tile as K, through transposing LDS loads.
//   avion_dkdv_kernel : key-stationary.  S = Q K^T and dP = dO V^T land with lane = key, K and V
//                       stay in registers as B operands, and P, dS feed dV^T = dO^T P and
//                       dK^T = Q^T dS from registers; the Q and dO tiles in LDS are read both as
//                       rows and, through transposing LDS loads, as columns.
// Each kernel recomputes S and dP for itself (7 contractions per tile pair instead of the
// algorithmic 5); the extra two are not counted as useful work anywhere.
#pragma once
#include "avion_common.h"

// --------------------------------------------------------------------------------------------- dQ
template <int D, int QT, int NW>
struct DqCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * QT * NW;
    using Stage = TileStage<D, BN, NT>;
    static constexpr int LDS_BYTES = 4 * Stage::BYTES;  // K0 K1 V0 V1
};

template <int D, int QT, int NW>
__global__ void __launch_bounds__(NW * 64)
avion_dq_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                const bf16* __restrict__ o, const bf16* __restrict__ dO, const float* __restrict__ lse,
                bf16* __restrict__ dq, float* __restrict__ delta, int H, int N, int nqb, int nblocks,
                float cs, float scale)
{
    using Cfg = DqCfg<D, QT, NW>;
    using Stage = typename Cfg::Stage;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Stage::STRIDE;
    constexpr int KS = D / 16;
    constexpr int CT = (D + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    auto kbuf = [&](int i) { return smem + i * Stage::BYTES; };
    auto vbuf = [&](int i) { return smem + (2 + i) * Stage::BYTES; };

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nqb, qb = logical % nqb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const SliceView kh(k + head_off, rs, N, D);
    const SliceView vh(v + head_off, rs, N, D);
    const int q0 = qb * BM + wave * 32 * QT;
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // Q and dO fragments (B operands), delta and LSE per lane
    bf16x8 qf[QT][KS], gf[QT][KS];
    float lc[QT], dl[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = min(q0 + 32 * qt + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[qt][ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
            gf[qt][ks] = *reinterpret_cast<const bf16x8*>(dO + off + ks * 16);
            const bf16x8 of = *reinterpret_cast<const bf16x8*>(o + off + ks * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf((float)of[e], (float)gf[qt][ks][e], part);
        }
        dl[qt] = both_halves_sum(part);
        lc[qt] = lse[(long)bh * N + row] * kLog2e;
        if (wave_active && g == 0 && q0 + 32 * qt + l32 < N) delta[(long)bh * N + row] = dl[qt];
    }

    f32x16 acc[CT][QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[ct][qt] = f32x16_zero();

    Stage kst, vst;
    if constexpr (D % 32 != 0) {
        Stage::zero_pad(kbuf(0), tid);
        Stage::zero_pad(kbuf(1), tid);
    }
    kst.load(kh, 0, tid);
    vst.load(vh, 0, tid);
    kst.store(kbuf(0), tid);
    vst.store(vbuf(0), tid);
    __syncthreads();

    const int ntiles = (N + BN - 1) / BN;
    for (int t = 0; t < ntiles; ++t) {
        const char* kc = kbuf(t & 1);
        const char* vc = vbuf(t & 1);
        const bool more = t + 1 < ntiles;
        if (more) {
            kst.load(kh, (t + 1) * BN, tid);
            vst.load(vh, (t + 1) * BN, tid);
        }
        if (wave_active) {
            const bool ragged = (t + 1) * BN > N;
#pragma unroll
            for (int kt = 0; kt < BN / 32; ++kt) {
                f32x16 s[QT], dp[QT];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 ak = nat_frag(kc, STRIDE, 32 * kt + l32, ks, g);
                    const bf16x8 av = nat_frag(vc, STRIDE, 32 * kt + l32, ks, g);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) {
                        s[qt] = mfma32(ak, qf[qt][ks], ks == 0 ? f32x16_zero() : s[qt]);
                        dp[qt] = mfma32(av, gf[qt][ks], ks == 0 ? f32x16_zero() : dp[qt]);
                    }
                }
                bf16x8 df[QT][2];
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const float nl = -lc[qt];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = fast_exp2(fmaf(s[qt][i], cs, nl));
                        s[qt][i] = p * (dp[qt][i] - dl[qt]);
                    }
                    // keys beyond N were staged as zero rows; force their dS to zero as well so
                    // that an overflowing weight cannot turn 0 * inf into NaN
                    if (ragged) {
                        const int key0 = t * BN + 32 * kt + 4 * g;
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (key0 + 8 * (i / 4) + (i % 4) >= N) s[qt][i] = 0.f;
                    }
                    df[qt][0] = acc_to_frag(s[qt], 0);
                    df[qt][1] = acc_to_frag(s[qt], 1);
                }
                // dQ^T += K^T dS^T
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 a = tr_frag(kc, STRIDE, tr_off, ct, 2 * kt + half);
#pragma unroll
                        for (int qt = 0; qt < QT; ++qt) acc[ct][qt] = mfma32(a, df[qt][half], acc[ct][qt]);
                    }
            }
        }
        if (more) {
            kst.store(kbuf((t + 1) & 1), tid);
            vst.store(vbuf((t + 1) & 1), tid);
        }
        __syncthreads();
    }

    if (!wave_active) return;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = q0 + 32 * qt + l32;
        if (row < N) {
            bf16* drow = dq + head_off + (long)row * rs;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const int c0 = 32 * ct + 8 * a4 + 4 * g;
                    if (c0 < D)
                        store_bf16x4(drow + c0, acc[ct][qt][4 * a4 + 0] * scale, acc[ct][qt][4 * a4 + 1] * scale,
                                     acc[ct][qt][4 * a4 + 2] * scale, acc[ct][qt][4 * a4 + 3] * scale);
                }
        }
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
template <int D, int KT, int NW, int BQ_ = 32>
struct DkvCfg {
    static constexpr int BQ = BQ_;  // queries per LDS tile
    static constexpr int NT = NW * 64;
    static constexpr int BNK = 32 * KT * NW;  // keys per workgroup
    using Stage = TileStage<D, BQ, NT>;
    static constexpr int ROWV_BYTES = 2 * BQ * 4;  // LSE*log2e and delta of the tile's queries
    static constexpr int BUF_BYTES = 2 * Stage::BYTES + ROWV_BYTES;
    static constexpr int LDS_BYTES = 2 * BUF_BYTES;
};

template <int D, int KT, int NW, int BQ_>
__global__ void __launch_bounds__(NW * 64)
avion_dkdv_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                  const bf16* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ delta,
                  bf16* __restrict__ dk, bf16* __restrict__ dv, int H, int N, int nkb, int nblocks,
                  float cs, float scale)
{
    using Cfg = DkvCfg<D, KT, NW, BQ_>;
    using Stage = typename Cfg::Stage;
    constexpr int BQ = Cfg::BQ, BNK = Cfg::BNK, STRIDE = Stage::STRIDE;
    constexpr int KS = D / 16;
    constexpr int CT = (D + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // per buffer: Q tile | dO tile | lc[BQ] | dl[BQ]
    constexpr int OFF_G = Stage::BYTES, OFF_ROW = 2 * Stage::BYTES;

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nkb, kb = logical % nkb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const SliceView qh(q + head_off, rs, N, D);
    const SliceView gh(dO + head_off, rs, N, D);
    const float* lrow = lse + (long)bh * N;
    const float* drow = delta + (long)bh * N;
    const int k0 = kb * BNK + wave * 32 * KT;  // first key of this wavefront
    const bool wave_active = k0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // K and V fragments (B operands: lane = key) stay in registers
    bf16x8 kf[KT][KS], vf[KT][KS];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
        const int row = min(k0 + 32 * kt + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[kt][ks] = *reinterpret_cast<const bf16x8*>(k + off + ks * 16);
            vf[kt][ks] = *reinterpret_cast<const bf16x8*>(v + off + ks * 16);
        }
    }

    f32x16 dka[CT][KT], dva[CT][KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            dka[ct][kt] = f32x16_zero();
            dva[ct][kt] = f32x16_zero();
        }

    Stage qst, gst;
    float lc_r = 0.f, dl_r = 0.f;
    auto load_tile = [&](int r0) {
        qst.load(qh, r0, tid);
        gst.load(gh, r0, tid);
        if (tid < BQ) {
            const int tok = r0 + tid;
            // queries beyond N get weight exp2(-inf) = 0, hence dS = 0 as well
            lc_r = tok < N ? lrow[tok] * kLog2e : INFINITY;
            dl_r = tok < N ? drow[tok] : 0.f;
        }
    };
    auto store_tile = [&](char* buf) {
        qst.store(buf, tid);
        gst.store(buf + OFF_G, tid);
        if (tid < BQ) {
            reinterpret_cast<float*>(buf + OFF_ROW)[tid] = lc_r;
            reinterpret_cast<float*>(buf + OFF_ROW)[BQ + tid] = dl_r;
        }
    };
    if constexpr (D % 32 != 0) {
        for (int i = 0; i < 2; ++i) {
            Stage::zero_pad(smem + i * Cfg::BUF_BYTES, tid);
            Stage::zero_pad(smem + i * Cfg::BUF_BYTES + OFF_G, tid);
        }
    }
    load_tile(0);
    store_tile(smem);
    __syncthreads();

    const int ntiles = (N + BQ - 1) / BQ;
    for (int t = 0; t < ntiles; ++t) {
        const char* buf = smem + (t & 1) * Cfg::BUF_BYTES;
        const bool more = t + 1 < ntiles;
        if (more) load_tile((t + 1) * BQ);
        if (wave_active) {
#pragma unroll
            for (int qt = 0; qt < BQ / 32; ++qt) {
                // S and dP tiles: rows = 32 queries, cols = 32 keys
                f32x16 s[KT], dp[KT];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 aq = nat_frag(buf, STRIDE, 32 * qt + l32, ks, g);
                    const bf16x8 ag = nat_frag(buf + OFF_G, STRIDE, 32 * qt + l32, ks, g);
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt) {
                        s[kt] = mfma32(aq, kf[kt][ks], ks == 0 ? f32x16_zero() : s[kt]);
                        dp[kt] = mfma32(ag, vf[kt][ks], ks == 0 ? f32x16_zero() : dp[kt]);
                    }
                }
                // per accumulator row (query): LSE*log2e and delta, broadcast reads from LDS
                const float* rowv = reinterpret_cast<const float*>(buf + OFF_ROW) + 32 * qt + 4 * g;
                bf16x8 pf[KT][2], df[KT][2];
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const f32x4 l4 = *reinterpret_cast<const f32x4*>(rowv + 8 * a4);
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(rowv + BQ + 8 * a4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = 4 * a4 + e;
#pragma unroll
                        for (int kt = 0; kt < KT; ++kt) {
                            const float p = fast_exp2(fmaf(s[kt][i], cs, -l4[e]));
                            s[kt][i] = p;
                            dp[kt][i] = p * (dp[kt][i] - d4[e]);
                        }
                    }
                }
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        pf[kt][half] = acc_to_frag(s[kt], half);
                        df[kt][half] = acc_to_frag(dp[kt], half);
                    }
                // dV^T += dO^T P ,  dK^T += Q^T dS   (contraction over the 32 queries, 2 steps)
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 ag = tr_frag(buf + OFF_G, STRIDE, tr_off, ct, 2 * qt + half);
                        const bf16x8 aq = tr_frag(buf, STRIDE, tr_off, ct, 2 * qt + half);
#pragma unroll
                        for (int kt = 0; kt < KT; ++kt) {
                            dva[ct][kt] = mfma32(ag, pf[kt][half], dva[ct][kt]);
                            dka[ct][kt] = mfma32(aq, df[kt][half], dka[ct][kt]);
                        }
                    }
            }
        }
        if (more) store_tile(smem + ((t + 1) & 1) * Cfg::BUF_BYTES);
        __syncthreads();
    }

    if (!wave_active) return;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
        const int row = k0 + 32 * kt + l32;
        if (row < N) {
            bf16* dkrow = dk + head_off + (long)row * rs;
            bf16* dvrow = dv + head_off + (long)row * rs;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const int c0 = 32 * ct + 8 * a4 + 4 * g;
                    if (c0 < D) {
                        store_bf16x4(dkrow + c0, dka[ct][kt][4 * a4 + 0] * scale, dka[ct][kt][4 * a4 + 1] * scale,
                                     dka[ct][kt][4 * a4 + 2] * scale, dka[ct][kt][4 * a4 + 3] * scale);
                        store_bf16x4(dvrow + c0, dva[ct][kt][4 * a4 + 0], dva[ct][kt][4 * a4 + 1],
                                     dva[ct][kt][4 * a4 + 2], dva[ct][kt][4 * a4 + 3]);
                    }
                }
        }
    }
}
