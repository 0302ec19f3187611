// Forward kernel: O = softmax(scale * Q K^T) V and LSE, one pass over the keys, nothing N x N stored
// (Sec. 3, "Flash Attention": implicit softmax weights, block-wise work out of on-chip memory;
// Sec. 1: block results combined into the exact output).
//
// Work split: one workgroup = NW wavefronts = 32*QT*NW consecutive queries of one (batch, head).
// Each wavefront owns 32*QT queries and keeps, per query tile of 32:
//   Q as MFMA B-operand fragments (lane = query, 8 channels per 16-deep step),
//   O^T accumulators (lane = query, registers = channels), the reference maximum and row sums.
// Keys and values come in LDS tiles of 64 tokens in their natural row layout, four buffers deep,
// filled straight from global memory by LDS-direct loads (no staging registers, no LDS writes):
// K rows are the A operand of S^T = K Q^T, and V is read through transposing LDS loads as the A
// operand of O^T = V^T P^T.  Computing the transposed products keeps every score of a query inside
// one lane pair, so the accumulator of the first contraction is, after rounding to bf16, directly
// the B operand of the second one (no LDS round trip).
//
// Schedule.  A wavefront issues in order and an MFMA queued behind another blocks what follows, so
// the three independent strands of a unit (32 keys x 32*QT queries) are interleaved instruction by
// instruction in program order:
//   matrix cores : S^T of the NEXT unit (second accumulator set) and the P V update of the PREVIOUS
//                  unit (from its saved bf16 weights);
//   vector ALUs  : exp2, row sums and bf16 rounding of the CURRENT unit;
//   LDS          : operand fragments a few MFMAs ahead of their use.
//
// Softmax reference.  Weights are exp2(cs*s - m) with m fixed per query to the maximum over the
// first 32 keys.  Softmax is invariant to m, fp32/bf16 keep their relative precision at any
// magnitude, and the final division by the row sum cancels m exactly; the only failure mode is
// overflow when a later score exceeds m by ~100 binades.  That is detected from the final row sum
// (workgroup-wide), and the whole workgroup then recomputes its rows with the classic running
// maximum (avion_fwd_safe_pass).  Random or trained activations never get there.
#pragma once
#include "avion_common.h"

template <int D, int QT, int NW>
struct FwdCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * QT * NW;
    static constexpr int NBUF = 4;
    using Stage = TileStage<D, BN, NT>;
    static constexpr int LDS_BYTES = 2 * NBUF * Stage::BYTES;  // K0..K3 V0..V3
    // wavefronts per SIMD the register budget is sized for: as many as LDS lets a compute unit hold
    static constexpr int WAVES_PER_SIMD = (160 * 1024 / LDS_BYTES) * NW / 4;
};

// row sums above this (or not finite) send the workgroup to the safe pass
constexpr float kRowSumLimit = 7.9e28f;  // 2^96

// Classic online softmax with a running maximum, one 64-key tile at a time, two LDS buffers.
// Used only as the fallback described above; same register layouts as the main loop.
template <int D, int QT, int NW>
DEVINL void avion_fwd_safe_pass(char* smem, const SliceView& kh, const SliceView& vh, const bf16x8 (&qf)[QT][D / 16],
                                f32x16 (&oacc)[(D + 31) / 32][QT], float (&m_used)[QT], float (&lsum)[QT],
                                float (&rsum)[QT], int N, float cs, bool wave_active, int tid, int l32, int g,
                                int tr_off, int v_off)
{
    using Stage = typename FwdCfg<D, QT, NW>::Stage;
    constexpr int BN = 64, STRIDE = Stage::STRIDE, KS = D / 16, CT = (D + 31) / 32;
    auto kbuf = [&](int i) { return smem + i * Stage::BYTES; };
    auto vbuf = [&](int i) { return smem + v_off + i * Stage::BYTES; };  // two K and two V buffers are used
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_used[qt] = -INFINITY;
        lsum[qt] = 0.f;
        rsum[qt] = 0.f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) oacc[ct][qt] = f32x16_zero();
    }
    Stage kst, vst;
    wait_all_loads();  // tiles the main loop requested past the end must have landed
    __syncthreads();
    if constexpr (D % 32 != 0) {
        Stage::zero_pad(vbuf(0), tid);
        Stage::zero_pad(vbuf(1), tid);
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
#pragma unroll
            for (int kt = 0; kt < BN / 32; ++kt) {
                f32x16 s[QT];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = nat_frag(kc, STRIDE, 32 * kt + l32, ks, g);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) s[qt] = mfma32(a, qf[qt][ks], ks == 0 ? f32x16_zero() : s[qt]);
                }
                const int key0 = t * BN + 32 * kt + 4 * g;
                if (key0 + 28 >= N) {
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (key0 + 8 * (i / 4) + (i % 4) >= N) {
#pragma unroll
                            for (int qt = 0; qt < QT; ++qt) s[qt][i] = -INFINITY;
                        }
                }
                bf16x8 pf[QT][2];
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const float m2 = both_halves_max(max16(s[qt])) * cs;
                    const float mn = fmaxf(m_used[qt], m2);  // finite: key 0 exists for every query
                    const float alpha = fast_exp2(m_used[qt] - mn);
                    m_used[qt] = mn;
                    lsum[qt] *= alpha;
                    rsum[qt] *= alpha;
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[ct][qt][i] *= alpha;
                    float rowsum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = fast_exp2(fmaf(s[qt][i], cs, -mn));
                        s[qt][i] = p;
                        rowsum += p;
                    }
                    lsum[qt] += rowsum;
                    pf[qt][0] = acc_to_frag(s[qt], 0);
                    pf[qt][1] = acc_to_frag(s[qt], 1);
                    rsum[qt] = frag_sum(pf[qt][1], frag_sum(pf[qt][0], rsum[qt]));
                }
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 a = tr_frag(vc, STRIDE, tr_off, ct, 2 * kt + half);
#pragma unroll
                        for (int qt = 0; qt < QT; ++qt) oacc[ct][qt] = mfma32(a, pf[qt][half], oacc[ct][qt]);
                    }
            }
        }
        if (more) {
            kst.store(kbuf((t + 1) & 1), tid);
            vst.store(vbuf((t + 1) & 1), tid);
        }
        __syncthreads();
    }
}

template <int D, int QT, int NW>
__global__ void __launch_bounds__(NW * 64, (FwdCfg<D, QT, NW>::WAVES_PER_SIMD))
avion_fwd_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                 bf16* __restrict__ o, float* __restrict__ lse, int H, int N, int nqb, int nblocks, float cs)
{
    using Cfg = FwdCfg<D, QT, NW>;
    using Stage = typename Cfg::Stage;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Stage::STRIDE;
    constexpr int KS = D / 16;         // 16-deep steps over the channels
    constexpr int CT = (D + 31) / 32;  // 32-channel tiles of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    auto kbuf = [&](int ti) { return smem + (ti & 3) * Stage::BYTES; };
    auto vbuf = [&](int ti) { return smem + (4 + (ti & 3)) * Stage::BYTES; };

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nqb, qb = logical % nqb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
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
        m_used[qt] = 0.f;
        lsum[qt] = 0.f;
        rsum[qt] = 0.f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) oacc[ct][qt] = f32x16_zero();
    }

    // K/V tile pairs stream through a ring of four LDS buffers each
    using Ring = PairRing<D, NW>;
    static_assert(Ring::TILE_BYTES == Stage::BYTES && Ring::LDS_BYTES == Cfg::LDS_BYTES, "ring and staging layouts agree");
    constexpr int NPW = Ring::NPW;
    const int ntiles = (N + BN - 1) / BN;
    const Ring ring(k + head_off, v + head_off, kh.bytes, kh.row_bytes, smem, wave, lane);
    ring.fetch_pair(0);
    ring.fetch_pair(1);
    ring.fetch_pair(2);
    Ring::template landed_barrier<true>();

    // MFMAs of one unit in issue order: groups of QT sharing one LDS fragment; groups of the
    // previous unit's P V update (kind 0, arg = half*CT+ct) alternate with groups of the next
    // unit's S^T (kind 1, arg = ks).
    constexpr int NA = 2 * CT, NB = KS, NG = NA + NB, NM = NG * QT;
    struct Plan {
        int kind[NG], arg[NG];
    };
    constexpr Plan plan = [] {
        Plan p{};
        int n = 0, ia = 0, ib = 0;
        while (ia < NA || ib < NB) {
            if (ia < NA) p.kind[n] = 0, p.arg[n++] = ia++;
            if (ib < NB) p.kind[n] = 1, p.arg[n++] = ib++;
        }
        return p;
    }();
    constexpr int LA = 2;  // fragment reads run this many groups ahead
    constexpr int NE = 16 * QT;    // score elements per lane and unit
    static_assert(NPW + 2 <= NG, "the tile loads must fit the MFMA groups of a unit");
    // Group of the first unit of an iteration after which the wavefronts synchronise.  Before it,
    // all reads of the PREVIOUS V tile must have returned, because the next loads overwrite that
    // tile pair; after it come the first reads of the NEXT K tile (requested LA groups ahead for
    // the following unit), because only then is it complete.
    static_assert(LA >= 1 && plan.kind[0] == 0 && plan.kind[1] == 1, "the first read of the next tile is the unit's second fragment");
    constexpr int LAST_PREV_GROUP = [] {
        int last = 0;
        for (int i = 0; i < NG; ++i)
            if (plan.kind[i] == 0) last = i;
        return last;
    }();
    constexpr int FIRST_NEXT_GROUP = NG - LA + 1;
    constexpr int SYNC_GROUP = LAST_PREV_GROUP < FIRST_NEXT_GROUP ? LAST_PREV_GROUP : FIRST_NEXT_GROUP - 1;
    constexpr bool SYNC_DRAINS = LAST_PREV_GROUP > SYNC_GROUP;  // then outstanding LDS reads are waited for

    // Which LDS tiles a unit reads: S^T of the NEXT unit from (knext, half hnext), the P V update of
    // the PREVIOUS unit from (vprev, half hprev).
    struct Where {
        const char *knext, *vprev;
        int hnext, hprev;
    };
    auto frag = [&](const Where& w, int gi) -> bf16x8 {
        const int kd = plan.kind[gi], ar = plan.arg[gi];
        if (kd == 0) return tr_frag(w.vprev, STRIDE, tr_off, ar % CT, 2 * w.hprev + ar / CT);
        return nat_frag(w.knext, STRIDE, 32 * w.hnext + l32, ar, g);
    };

    // One unit: MASKED units replace scores of keys at or beyond N by -inf first.  `pre` arrives
    // holding the first LA fragments of this unit and leaves holding those of the unit that follows
    // (`wn`), so the LDS pipeline never drains between units.  side(j), j = 0 .. NPW-1, is called in
    // groups 2, 3, ...: the tile loads.
    auto unit = [&](auto sync, auto masked, int key_base, const Where& w, const Where& wn, f32x16 (&s_c)[QT],
                    f32x16 (&s_n)[QT], const u32x4 (&pf_p)[QT][2], u32x4 (&pf_c)[QT][2], bf16x8 (&pre)[LA],
                    auto&& side) {
        if constexpr (decltype(masked)::value) {
            const int key0 = key_base + 4 * g;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (key0 + 8 * (i / 4) + (i % 4) >= N) {
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) s_c[qt][i] = -INFINITY;
                }
        }
        bf16x8 fr[NG];
#pragma unroll
        for (int gi = 0; gi < LA; ++gi) fr[gi] = pre[gi];
        const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if (gi + LA < NG) fr[gi + LA] = frag(w, gi + LA);
            else pre[gi + LA - NG] = frag(wn, gi + LA - NG);
            const int kd = plan.kind[gi], ar = plan.arg[gi];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                if (kd == 0)
                    oacc[ar % CT][qt] = mfma32(fr[gi], as_bf16x8(pf_p[qt][ar / CT]), oacc[ar % CT][qt]);
                else
                    s_n[qt] = mfma32(fr[gi], qf[qt][ar], ar == 0 ? f32x16_zero() : s_n[qt]);
                // vector-ALU share of this MFMA slot
                const int m = gi * QT + qt;
                const int e0 = m * NE / NM, e1 = (m + 1) * NE / NM;
#pragma unroll
                for (int e = e0; e < e1; ++e) {
                    const int eq = e / 16, i = e % 16;
                    const float p = fast_exp2(fmaf(s_c[eq][i], cs, -m_used[eq]));
                    s_c[eq][i] = p;
                    lsum[eq] += p;
                    if (i % 2 == 1) {
                        // the second row sum runs over the weights as rounded to bf16, i.e. the
                        // numbers the second contraction multiplies V with; O is divided by it
                        const unsigned wgt = pack_bf16(s_c[eq][i - 1], p);
                        pf_c[eq][i / 8][(i / 2) % 4] = wgt;
                        rsum[eq] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, wgt), ones, rsum[eq], false);
                    }
                }
                if (qt == QT - 1) {
                    if (gi >= 2 && gi - 2 < NPW) side(gi - 2);
                    if (decltype(sync)::value && gi == SYNC_GROUP) Ring::template landed_barrier<SYNC_DRAINS>();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // P V update of one unit outside the pipeline (the very last one)
    auto pv_only = [&](const char* vb, int hq, const u32x4 (&pf)[QT][2]) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 a = tr_frag(vb, STRIDE, tr_off, ct, 2 * hq + half);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) oacc[ct][qt] = mfma32(a, as_bf16x8(pf[qt][half]), oacc[ct][qt]);
            }
    };

    f32x16 sA[QT], sB[QT];
    u32x4 pfA[QT][2], pfB[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            pfA[qt][i] = z, pfB[qt][i] = z;
        }
    if (wave_active) {
        // S^T of unit 0 and the per-query reference maximum over its (valid) keys
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = nat_frag(kbuf(0), STRIDE, l32, ks, g);
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) sA[qt] = mfma32(a, qf[qt][ks], ks == 0 ? f32x16_zero() : sA[qt]);
        }
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            f32x16 tmp = sA[qt];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (4 * g + 8 * (i / 4) + (i % 4) >= N) tmp[i] = -INFINITY;
            m_used[qt] = both_halves_max(max16(tmp)) * cs;
        }
    }
    wait_all_loads();

    // One step = one 64-key tile = two units.  Unit 2t: current = A; next = unit 2t+1 (K tile t,
    // second half); previous = unit 2t-1 (V tile t-1, second half; at t = 0 its weights are zero
    // and V tile 0 stands in).  Unit 2t+1: current = B; next = unit 2t+2 (K tile t+1, first half;
    // past the last tile a zero tile whose scores are never used); previous = unit 2t (V tile t,
    // first half).  One synchronisation per step, inside unit 2t: it certifies that tile pair t+1
    // is complete (first read right after it) and that nobody reads pair t-1 any more, whose
    // buffers the loads of pair t+3, issued during unit 2t+1, overwrite.  A tile therefore has one
    // and a half steps to arrive.
    auto where_a = [&](int t) { return Where{kbuf(t), vbuf(t - 1 < 0 ? 0 : t - 1), 1, 1}; };
    auto where_b = [&](int t) { return Where{kbuf(t + 1), vbuf(t), 0, 0}; };
    bf16x8 pre[LA];
    {
        const Where w0 = where_a(0);
#pragma unroll
        for (int gi = 0; gi < LA; ++gi) pre[gi] = frag(w0, gi);
    }
    for (int t = 0; t < ntiles; ++t) {
        const Where wa = where_a(t), wb = where_b(t), wa1 = where_a(t + 1);
        auto next_tile = [&](int j) { ring.fetch(t + 3, j); };
        auto nothing = [](int) {};
        if (wave_active) {
            if ((t + 1) * BN > N) {
                unit(std::true_type{}, std::true_type{}, t * BN, wa, wb, sA, sB, pfB, pfA, pre, nothing);
                unit(std::false_type{}, std::true_type{}, t * BN + 32, wb, wa1, sB, sA, pfA, pfB, pre, next_tile);
            } else {
                unit(std::true_type{}, std::false_type{}, 0, wa, wb, sA, sB, pfB, pfA, pre, nothing);
                unit(std::false_type{}, std::false_type{}, 0, wb, wa1, sB, sA, pfA, pfB, pre, next_tile);
            }
        } else {
            Ring::template landed_barrier<false>();
            ring.fetch_pair(t + 3);
        }
    }
    if (wave_active) pv_only(vbuf(ntiles - 1), 1, pfB);

    // overflow of the fixed reference: redo this workgroup's rows with the running maximum
    bool bad = false;
    if (wave_active) {
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            const float l = both_halves_sum(lsum[qt]);
            bad = bad || !(l <= kRowSumLimit);
        }
    }
    wait_all_loads();  // zero tiles requested past the end must have landed before LDS is reused
    if (__syncthreads_or(bad ? 1 : 0))
        avion_fwd_safe_pass<D, QT, NW>(smem, kh, vh, qf, oacc, m_used, lsum, rsum, N, cs, wave_active, tid, l32, g, tr_off,
                                       4 * Stage::BYTES);

    // every wavefront is past its last tile read (barrier above): the tile buffers are free and
    // serve as the per-wavefront staging area of the output rows
    if (!wave_active) return;
    char* region = smem + wave * RowStore<D>::BYTES;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float l = both_halves_sum(lsum[qt]);
        const float inv = 1.0f / both_halves_sum(rsum[qt]);
        const int row0 = q0 + 32 * qt;
        f32x16 tile[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) tile[ct] = oacc[ct][qt];
        // each lane scales by its own query's divisor before the rows are transposed
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) tile[ct][i] *= inv;
        RowStore<D>::run(region, tile, 1.0f, oh + (long)row0 * rs, rs, N - row0, lane);
        if (g == 0 && row0 + l32 < N) lse[(long)bh * N + row0 + l32] = (m_used[qt] + __builtin_amdgcn_logf(l)) * kLn2;
    }
}


// ---------------------------------------------------------------------------------------------
// Occupancy-oriented forward kernel.  Same mathematics, layouts and fallback as avion_fwd_kernel,
// but no software pipelining: each wavefront runs S^T, softmax, P V of one 32-key unit after the
// other with few live registers, and a compute unit holds many wavefronts (small LDS footprint:
// two K/V tile pairs), so that while one wavefront waits for its matrix instructions another one
// issues vector work.  One workgroup barrier per 64-key tile: passing it certifies that the next
// tile pair has landed and that the previous one is no longer read, so its buffers can be refilled.
// ---------------------------------------------------------------------------------------------
template <int D, int NW>
struct FwdOccCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * NW;
    using Ring = PairRing<D, NW, 2>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    static constexpr int WAVES_PER_SIMD = (160 * 1024 / LDS_BYTES) * NW / 4 > 4 ? 4 : (160 * 1024 / LDS_BYTES) * NW / 4;
};

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64, (FwdOccCfg<D, NW>::WAVES_PER_SIMD))
avion_fwd_occ_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                     bf16* __restrict__ o, float* __restrict__ lse, int H, int N, int nqb, int nblocks, float cs)
{
    using Cfg = FwdOccCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16, CT = (D + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nqb, qb = logical % nqb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const SliceView kh(k + head_off, rs, N, D);
    const SliceView vh(v + head_off, rs, N, D);
    const int q0 = qb * BM + wave * 32;
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    const int ntiles = (N + BN - 1) / BN;

    const Ring ring(k + head_off, v + head_off, kh.bytes, kh.row_bytes, smem, wave, lane);
    ring.fetch_pair(0);

    bf16x8 qf[1][KS];
    {
        const int row = min(q0 + l32, N - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[0][ks] = *reinterpret_cast<const bf16x8*>(q + head_off + (long)row * rs + ks * 16 + g * 8);
    }
    f32x16 oacc[CT][1];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) oacc[ct][0] = f32x16_zero();
    float m_used[1] = {0.f}, lsum[1] = {0.f}, rsum[1] = {0.f};

    wait_all_loads();
    Ring::template landed_barrier<false, 0>();  // tile pair 0 is in LDS

    // S^T of one unit (32 keys starting at row 32*hk of the K tile); RAGGED units reach past the
    // last key and start from the key mask instead of zero
    auto scores = [&](auto ragged, const char* kt, int hk, int key_base) -> f32x16 {
        constexpr bool RAGGED = decltype(ragged)::value;
        f32x16 s;
        if constexpr (RAGGED) s = key_mask_block(key_base, g, N);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            s = mfma32(nat_frag(kt, STRIDE, 32 * hk + l32, ks, g), qf[0][ks], ks == 0 && !RAGGED ? f32x16_zero() : s);
        return s;
    };
    // reference maximum: over the first 32 keys
    if (wave_active) m_used[0] = both_halves_max(max16(scores(std::true_type{}, ring.a_tile(0), 0, 0))) * cs;

    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
    for (int t = 0; t < ntiles; ++t) {
        ring.fetch_pair(t + 1);  // into the buffers of pair t-1, which nobody reads any more
        if (wave_active) {
            const char* kt = ring.a_tile(t);
            const char* vt = ring.b_tile(t);
#pragma unroll
            for (int hk = 0; hk < 2; ++hk) {
                const int key_base = t * BN + 32 * hk;
                f32x16 s;
                if (key_base + 32 > N) s = scores(std::true_type{}, kt, hk, key_base);
                else s = scores(std::false_type{}, kt, hk, key_base);
                // the V^T operands are requested before the vector work so that they are there after it
                bf16x8 vf[2][CT];
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) vf[half][ct] = tr_frag(vt, STRIDE, tr_off, ct, 2 * hk + half);
                u32x4 pf[2];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = fast_exp2(fmaf(s[i], cs, -m_used[0]));
                    s[i] = p;
                    lsum[0] += p;
                    if (i % 2 == 1) {
                        const unsigned wgt = pack_bf16(s[i - 1], p);
                        pf[i / 8][(i / 2) % 4] = wgt;
                        rsum[0] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, wgt), ones, rsum[0], false);
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) oacc[ct][0] = mfma32(vf[half][ct], as_bf16x8(pf[half]), oacc[ct][0]);
            }
        }
        Ring::template landed_barrier<false, 0>();  // pair t+1 has landed; pair t is no longer read
    }

    bool bad = false;
    if (wave_active) bad = !(both_halves_sum(lsum[0]) <= kRowSumLimit);
    if (__syncthreads_or(bad ? 1 : 0))
        avion_fwd_safe_pass<D, 1, NW>(smem, kh, vh, qf, oacc, m_used, lsum, rsum, N, cs, wave_active, tid, l32, g, tr_off,
                                      2 * Ring::TILE_BYTES);
    if (!wave_active) return;
    const float l = both_halves_sum(lsum[0]);
    const float inv = 1.0f / both_halves_sum(rsum[0]);
    f32x16 tile[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) tile[ct][i] = oacc[ct][0][i] * inv;
    RowStore<D>::run(smem + wave * RowStore<D>::BYTES, tile, 1.0f, o + head_off + (long)q0 * rs, rs, N - q0, lane);
    if (g == 0 && q0 + l32 < N) lse[(long)bh * N + q0 + l32] = (m_used[0] + __builtin_amdgcn_logf(l)) * kLn2;
}
