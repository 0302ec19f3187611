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
// One wavefront owns 32 queries (Q, dO as B-operand fragments, LSE and delta as per-lane scalars);
// the workgroup's NW wavefronts share K/V tile pairs of 64 keys that stream through a ring of four
// LDS buffers each, filled by LDS-direct loads.  Work is cut into units of 32 keys and pipelined
// like the other two kernels: in program order a unit interleaves, instruction by instruction,
//   matrix cores : S^T = K Q^T and dP^T = V dO^T of the NEXT unit (second accumulator pair; the dP
//                  accumulator starts from -delta), and dQ^T += K^T dS^T of the PREVIOUS unit;
//   vector ALUs  : P = exp2(cs*S - lc) and dS = P o (dP - delta) of the CURRENT unit, rounded to bf16.
template <int D, int NW>
struct DqCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * NW;
    using Ring = PairRing<D, NW>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    // wavefronts per SIMD the register budget is sized for: as many as LDS lets a compute unit hold
    static constexpr int WAVES_PER_SIMD = (160 * 1024 / LDS_BYTES) * NW / 4;
};

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64, (DqCfg<D, NW>::WAVES_PER_SIMD))
avion_dq_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                const bf16* __restrict__ o, const bf16* __restrict__ dO, const float* __restrict__ lse,
                bf16* __restrict__ dq, float* __restrict__ rowsc, int H, int N, int nqb, int nblocks,
                float cs, float scale)
{
    using Cfg = DqCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16;
    constexpr int CT = (D + 31) / 32;
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
    const int q0 = qb * BM + wave * 32;
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // K/V tile pairs: request the first three before anything else
    const int ntiles = (N + BN - 1) / BN;
    const Ring ring(k + head_off, v + head_off, kh.bytes, kh.row_bytes, smem, wave, lane);
    ring.fetch_pair(0);
    ring.fetch_pair(1);
    ring.fetch_pair(2);

    // Q and dO fragments (B operands), delta and LSE per lane
    bf16x8 qf[KS], gf[KS];
    float lc, dl;
    {
        const int row = min(q0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
            gf[ks] = *reinterpret_cast<const bf16x8*>(dO + off + ks * 16);
            const bf16x8 of = *reinterpret_cast<const bf16x8*>(o + off + ks * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf((float)of[e], (float)gf[ks][e], part);
        }
        dl = both_halves_sum(part);
        lc = lse[(long)bh * N + row] * kLog2e;
        // per-query scalars for the dK/dV pass, in the form it consumes them: LSE*log2e and -delta,
        // each array padded to a multiple of 64 rows with +inf (weight 0) and 0
        const int qrow = q0 + l32, npad = (N + 63) & ~63;
        if (g == 0 && qrow < npad) {
            float* ws = rowsc + (long)bh * 2 * npad;
            ws[qrow] = qrow < N ? lc : INFINITY;
            ws[npad + qrow] = qrow < N ? -dl : 0.f;
        }
    }
    const float nlc = -lc;
    // -delta of the lane's query in every element: the initial value of each dP accumulator, so
    // that the MFMAs deliver dP - delta and the subtraction costs no vector-ALU instruction
    f32x16 ndl;
#pragma unroll
    for (int i = 0; i < 16; ++i) ndl[i] = -dl;

    f32x16 acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x16_zero();

    // The MFMAs of one unit, in issue order: each dQ update of the previous unit is followed by a
    // pair (S, dP) of the next unit.  kind: 0 dQ, 2 S, 3 dP; arg: half*CT+ct or ks.
    constexpr int NA = 2 * CT, NB = KS, NM = NA + 2 * NB;
    struct Plan {
        int kind[NM], arg[NM];
    };
    constexpr Plan plan = [] {
        Plan p{};
        int n = 0, ia = 0, ib = 0;
        while (ia < NA || ib < NB) {
            if (ia < NA) p.kind[n] = 0, p.arg[n++] = ia++;
            if (ib < NB) {
                p.kind[n] = 2, p.arg[n++] = ib;
                p.kind[n] = 3, p.arg[n++] = ib++;
            }
        }
        return p;
    }();
    constexpr int LA = 3;  // LDS fragment reads run this many MFMAs ahead of their use
    constexpr int NPW = Ring::NPW;
    static_assert(NPW + 2 <= NM, "the tile loads must fit the MFMA slots of a unit");
    // Slot of the first unit of an iteration after which the wavefronts synchronise.  Before it, all
    // reads of the PREVIOUS K tile (dQ operands) must have returned, because the next loads
    // overwrite that tile pair; after it come the first reads of the NEXT tile pair (requested LA
    // slots ahead for the following unit), because only then is it complete.
    static_assert(LA >= 1 && plan.kind[0] == 0 && plan.kind[1] >= 2, "the first read of the next tile is the unit's second fragment");
    constexpr int LAST_PREV_SLOT = [] {
        int last = 0;
        for (int i = 0; i < NM; ++i)
            if (plan.kind[i] == 0) last = i;
        return last;
    }();
    constexpr int FIRST_NEXT_SLOT = NM - LA + 1;
    constexpr int SYNC_SLOT = LAST_PREV_SLOT < FIRST_NEXT_SLOT ? LAST_PREV_SLOT : FIRST_NEXT_SLOT - 1;
    constexpr bool SYNC_DRAINS = LAST_PREV_SLOT > SYNC_SLOT;  // then outstanding LDS reads are waited for

    // Which LDS tiles a unit reads: S, dP of the NEXT unit from half hnext of (knext, vnext); the dQ
    // update of the PREVIOUS unit from half hprev of kprev.
    struct Where {
        const char *knext, *vnext, *kprev;
        int hnext, hprev;
    };
    auto frag = [&](const Where& w, int i) -> bf16x8 {
        const int kd = plan.kind[i], ar = plan.arg[i];
        if (kd == 0) return tr_frag(w.kprev, STRIDE, tr_off, ar % CT, 2 * w.hprev + ar / CT);
        if (kd == 2) return nat_frag(w.knext, STRIDE, 32 * w.hnext + l32, ar, g);
        return nat_frag(w.vnext, STRIDE, 32 * w.hnext + l32, ar, g);
    };

    // One unit.  cur = S, dP of the current unit (dS ends up in dp_c), nxt = accumulators of the
    // next unit, df_p / df_c = bf16 dS fragments of the previous / current unit.  When the NEXT
    // unit reaches past the last key (next_ragged), its score accumulator starts from the key mask
    // instead of zero.  `pre` arrives holding the first LA fragments of this unit and leaves holding
    // those of the unit that follows (`wn`).  side(j), j = 0 .. NPW-1, is called in slots 2, 3, ...:
    // the tile loads.
    auto unit = [&](auto sync, auto next_ragged, int next_key_base, const Where& w, const Where& wn, f32x16& s_c,
                    f32x16& dp_c, f32x16& s_n, f32x16& dp_n, const u32x4 (&df_p)[2], u32x4 (&df_c)[2],
                    bf16x8 (&pre)[LA], auto&& side) {
        constexpr bool RAGGED = decltype(next_ragged)::value;
        bf16x8 fr[NM];
#pragma unroll
        for (int i = 0; i < LA; ++i) fr[i] = pre[i];
        if constexpr (RAGGED) s_n = key_mask_block(next_key_base, g, N);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            if (i + LA < NM) fr[i + LA] = frag(w, i + LA);
            else pre[i + LA - NM] = frag(wn, i + LA - NM);
            const int kd = plan.kind[i], ar = plan.arg[i];
            if (kd == 0) acc[ar % CT] = mfma32(fr[i], as_bf16x8(df_p[ar / CT]), acc[ar % CT]);
            if (kd == 2) s_n = mfma32(fr[i], qf[ar], ar == 0 && !RAGGED ? f32x16_zero() : s_n);
            if (kd == 3) dp_n = mfma32(fr[i], gf[ar], ar == 0 ? ndl : dp_n);
            // vector-ALU share of this slot: elements e0..e1-1 of the current unit
            const int e0 = i * 16 / NM, e1 = (i + 1) * 16 / NM;
#pragma unroll
            for (int e = e0; e < e1; ++e) {
                const float pe = fast_exp2(fmaf(s_c[e], cs, nlc));
                dp_c[e] = pe * dp_c[e];  // dp_c already holds dP - delta
                if (e % 2 == 1) df_c[e / 8][(e / 2) % 4] = pack_bf16(dp_c[e - 1], dp_c[e]);
            }
            if (i >= 2 && i - 2 < NPW) side(i - 2);
            if (decltype(sync)::value && i == SYNC_SLOT) Ring::template landed_barrier<SYNC_DRAINS>();
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    Ring::template landed_barrier<true>();  // pairs 0 and 1 are in LDS

    f32x16 sA, dpA, sB, dpB;
    u32x4 dfA[2], dfB[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        dfA[i] = z, dfB[i] = z;
    }
    if (wave_active) {
        sA = key_mask_block(0, g, N);  // all zeros unless N < 32
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ak = nat_frag(ring.a_tile(0), STRIDE, l32, ks, g);
            const bf16x8 av = nat_frag(ring.b_tile(0), STRIDE, l32, ks, g);
            sA = mfma32(ak, qf[ks], sA);
            dpA = mfma32(av, gf[ks], ks == 0 ? ndl : dpA);
        }
    }
    wait_all_loads();

    // One step = one 64-key tile pair = two units.  Unit 2t: current = A; next = unit 2t+1 (second
    // half of pair t); previous = unit 2t-1 (second half of K tile t-1; at t = 0 its dS is zero and
    // tile 0 stands in).  Unit 2t+1: current = B; next = unit 2t+2 (first half of pair t+1; past the
    // last tile a zero tile whose scores are never used); previous = unit 2t.  One synchronisation
    // per step, inside unit 2t: it certifies that pair t+1 is complete (first read right after it)
    // and that nobody reads pair t-1 any more, whose buffers the loads of pair t+3, issued during
    // unit 2t+1, overwrite.  A pair therefore has one and a half steps to arrive.
    auto where_a = [&](int t) { return Where{ring.a_tile(t), ring.b_tile(t), ring.a_tile(t - 1 < 0 ? 0 : t - 1), 1, 1}; };
    auto where_b = [&](int t) { return Where{ring.a_tile(t + 1), ring.b_tile(t + 1), ring.a_tile(t), 0, 0}; };
    bf16x8 pre[LA];
    {
        const Where w0 = where_a(0);
#pragma unroll
        for (int i = 0; i < LA; ++i) pre[i] = frag(w0, i);
    }
    for (int t = 0; t < ntiles; ++t) {
        const Where wa = where_a(t), wb = where_b(t), wa1 = where_a(t + 1);
        auto next_pair = [&](int j) { ring.fetch(t + 3, j); };
        auto nothing = [](int) {};
        if (wave_active) {
            // unit 2t prepares the scores of keys 64t+32.., unit 2t+1 those of keys 64(t+1)..
            if ((t + 1) * BN > N)
                unit(std::true_type{}, std::true_type{}, t * BN + 32, wa, wb, sA, dpA, sB, dpB, dfB, dfA, pre, nothing);
            else
                unit(std::true_type{}, std::false_type{}, 0, wa, wb, sA, dpA, sB, dpB, dfB, dfA, pre, nothing);
            if ((t + 1) * BN + 32 > N)
                unit(std::false_type{}, std::true_type{}, (t + 1) * BN, wb, wa1, sB, dpB, sA, dpA, dfA, dfB, pre, next_pair);
            else
                unit(std::false_type{}, std::false_type{}, 0, wb, wa1, sB, dpB, sA, dpA, dfA, dfB, pre, next_pair);
        } else {
            Ring::template landed_barrier<false>();
            ring.fetch_pair(t + 3);
        }
    }
    // the last unit's contribution
    if (wave_active) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 a = tr_frag(ring.a_tile(ntiles - 1), STRIDE, tr_off, ct, 2 + half);
                acc[ct] = mfma32(a, as_bf16x8(dfB[half]), acc[ct]);
            }
    }
    wait_all_loads();  // zero tiles requested past the end must have landed before LDS is reused
    __syncthreads();   // all tile reads are done: the buffers now stage the output rows
    if (!wave_active) return;
    char* region = smem + wave * RowStore<D>::BYTES;
    RowStore<D>::run(region, acc, scale, dq + head_off + (long)q0 * rs, rs, N - q0, lane);
}

// Occupancy-oriented dQ kernel.  Same mathematics and layouts as avion_dq_kernel, but no software
// pipelining: each wavefront runs S^T / dP^T, the vector work and the dQ^T update of one 32-key unit
// after the other with few live registers, and a compute unit holds many wavefronts (two K/V tile
// pairs in LDS), so that while one wavefront waits for its matrix instructions another one issues
// vector work.  One workgroup barrier per 64-key tile pair: passing it certifies that the next pair
// has landed and that the previous one is no longer read, so its buffers can be refilled.
template <int D, int NW>
struct DqOccCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * NW;
    using Ring = PairRing<D, NW, 2>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    static constexpr int WAVES_PER_SIMD = D == 64 ? 3 : 2;  // LDS would allow more; registers do not
};

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64, (DqOccCfg<D, NW>::WAVES_PER_SIMD))
avion_dq_occ_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                    const bf16* __restrict__ o, const bf16* __restrict__ dO, const float* __restrict__ lse,
                    bf16* __restrict__ dq, float* __restrict__ rowsc, int H, int N, int nqb, int nblocks,
                    float cs, float scale)
{
    using Cfg = DqOccCfg<D, NW>;
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
    const int q0 = qb * BM + wave * 32;
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    const int ntiles = (N + BN - 1) / BN;

    const Ring ring(k + head_off, v + head_off, kh.bytes, kh.row_bytes, smem, wave, lane);
    ring.fetch_pair(0);

    // Q and dO fragments (B operands), delta and LSE per lane
    bf16x8 qf[KS], gf[KS];
    float lc, dl;
    {
        const int row = min(q0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
            gf[ks] = *reinterpret_cast<const bf16x8*>(dO + off + ks * 16);
            const bf16x8 of = *reinterpret_cast<const bf16x8*>(o + off + ks * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf((float)of[e], (float)gf[ks][e], part);
        }
        dl = both_halves_sum(part);
        lc = lse[(long)bh * N + row] * kLog2e;
        // per-query scalars for the dK/dV pass, in the form it consumes them: LSE*log2e and -delta,
        // each array padded to a multiple of 64 rows with +inf (weight 0) and 0
        const int qrow = q0 + l32, npad = (N + 63) & ~63;
        if (g == 0 && qrow < npad) {
            float* ws = rowsc + (long)bh * 2 * npad;
            ws[qrow] = qrow < N ? lc : INFINITY;
            ws[npad + qrow] = qrow < N ? -dl : 0.f;
        }
    }
    const float nlc = -lc;
    f32x16 acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x16_zero();

    wait_all_loads();
    Ring::template landed_barrier<false, 0>();  // tile pair 0 is in LDS

    // one 32-key unit: rows 32*hk.. of the tile pair; RAGGED units reach past the last key and
    // start the score accumulator from the key mask instead of zero
    auto unit = [&](auto ragged, const char* kt, const char* vt, int hk, int key_base) {
        constexpr bool RAGGED = decltype(ragged)::value;
        f32x16 s, dp;
        if constexpr (RAGGED) s = key_mask_block(key_base, g, N);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ak = nat_frag(kt, STRIDE, 32 * hk + l32, ks, g);
            const bf16x8 av = nat_frag(vt, STRIDE, 32 * hk + l32, ks, g);
            s = mfma32(ak, qf[ks], ks == 0 && !RAGGED ? f32x16_zero() : s);
            dp = mfma32(av, gf[ks], ks == 0 ? f32x16_zero() : dp);
        }
        // the K^T operands are requested before the vector work so that they are there after it
        bf16x8 kt_f[2][CT];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) kt_f[half][ct] = tr_frag(kt, STRIDE, tr_off, ct, 2 * hk + half);
        u32x4 df[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pe = fast_exp2(fmaf(s[i], cs, nlc));
            s[i] = pe * (dp[i] - dl);
            if (i % 2 == 1) df[i / 8][(i / 2) % 4] = pack_bf16(s[i - 1], s[i]);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[ct] = mfma32(kt_f[half][ct], as_bf16x8(df[half]), acc[ct]);
    };

    for (int t = 0; t < ntiles; ++t) {
        ring.fetch_pair(t + 1);  // into the buffers of pair t-1, which nobody reads any more
        if (wave_active) {
#pragma unroll
            for (int hk = 0; hk < 2; ++hk) {
                const int key_base = t * BN + 32 * hk;
                if (key_base + 32 > N) unit(std::true_type{}, ring.a_tile(t), ring.b_tile(t), hk, key_base);
                else unit(std::false_type{}, ring.a_tile(t), ring.b_tile(t), hk, key_base);
            }
        }
        Ring::template landed_barrier<false, 0>();  // pair t+1 has landed; pair t is no longer read
    }
    if (!wave_active) return;
    RowStore<D>::run(smem + wave * RowStore<D>::BYTES, acc, scale, dq + head_off + (long)q0 * rs, rs, N - q0, lane);
}

// ------------------------------------------------------------------------------------------ dK, dV
// One wavefront owns 32 keys; the workgroup's NW wavefronts share LDS tiles of BQ = 64 queries
// (Q and dO rows, LSE*log2e and -delta), four buffers deep, filled straight from global memory by
// LDS-direct loads (no staging registers, no LDS write instructions).  Work is cut into units of 32
// queries.  In program order every unit holds three independent strands that are interleaved
// instruction by instruction, because a wavefront issues in order and an MFMA that is queued behind
// another one blocks everything after it:
//   matrix cores : S and dP of the NEXT unit (into a second accumulator pair), and the dV^T, dK^T
//                  updates of the PREVIOUS unit (from its saved bf16 P and dS fragments);
//   vector ALUs  : P = exp2(cs*S - lc), dS = P o (dP - delta) of the CURRENT unit, rounded to bf16
//                  (the dP accumulator starts from -delta, so the subtraction costs nothing).
template <int D, int NW>
struct DkvCfg {
    static constexpr int BQ = 64;  // queries per LDS tile (two units)
    static constexpr int NT = NW * 64;
    static constexpr int BNK = 32 * NW;  // keys per workgroup
    static constexpr int NBUF = 4;
    using Stage = TileStage<D, BQ, NT>;
    static constexpr int ROWV_BYTES = 1024;  // lc[BQ] | -delta[BQ] | unused: one 1 KB load
    static constexpr int BUF_BYTES = 2 * Stage::BYTES + ROWV_BYTES;
    static constexpr int LDS_BYTES = NBUF * BUF_BYTES;
};

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64)
avion_dkdv_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                  const bf16* __restrict__ dO, const float* __restrict__ rowsc,
                  bf16* __restrict__ dk, bf16* __restrict__ dv, int H, int N, int nkb, int nblocks,
                  float cs, float scale)
{
    using Cfg = DkvCfg<D, NW>;
    using Stage = typename Cfg::Stage;
    constexpr int BQ = Cfg::BQ, BNK = Cfg::BNK, STRIDE = Stage::STRIDE;
    constexpr int KS = D / 16;
    constexpr int CT = (D + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // per buffer: Q tile | dO tile | lc[BQ] | -delta[BQ]
    constexpr int OFF_G = Stage::BYTES, OFF_ROW = 2 * Stage::BYTES;
    auto tilebuf = [&](int ti) { return smem + (ti & 3) * Cfg::BUF_BYTES; };

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nkb, kb = logical % nkb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const SliceView qh(q + head_off, rs, N, D);
    const SliceView gh(dO + head_off, rs, N, D);
    // per-query scalars as the dQ pass left them: lc[npad] = LSE*log2e, then -delta[npad]
    const int npad = (N + 63) & ~63;
    const RawBuffer rowsc_buf(rowsc + (long)bh * 2 * npad, 2 * npad * 4);
    const RawBuffer q_buf(q + head_off, qh.bytes), g_buf(dO + head_off, gh.bytes);
    const int k0 = kb * BNK + wave * 32;  // first key of this wavefront
    const bool wave_active = k0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // K and V fragments (B operands: lane = key) stay in registers
    bf16x8 kf[KS], vf[KS];
    {
        const int row = min(k0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(k + off + ks * 16);
            vf[ks] = *reinterpret_cast<const bf16x8*>(v + off + ks * 16);
        }
    }

    f32x16 dka[CT], dva[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        dka[ct] = f32x16_zero();
        dva[ct] = f32x16_zero();
    }

    // Tile movement.  A tile buffer is a sequence of 1 KB blocks, each filled by one LDS-direct
    // load of one wavefront: NTI blocks of Q rows, NTI of dO rows (row stride STRIDE, so a block
    // holds 64 consecutive 16-byte chunks of the padded rows; lanes that land on a pad chunk fetch
    // from beyond the buffer and deposit zeros), then one block with the 64 lc and 64 -delta values.
    // Wavefront w issues blocks w, w+NW, ... of Q and of dO; the remaining blocks (the last of Q,
    // the last of dO, the scalars) go one each to wavefronts 0, 1, 2, and further wavefronts repeat
    // the scalars so that every wavefront issues the same number NPW of loads per tile.
    static_assert(Stage::BYTES % 1024 == 0, "a tile must be a whole number of 1 KB blocks");
    constexpr int NTI = Stage::BYTES / 1024, FULL = NTI / NW, REM = NTI % NW;
    static_assert(REM == 1 && NW >= 3, "block distribution assumes one left-over block per tensor");
    constexpr int NPW = 2 * FULL + 1;
    const unsigned row_bytes = qh.row_bytes;
    auto block_voff = [&](int blk) { return padded_block_voff<D>(blk, lane, row_bytes); };
    unsigned voff[FULL];
#pragma unroll
    for (int m = 0; m < FULL; ++m) voff[m] = block_voff(wave + NW * m);
    const bool left_is_rows = wave < 2;  // wavefront 0: last Q block, 1: last dO block, else scalars
    const unsigned left_voff = left_is_rows ? block_voff(NTI - 1)
                               : lane < 16  ? (unsigned)lane * 16
                               : lane < 32  ? (unsigned)(npad * 4 + (lane - 16) * 16)
                                            : kOutOfRangeBase;
    const unsigned left_step = left_is_rows ? BQ * row_bytes : BQ * 4;  // per tile
    const RawBuffer left_buf = pick(wave == 0, q_buf, pick(wave == 1, g_buf, rowsc_buf));
    const int left_lds = wave == 0 ? (NTI - 1) * 1024 : wave == 1 ? OFF_G + (NTI - 1) * 1024 : OFF_ROW;
    const unsigned smem_addr = lds_address(smem);
    const int ntiles = (N + BQ - 1) / BQ;
    // load j (0 <= j < NPW) of this wavefront for tile `ti`; tiles past the end arrive as zeros
    auto fetch = [&](int ti, int j) {
        const unsigned buf = smem_addr + (ti & 3) * Cfg::BUF_BYTES;
        const unsigned base = (unsigned)ti * BQ * row_bytes;
        if (j < FULL) load_to_lds16(q_buf, buf + (wave + NW * j) * 1024, voff[j] + base);
        else if (j < 2 * FULL) load_to_lds16(g_buf, buf + OFF_G + (wave + NW * (j - FULL)) * 1024, voff[j - FULL] + base);
        else {
            const unsigned off = left_voff + (unsigned)ti * left_step;
            load_to_lds16(left_buf, buf + left_lds, (left_is_rows || ti < ntiles) ? off : kOutOfRangeBase);
        }
    };
    auto fetch_tile = [&](int ti) {
#pragma unroll
        for (int j = 0; j < NPW; ++j) fetch(ti, j);
    };
    // Wait until at most one tile's worth of this wavefront's loads is still in flight, then meet
    // the other wavefronts: after it, every tile but the most recently requested one is in LDS.
    // (Plain instructions instead of __syncthreads(): its fences would wait for ALL loads.)
    auto tiles_landed_barrier = [&](auto drain_lds) {
        if constexpr (decltype(drain_lds)::value)
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(NPW) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NPW) : "memory");
    };
    fetch_tile(0);
    fetch_tile(1);
    fetch_tile(2);
    tiles_landed_barrier(std::true_type{});

    // S and dP of one unit: rows = 32 queries (half hq of the tile), cols = this wave's 32 keys
    // -delta of the 16 queries this lane's accumulator registers belong to (broadcast LDS reads);
    // used as the initial value of the dP accumulator, so that the MFMAs deliver dP - delta
    auto neg_delta_rows = [&](const char* buf, int hq) -> f32x16 {
        const float* rowv = reinterpret_cast<const float*>(buf + OFF_ROW) + BQ + 32 * hq + 4 * g;
        f32x16 r;
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(rowv + 8 * a4);
#pragma unroll
            for (int e = 0; e < 4; ++e) r[4 * a4 + e] = d4[e];
        }
        return r;
    };
    // S and dP - delta of one unit: rows = 32 queries (half hq of the tile), cols = this wave's keys
    auto scores = [&](const char* buf, int hq, f32x16& s, f32x16& dp) {
        dp = neg_delta_rows(buf, hq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 aq = nat_frag(buf, STRIDE, 32 * hq + l32, ks, g);
            const bf16x8 ag = nat_frag(buf + OFF_G, STRIDE, 32 * hq + l32, ks, g);
            s = mfma32(aq, kf[ks], ks == 0 ? f32x16_zero() : s);
            dp = mfma32(ag, vf[ks], dp);
        }
    };
    // dV^T += dO^T P ,  dK^T += Q^T dS  of one unit (contraction over its 32 queries, 2 steps)
    auto accumulate = [&](const char* buf, int hq, const u32x4 (&pf)[2], const u32x4 (&df)[2]) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 ag = tr_frag(buf + OFF_G, STRIDE, tr_off, ct, 2 * hq + half);
                const bf16x8 aq = tr_frag(buf, STRIDE, tr_off, ct, 2 * hq + half);
                dva[ct] = mfma32(ag, as_bf16x8(pf[half]), dva[ct]);
                dka[ct] = mfma32(aq, as_bf16x8(df[half]), dka[ct]);
            }
    };

    // The MFMAs of one unit, in issue order: pairs (dV, dK) of the previous unit alternate with
    // pairs (S, dP) of the next unit.  kind: 0 dV, 1 dK, 2 S, 3 dP; arg: half*CT+ct or ks.
    constexpr int NA = 2 * CT, NB = KS, NM = 2 * (NA + NB);
    struct Plan {
        int kind[NM], arg[NM];
    };
    constexpr Plan plan = [] {
        Plan p{};
        int n = 0, ia = 0, ib = 0;
        while (ia < NA || ib < NB) {
            if (ia < NA) {
                p.kind[n] = 0, p.arg[n++] = ia;
                p.kind[n] = 1, p.arg[n++] = ia++;
            }
            if (ib < NB) {
                p.kind[n] = 2, p.arg[n++] = ib;
                p.kind[n] = 3, p.arg[n++] = ib++;
            }
        }
        return p;
    }();
    constexpr int LA = 3;  // LDS fragment reads run this many MFMAs ahead of their use
    static_assert(NPW + 2 <= NM, "the tile loads must fit the MFMA slots of a unit");
    // Slot of the first unit of an iteration after which the wavefronts synchronise.  Before it, all
    // reads of the PREVIOUS tile (dV, dK operands) must have returned, because the next loads
    // overwrite that tile; after it come the first reads of the NEXT tile (the S operand fetched
    // LA slots ahead for the following unit), because only then is it complete.
    constexpr int LAST_PREV_SLOT = [] {
        int last = 0;
        for (int i = 0; i < NM; ++i)
            if (plan.kind[i] <= 1) last = i;
        return last;
    }();
    static_assert(LA >= 2 && plan.kind[0] <= 1 && plan.kind[1] <= 1 && plan.kind[2] >= 2,
                  "the first read of the next tile is the unit's third fragment");
    constexpr int FIRST_NEXT_SLOT = NM - LA + 2;  // where the following unit's third fragment is requested
    constexpr int SYNC_SLOT = LAST_PREV_SLOT < FIRST_NEXT_SLOT ? LAST_PREV_SLOT : FIRST_NEXT_SLOT - 1;
    constexpr bool SYNC_DRAINS = LAST_PREV_SLOT > SYNC_SLOT;  // then outstanding LDS reads are waited for

    // Which LDS buffers a unit reads: S, dP of the NEXT unit from (bnext, half hnext); LSE of the
    // CURRENT unit from (bcur, hcur); dV, dK of the PREVIOUS unit from (bprev, hprev).
    struct Where {
        const char *bnext, *bcur, *bprev;
        int hnext, hcur, hprev;
    };
    auto frag = [&](const Where& w, int i) -> bf16x8 {
        const int kd = plan.kind[i], ar = plan.arg[i];
        if (kd == 0) return tr_frag(w.bprev + OFF_G, STRIDE, tr_off, ar % CT, 2 * w.hprev + ar / CT);
        if (kd == 1) return tr_frag(w.bprev, STRIDE, tr_off, ar % CT, 2 * w.hprev + ar / CT);
        if (kd == 2) return nat_frag(w.bnext, STRIDE, 32 * w.hnext + l32, ar, g);
        return nat_frag(w.bnext + OFF_G, STRIDE, 32 * w.hnext + l32, ar, g);
    };
    auto lse_rows = [&](const Where& w, int a4) -> f32x4 {
        return *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(w.bcur + OFF_ROW) + 32 * w.hcur + 4 * g + 8 * a4);
    };

    // One unit.  cur = S, dP of the current unit (turned into P, dS in place), nxt = accumulators of
    // the next unit, *_p = bf16 fragments of the previous unit, *_c = those of the current one.
    // `pre` and `l4pre` arrive holding the first LA fragments and the first four LSE values of this
    // unit and leave holding those of the unit that follows (`wn`), so the LDS pipeline never
    // drains between units.  side(j), j = 0 .. NPW-1, is called in slots 2, 3, ...: the tile loads.
    auto unit = [&](auto sync, const Where& w, const Where& wn, f32x16& s_c, f32x16& dp_c, f32x16& s_n,
                    f32x16& dp_n, const u32x4 (&pf_p)[2], const u32x4 (&df_p)[2], u32x4 (&pf_c)[2],
                    u32x4 (&df_c)[2], bf16x8 (&pre)[LA], f32x4& l4pre, auto&& side) {
        bf16x8 fr[NM];
        f32x4 l4[4];
#pragma unroll
        for (int i = 0; i < LA; ++i) fr[i] = pre[i];
        l4[0] = l4pre;
        dp_n = neg_delta_rows(w.bnext, w.hnext);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            if (i + LA < NM) fr[i + LA] = frag(w, i + LA);
            else pre[i + LA - NM] = frag(wn, i + LA - NM);
            const int kd = plan.kind[i], ar = plan.arg[i];
            if (kd == 0) dva[ar % CT] = mfma32(fr[i], as_bf16x8(pf_p[ar / CT]), dva[ar % CT]);
            if (kd == 1) dka[ar % CT] = mfma32(fr[i], as_bf16x8(df_p[ar / CT]), dka[ar % CT]);
            if (kd == 2) s_n = mfma32(fr[i], kf[ar], ar == 0 ? f32x16_zero() : s_n);
            if (kd == 3) dp_n = mfma32(fr[i], vf[ar], dp_n);
            // vector-ALU share of this slot: elements e0..e1-1 of the current unit
            const int e0 = i * 16 / NM, e1 = (i + 1) * 16 / NM;
#pragma unroll
            for (int e = e0; e < e1; ++e) {
                if (e % 4 == 0 && e + 4 < 16) l4[e / 4 + 1] = lse_rows(w, e / 4 + 1);  // next four queries
                const float pe = fast_exp2(fmaf(s_c[e], cs, -l4[e / 4][e % 4]));
                s_c[e] = pe;
                dp_c[e] = pe * dp_c[e];  // dp_c already holds dP - delta
                if (e % 2 == 1) {
                    pf_c[e / 8][(e / 2) % 4] = pack_bf16(s_c[e - 1], s_c[e]);
                    df_c[e / 8][(e / 2) % 4] = pack_bf16(dp_c[e - 1], dp_c[e]);
                }
            }
            if (i == NM - 1) l4pre = lse_rows(wn, 0);
            if (i >= 2 && i - 2 < NPW) side(i - 2);
            if (decltype(sync)::value && i == SYNC_SLOT) tiles_landed_barrier(std::bool_constant<SYNC_DRAINS>{});
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    f32x16 sA, dpA, sB, dpB;
    u32x4 pfA[2], dfA[2], pfB[2], dfB[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        pfA[i] = z, dfA[i] = z, pfB[i] = z, dfB[i] = z;
    }
    if (wave_active) scores(tilebuf(0), 0, sA, dpA);
    wait_all_loads();

    // Unit 2t (first query half of tile t) and unit 2t+1 (second half).  One synchronisation per
    // iteration, inside unit 2t: it certifies that tile t+1 is complete (first read right after it)
    // and that nobody reads tile t-1 any more, whose buffer the loads of tile t+3, issued during
    // unit 2t+1, overwrite.  A tile therefore has one and a half iterations to arrive.
    auto where_a = [&](int t) {  // unit 2t: previous = second half of tile t-1 (zero weights at t = 0)
        return Where{tilebuf(t), tilebuf(t), tilebuf(t - 1 < 0 ? 0 : t - 1), 1, 0, 1};
    };
    auto where_b = [&](int t) {  // unit 2t+1: next = first half of tile t+1
        return Where{tilebuf(t + 1), tilebuf(t), tilebuf(t), 0, 1, 0};
    };
    bf16x8 pre[LA];
    f32x4 l4pre;
    {
        const Where w0 = where_a(0);
#pragma unroll
        for (int i = 0; i < LA; ++i) pre[i] = frag(w0, i);
        l4pre = lse_rows(w0, 0);
    }
    for (int t = 0; t < ntiles; ++t) {
        const Where wa = where_a(t), wb = where_b(t), wa1 = where_a(t + 1);
        auto next_tile = [&](int j) { fetch(t + 3, j); };
        if (wave_active) {
            unit(std::true_type{}, wa, wb, sA, dpA, sB, dpB, pfB, dfB, pfA, dfA, pre, l4pre, [](int) {});
            unit(std::false_type{}, wb, wa1, sB, dpB, sA, dpA, pfA, dfA, pfB, dfB, pre, l4pre, next_tile);
        } else {
            tiles_landed_barrier(std::false_type{});
            fetch_tile(t + 3);
        }
    }

    if (wave_active) accumulate(tilebuf(ntiles - 1), 1, pfB, dfB);  // the last unit's contribution
    wait_all_loads();  // zero tiles requested past the end must have landed before LDS is reused
    __syncthreads();   // all tile reads are done: the buffers now stage the output rows
    if (!wave_active) return;
    char* region = smem + wave * RowStore<D>::BYTES;
    RowStore<D>::run(region, dka, scale, dk + head_off + (long)k0 * rs, rs, N - k0, lane);
    RowStore<D>::run(region, dva, 1.0f, dv + head_off + (long)k0 * rs, rs, N - k0, lane);
}

// Occupancy-oriented dK/dV kernel.  Same mathematics and layouts as avion_dkdv_kernel, but no
// software pipelining: each wavefront runs S / dP, the vector work and the dV^T / dK^T updates of
// one 32-query unit after the other, with two (Q | dO | scalars) buffers in LDS, so that more
// wavefronts fit a compute unit and cover each other's waits.  One workgroup barrier per 64-query
// tile: passing it certifies that the next tile has landed and that the previous one is no longer
// read, so its buffer can be refilled.
template <int D, int NW>
struct DkvOccCfg {
    static constexpr int BQ = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BNK = 32 * NW;
    using Ring = RowsAndScalarsRing<D, NW, 2>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    static constexpr int WAVES_PER_SIMD = 2;  // a floor for the register budget; D = 64 fits three
};

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64, (DkvOccCfg<D, NW>::WAVES_PER_SIMD))
avion_dkdv_occ_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                      const bf16* __restrict__ dO, const float* __restrict__ rowsc, bf16* __restrict__ dk,
                      bf16* __restrict__ dv, int H, int N, int nkb, int nblocks, float cs, float scale)
{
    using Cfg = DkvOccCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BQ = Cfg::BQ, BNK = Cfg::BNK, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16, CT = (D + 31) / 32;
    constexpr int OFF_G = Ring::OFF_B, OFF_ROW = Ring::OFF_SCALARS;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nkb, kb = logical % nkb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const long rs = (long)H * D;
    const long head_off = ((long)b * N * H + h) * D;
    const SliceView qh(q + head_off, rs, N, D);
    const int npad = (N + 63) & ~63;
    const int ntiles = (N + BQ - 1) / BQ;
    const int k0 = kb * BNK + wave * 32;  // first key of this wavefront
    const bool wave_active = k0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    const Ring ring(q + head_off, dO + head_off, qh.bytes, qh.row_bytes, rowsc + (long)bh * 2 * npad, npad, ntiles, smem,
                    wave, lane);
    ring.fetch_tile(0);

    // K and V fragments (B operands: lane = key) stay in registers
    bf16x8 kf[KS], vf[KS];
    {
        const int row = min(k0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(k + off + ks * 16);
            vf[ks] = *reinterpret_cast<const bf16x8*>(v + off + ks * 16);
        }
    }
    f32x16 dka[CT], dva[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        dka[ct] = f32x16_zero();
        dva[ct] = f32x16_zero();
    }
    wait_all_loads();
    Ring::template landed_barrier<false, 0>();  // tile 0 is in LDS

    for (int t = 0; t < ntiles; ++t) {
        ring.fetch_tile(t + 1);  // into the buffer of tile t-1, which nobody reads any more
        if (wave_active) {
            const char* buf = ring.buf(t);
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) {
                const float* rowv = reinterpret_cast<const float*>(buf + OFF_ROW) + 32 * hq + 4 * g;
                // dP starts from -delta of the accumulator rows' queries (broadcast LDS reads)
                f32x16 s, dp;
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(rowv + BQ + 8 * a4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dp[4 * a4 + e] = d4[e];
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 aq = nat_frag(buf, STRIDE, 32 * hq + l32, ks, g);
                    const bf16x8 ag = nat_frag(buf + OFF_G, STRIDE, 32 * hq + l32, ks, g);
                    s = mfma32(aq, kf[ks], ks == 0 ? f32x16_zero() : s);
                    dp = mfma32(ag, vf[ks], dp);
                }
                f32x4 l4[4];
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) l4[a4] = *reinterpret_cast<const f32x4*>(rowv + 8 * a4);
                // per query half (16 queries): transposed operands requested before the vector work
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    bf16x8 tg[CT], tq[CT];
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        tg[ct] = tr_frag(buf + OFF_G, STRIDE, tr_off, ct, 2 * hq + half);
                        tq[ct] = tr_frag(buf, STRIDE, tr_off, ct, 2 * hq + half);
                    }
                    u32x4 pf, df;
#pragma unroll
                    for (int e = 8 * half; e < 8 * half + 8; ++e) {
                        const float pe = fast_exp2(fmaf(s[e], cs, -l4[e / 4][e % 4]));
                        s[e] = pe;
                        dp[e] = pe * dp[e];
                        if (e % 2 == 1) {
                            pf[(e / 2) % 4] = pack_bf16(s[e - 1], s[e]);
                            df[(e / 2) % 4] = pack_bf16(dp[e - 1], dp[e]);
                        }
                    }
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        dva[ct] = mfma32(tg[ct], as_bf16x8(pf), dva[ct]);
                        dka[ct] = mfma32(tq[ct], as_bf16x8(df), dka[ct]);
                    }
                }
            }
        }
        Ring::template landed_barrier<false, 0>();  // tile t+1 has landed; tile t is no longer read
    }
    if (!wave_active) return;
    char* region = smem + wave * RowStore<D>::BYTES;
    RowStore<D>::run(region, dka, scale, dk + head_off + (long)k0 * rs, rs, N - k0, lane);
    RowStore<D>::run(region, dva, 1.0f, dv + head_off + (long)k0 * rs, rs, N - k0, lane);
}
