// Backward kernels.  P is rebuilt tile by tile from Q, K and the saved LSE, so no N x N matrix is
// read or written (Sec. 3, "Flash Attention": the weights stay implicit; Sec. 4.1: the attention
// activation memory disappears).  With s = scale*<q_i,k_j>, P = exp(s - LSE_i),
// delta_i = sum_c dO_ic O_ic:
//     dV = P^T dO ,  dP = dO V^T ,  dS = P o (dP - delta) ,  dQ = scale dS K ,  dK = scale dS^T Q.
//
// Two kernels, both free of atomics (results are bit-reproducible):
//   avion_dq_kernel   : query-stationary.  Also computes delta from O and dO and leaves it, with a
//                       rescaled copy of LSE, for the second kernel.  Same shape as the forward:
//                       S^T = K Q^T and dP^T = V dO^T land with lane = query, so LSE and delta are
//                       per-lane scalars and dS^T feeds dQ^T = K^T dS^T as a B operand straight
//                       from registers; K^T comes from the same LDS tile as K, through transposing
//                       LDS loads.
//   avion_dkdv_kernel : key-stationary.  S = Q K^T and dP = dO V^T land with lane = key, K and V
//                       stay in registers as B operands, and P, dS feed dV^T = dO^T P and
//                       dK^T = Q^T dS from registers; the Q and dO tiles in LDS are read both as
//                       rows and, through transposing LDS loads, as columns.
// Each kernel recomputes S and dP for itself (7 contractions per tile pair instead of the
// algorithmic 5); the extra two are not counted as useful work anywhere.
//
// Schedule (both kernels): as in the forward kernel, the per-wavefront code is kept simple and
// small in registers -- the contractions and the vector work of one 32 x 32 unit after the other --
// and several resident wavefronts per SIMD fill each other's waits.  Tiles stream through two LDS
// buffers filled by LDS-direct loads; one workgroup barrier per 64-row tile certifies that the next
// tile has landed and that the previous one is no longer read, so that its buffer can be refilled.
//
// Template parameters of both kernels: head dim D, wavefronts per workgroup NW, element format E
// (Bf16 or F16: contraction instruction and roundings), CAUSAL (query i sees keys 0..i: units that
// no (query, key) pair of a wavefront needs are skipped, units on the diagonal start their score
// accumulator from a mask of 0 / -1e30, whose weights come out as exactly 0).
#pragma once
#include "avion_common.h"

// --------------------------------------------------------------------------------------------- dQ
// One wavefront owns 32 queries (Q, dO as B-operand fragments, LSE and delta as per-lane scalars);
// the workgroup's NW wavefronts share (K | V) tiles of 64 keys.
template <int D, int NW>
struct DqCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * NW;
    using Ring = TileRing<D, NW, 2, false>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    static constexpr int WAVES_PER_SIMD = D == 64 ? 3 : 2;  // LDS would allow more; registers do not
};

// The work of one workgroup: query block qb of (batch, head) bh.
template <int D, int NW, typename E, bool CAUSAL>
DEVINL void avion_dq_body(char* smem, const raw16* __restrict__ q, const raw16* __restrict__ k,
                          const raw16* __restrict__ v, const raw16* __restrict__ o, const raw16* __restrict__ dO,
                          const float* __restrict__ lse, raw16* __restrict__ dq, float* __restrict__ rowsc, int H, int N,
                          int rs_qkv, int rs_o, int bh, int qb, float cs, float scale)
{
    using Cfg = DqCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16, CT = (D + 31) / 32;

    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    // token rows of Q, K, V, dQ are rs_qkv elements apart, those of O, dO rs_o
    const long rs = rs_qkv;
    const long head_off = (long)b * N * rs + (long)h * D;
    const long head_off_o = (long)b * N * rs_o + (long)h * D;
    const int q0 = qb * BM + wave * 32;
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    // keys seen by this lane's query, by any query of the wavefront, by all of them (see the forward)
    const int key_limit = CAUSAL ? min(N, q0 + l32 + 1) : N;
    const int wave_key_end = CAUSAL ? min(N, q0 + 32) : N;
    const int mask_from = CAUSAL ? min(N, q0 + 1) : N;
    const int ntiles = ((CAUSAL ? min(N, qb * BM + BM) : N) + BN - 1) / BN;

    const Ring ring(k + head_off, rs, v + head_off, rs, N, nullptr, 0, ntiles, smem, wave, lane);
    ring.fetch(0);

    // Q and dO fragments (B operands), delta and LSE per lane
    frag8 qf[KS], gf[KS];
    float lc, dl;
    {
        const int row = min(q0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
        const long off_o = head_off_o + (long)row * rs_o + g * 8;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *reinterpret_cast<const frag8*>(q + off + ks * 16);
            gf[ks] = *reinterpret_cast<const frag8*>(dO + off_o + ks * 16);
            const frag8 of = *reinterpret_cast<const frag8*>(o + off_o + ks * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf(E::widen(of, e), E::widen(gf[ks], e), part);
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

    Ring::landed_barrier();  // tile 0 is in LDS (and the fragments above have arrived)

    // one 32-key unit: rows 32*hk.. of the tile pair; RAGGED units reach past the last key and
    // start the score accumulator from the key mask instead of zero
    auto unit = [&](auto ragged, const char* kt, const char* vt, int hk, int key_base) {
        constexpr bool RAGGED = decltype(ragged)::value;
        f32x16 s, dp;
        if constexpr (RAGGED) s = key_mask_block(key_base, g, key_limit);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const frag8 ak = nat_frag(kt, STRIDE, 32 * hk + l32, ks, g);
            const frag8 av = nat_frag(vt, STRIDE, 32 * hk + l32, ks, g);
            s = E::mfma(ak, qf[ks], ks == 0 && !RAGGED ? f32x16_zero() : s);
            dp = E::mfma(av, gf[ks], ks == 0 ? f32x16_zero() : dp);
        }
        // the K^T operands are requested before the vector work so that they are there after it
        frag8 kt_f[2][CT];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) kt_f[half][ct] = tr_frag(kt, STRIDE, tr_off, ct, 2 * hk + half);
        u32x4 df[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pe = fast_exp2(fmaf(s[i], cs, nlc));
            s[i] = pe * (dp[i] - dl);
            if (i % 2 == 1) df[i / 8][(i / 2) % 4] = E::pack(s[i - 1], s[i]);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[ct] = E::mfma(kt_f[half][ct], as_frag8(df[half]), acc[ct]);
    };

    for (int t = 0; t < ntiles; ++t) {
        ring.fetch(t + 1);  // into the buffer of tile t-1, which nobody reads any more
        if (wave_active) {
#pragma unroll
            for (int hk = 0; hk < 2; ++hk) {
                const int key_base = t * BN + 32 * hk;
                if (key_base >= wave_key_end) continue;  // past the last key, or (causal) seen by no query of this wavefront
                if (key_base + 32 > mask_from) unit(std::true_type{}, ring.buf(t), ring.buf(t) + Ring::OFF_B, hk, key_base);
                else unit(std::false_type{}, ring.buf(t), ring.buf(t) + Ring::OFF_B, hk, key_base);
            }
        }
        Ring::landed_barrier();  // tile t+1 has landed; tile t is no longer read
    }
    if (!wave_active) return;
    RowStore<D, E>::run(smem + wave * RowStore<D, E>::BYTES, acc, scale, dq + head_off + (long)q0 * rs, rs, N - q0, lane);
}

template <int D, int NW, typename E, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64, (DqCfg<D, NW>::WAVES_PER_SIMD))
avion_dq_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                    const raw16* __restrict__ o, const raw16* __restrict__ dO, const float* __restrict__ lse,
                    raw16* __restrict__ dq, float* __restrict__ rowsc, int H, int N, int rs_qkv, int rs_o, int nqb,
                    int nblocks, float cs, float scale)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    avion_dq_body<D, NW, E, CAUSAL>(smem, q, k, v, o, dO, lse, dq, rowsc, H, N, rs_qkv, rs_o, logical / nqb, logical % nqb,
                                    cs, scale);
}

// ------------------------------------------------------------------------------------------ dK, dV
// One wavefront owns 32 keys (K, V as B-operand fragments); the workgroup's NW wavefronts share
// (Q | dO | per-query scalars) tiles of 64 queries.  The dP accumulator starts from -delta, so the
// subtraction in dS costs no vector-ALU instruction.
template <int D, int NW>
struct DkvCfg {
    static constexpr int BQ = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BNK = 32 * NW;
    using Ring = TileRing<D, NW, 2, true>;
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    // resident wavefronts per SIMD the register budget is held to: three for D = 64 (at most 168
    // registers; the schedule relies on three wavefronts filling each other's waits), two for D = 80
    static constexpr int WAVES_PER_SIMD = D == 64 ? 3 : 2;
};

// The work of one workgroup: key block kb of (batch, head) bh.
template <int D, int NW, typename E, bool CAUSAL>
DEVINL void avion_dkdv_body(char* smem, const raw16* __restrict__ q, const raw16* __restrict__ k,
                            const raw16* __restrict__ v, const raw16* __restrict__ dO, const float* __restrict__ rowsc,
                            raw16* __restrict__ dk, raw16* __restrict__ dv, int H, int N, int rs_qkv, int rs_o, int bh,
                            int kb, float cs, float scale)
{
    using Cfg = DkvCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BQ = Cfg::BQ, BNK = Cfg::BNK, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16, CT = (D + 31) / 32;
    constexpr int OFF_G = Ring::OFF_B, OFF_ROW = Ring::OFF_SCALARS;

    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    // token rows of Q, K, V, dK, dV are rs_qkv elements apart, those of dO rs_o
    const long rs = rs_qkv;
    const long head_off = (long)b * N * rs + (long)h * D;
    const long head_off_o = (long)b * N * rs_o + (long)h * D;
    const int npad = (N + 63) & ~63;
    const int ntiles = (N + BQ - 1) / BQ;
    const int k0 = kb * BNK + wave * 32;  // first key of this wavefront
    const bool wave_active = k0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);

    // causal attention: the keys of this workgroup are seen by the queries from its first key on only,
    // so the stream of query tiles starts there
    const int t0 = CAUSAL ? kb * BNK / BQ : 0;

    const Ring ring(q + head_off, rs, dO + head_off_o, rs_o, N, rowsc + (long)bh * 2 * npad, npad, ntiles, smem, wave,
                    lane);
    ring.fetch(t0);

    // K and V fragments (B operands: lane = key) stay in registers
    frag8 kf[KS], vf[KS];
    {
        const int row = min(k0 + l32, N - 1);
        const long off = head_off + (long)row * rs + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = *reinterpret_cast<const frag8*>(k + off + ks * 16);
            vf[ks] = *reinterpret_cast<const frag8*>(v + off + ks * 16);
        }
    }
    f32x16 dka[CT], dva[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        dka[ct] = f32x16_zero();
        dva[ct] = f32x16_zero();
    }
    Ring::landed_barrier();  // the first tile is in LDS (and the fragments above have arrived)

    for (int t = t0; t < ntiles; ++t) {
        ring.fetch(t + 1);  // into the buffer of tile t-1, which nobody reads any more
        if (wave_active) {
            const char* buf = ring.buf(t);
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) {
                const int query_base = t * BQ + 32 * hq;
                // causal: units whose queries all lie before this wavefront's keys contribute nothing;
                // units that straddle the diagonal start their scores from the mask
                if (query_base >= N) continue;  // past the last query
                if (CAUSAL && query_base + 32 <= k0) continue;
                const float* rowv = reinterpret_cast<const float*>(buf + OFF_ROW) + 32 * hq + 4 * g;
                // dP starts from -delta of the accumulator rows' queries (broadcast LDS reads)
                f32x16 s, dp;
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(rowv + BQ + 8 * a4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dp[4 * a4 + e] = d4[e];
                }
                if constexpr (CAUSAL) {
                    if (query_base < k0 + 31) s = query_mask_block(query_base, g, k0 + l32);
                    else s = f32x16_zero();
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const frag8 aq = nat_frag(buf, STRIDE, 32 * hq + l32, ks, g);
                    const frag8 ag = nat_frag(buf + OFF_G, STRIDE, 32 * hq + l32, ks, g);
                    s = E::mfma(aq, kf[ks], ks == 0 && !CAUSAL ? f32x16_zero() : s);
                    dp = E::mfma(ag, vf[ks], dp);
                }
                f32x4 l4[4];
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) l4[a4] = *reinterpret_cast<const f32x4*>(rowv + 8 * a4);
                // per query half (16 queries): transposed operands requested before the vector work
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    frag8 tg[CT], tq[CT];
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
                            pf[(e / 2) % 4] = E::pack(s[e - 1], s[e]);
                            df[(e / 2) % 4] = E::pack(dp[e - 1], dp[e]);
                        }
                    }
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        dva[ct] = E::mfma(tg[ct], as_frag8(pf), dva[ct]);
                        dka[ct] = E::mfma(tq[ct], as_frag8(df), dka[ct]);
                    }
                }
            }
        }
        Ring::landed_barrier();  // tile t+1 has landed; tile t is no longer read
    }
    if (!wave_active) return;
    char* region = smem + wave * RowStore<D, E>::BYTES;
    const int lane_now = lane_from_exec();
    RowStore<D, E>::run(region, dka, scale, dk + head_off + (long)k0 * rs, rs, N - k0, lane_now);
    RowStore<D, E>::run(region, dva, 1.0f, dv + head_off + (long)k0 * rs, rs, N - k0, lane_now);
}

template <int D, int NW, typename E, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64, (DkvCfg<D, NW>::WAVES_PER_SIMD))
avion_dkdv_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                      const raw16* __restrict__ dO, const float* __restrict__ rowsc, raw16* __restrict__ dk,
                      raw16* __restrict__ dv, int H, int N, int rs_qkv, int rs_o, int nkb, int nblocks, float cs,
                      float scale)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    avion_dkdv_body<D, NW, E, CAUSAL>(smem, q, k, v, dO, rowsc, dk, dv, H, N, rs_qkv, rs_o, logical / nkb, logical % nkb, cs,
                                      scale);
}

// ------------------------------------------------------------------------- whole backward, short sequences
// For N <= 32*NW one workgroup covers all queries and all keys of a (batch, head): the two passes
// then run back to back inside one workgroup, so that the second pass finds Q, K, V and dO in the
// L2 where the first one has just pulled them (launched separately it would fetch them from HBM
// again), and one launch is saved.  Same arithmetic, same bits as the two kernels.  The per-query
// scalars still travel through the workspace: a workgroup-scope fence makes the first pass's stores visible
// before the second pass's tile mover reads them, the barrier also frees the LDS the first pass
// used for its epilogue.
template <int D, int NW>
struct BwdSmallCfg {
    static constexpr int NT = NW * 64;
    static constexpr int MAX_N = 32 * NW;
    static constexpr int LDS_BYTES =
        DqCfg<D, NW>::LDS_BYTES > DkvCfg<D, NW>::LDS_BYTES ? DqCfg<D, NW>::LDS_BYTES : DkvCfg<D, NW>::LDS_BYTES;
};

template <int D, int NW, typename E, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64, (DkvCfg<D, NW>::WAVES_PER_SIMD))
avion_bwd_small_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                       const raw16* __restrict__ o, const raw16* __restrict__ dO, const float* __restrict__ lse,
                       raw16* __restrict__ dq, raw16* __restrict__ dk, raw16* __restrict__ dv, float* __restrict__ rowsc,
                       int H, int N, int rs_qkv, int rs_o, int nblocks, float cs, float scale)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int bh = xcd_local_id(blockIdx.x, nblocks);
    if (bh < 0) return;
    avion_dq_body<D, NW, E, CAUSAL>(smem, q, k, v, o, dO, lse, dq, rowsc, H, N, rs_qkv, rs_o, bh, 0, cs, scale);
    // Workgroup scope is enough (writer and reader wavefronts sit on one compute unit and share its
    // vector cache) and is only a wait for the stores; a device-scope fence would write back and
    // invalidate the L2 once per workgroup.
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __syncthreads();
    avion_dkdv_body<D, NW, E, CAUSAL>(smem, q, k, v, dO, rowsc, dk, dv, H, N, rs_qkv, rs_o, bh, 0, cs, scale);
}
