// Forward kernel: O = softmax(scale * Q K^T) V and LSE, one pass over the keys, nothing N x N stored
// (Sec. 3, "Flash Attention": implicit softmax weights, block-wise work out of on-chip memory;
// Sec. 1: block results combined into the exact output).
//
// Work split: one workgroup = NW wavefronts = 32*NW consecutive queries of one (batch, head).
// Each wavefront owns 32 queries and keeps
//   Q as MFMA B-operand fragments (lane = query, 8 channels per 16-deep step),
//   O^T accumulators (lane = query, registers = channels), the reference maximum and row sums.
// Keys and values come in LDS tiles of 64 tokens in their natural row layout, two (K | V) buffers,
// filled straight from global memory by LDS-direct loads (no staging registers, no LDS writes):
// K rows are the A operand of S^T = K Q^T, and V is read through transposing LDS loads as the A
// operand of O^T = V^T P^T.  Computing the transposed products keeps every score of a query inside
// one lane pair, so the accumulator of the first contraction is, after rounding to the element
// format E (bf16 or fp16), directly the B operand of the second one (no LDS round trip).
//
// Schedule.  A wavefront issues in order, and an MFMA queued behind another one blocks what
// follows it, so a single wavefront cannot keep the matrix cores and the vector ALUs busy at once.
// The kernel therefore keeps the per-wavefront code simple and small in registers -- S^T, softmax,
// P V of one 32-key unit after the other -- and relies on several resident wavefronts per SIMD
// (four for d = 64) to fill each other's waits.  One workgroup barrier per 64-key tile: passing it
// certifies that the next tile has landed and that the previous one is no longer read, so that its
// buffer can be refilled.
//
// Softmax reference.  Weights are exp2(cs*s - m) with m fixed per query to the maximum over the
// first 32 keys.  Softmax is invariant to m, floating point keeps its relative precision at any
// magnitude, and the final division by the row sum cancels m exactly; the only failure mode is
// overflow when a later score exceeds m by ~100 binades (bf16; ~15 binades for fp16, whose weights
// must stay below 65504).  That is detected from the final row sum against E::kRowSumLimit
// (workgroup-wide), and the whole workgroup then recomputes its rows with the classic running
// maximum (avion_fwd_safe_pass).  Random or trained activations never get there.
//
// Template parameters: head dim D, wavefronts per workgroup NW, element format E (Bf16 or F16),
// CAUSAL (query i sees keys 0..i; the reference m is then the maximum over the visible ones of the
// first 32 keys -- key 0 is visible to every query).
#pragma once
#include "avion_common.h"

template <int D, int NW>
struct FwdCfg {
    static constexpr int BN = 64;
    static constexpr int NT = NW * 64;
    static constexpr int BM = 32 * NW;
    using Ring = TileRing<D, NW, 2, false>;
    using Stage = TileStage<D, BN, NT>;  // the fallback pass stages its tiles through registers
    static_assert(Ring::TILE_BYTES == Stage::BYTES, "both movers use the same tile layout");
    static constexpr int LDS_BYTES = Ring::LDS_BYTES;
    // wavefronts per SIMD the register budget is sized for: what LDS lets a compute unit hold, at most 4
    static constexpr int WG_PER_CU = 160 * 1024 / LDS_BYTES;
    static constexpr int WAVES_PER_SIMD = WG_PER_CU * NW / 4 > 4 ? 4 : WG_PER_CU * NW / 4;
};

// Classic online softmax with a running maximum, one 64-key tile at a time, staged through
// registers into the ring's two buffers.  Used only as the fallback described above; same register
// layouts as the main loop.
// key_limit: this lane's query sees keys below it (N, or query + 1 for causal attention).
template <int D, int NW, typename E>
DEVINL void avion_fwd_safe_pass(char* smem, const SliceView& kh, const SliceView& vh, const frag8 (&qf)[D / 16],
                                f32x16 (&oacc)[(D + 31) / 32], float& m_used, float& lsum, float& rsum, int N,
                                int key_limit, float cs, bool wave_active, int tid, int l32, int g, int tr_off)
{
    using Cfg = FwdCfg<D, NW>;
    using Stage = typename Cfg::Stage;
    using Ring = typename Cfg::Ring;
    constexpr int BN = 64, STRIDE = Stage::STRIDE, KS = D / 16, CT = (D + 31) / 32;
    auto kbuf = [&](int i) { return smem + i * Ring::BUF_BYTES; };
    auto vbuf = [&](int i) { return smem + i * Ring::BUF_BYTES + Ring::OFF_B; };
    m_used = -INFINITY;
    lsum = 0.f;
    rsum = 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) oacc[ct] = f32x16_zero();
    Stage kst, vst;
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
                f32x16 s;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    s = E::mfma(nat_frag(kc, STRIDE, 32 * kt + l32, ks, g), qf[ks], ks == 0 ? f32x16_zero() : s);
                const int key0 = t * BN + 32 * kt + 4 * g;
                if (key0 + 28 >= key_limit) {
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (key0 + 8 * (i / 4) + (i % 4) >= key_limit) s[i] = -INFINITY;
                }
                const float m2 = both_halves_max(max16(s)) * cs;
                const float mn = fmaxf(m_used, m2);  // finite: key 0 is seen by every query
                const float alpha = fast_exp2(m_used - mn);
                m_used = mn;
                lsum *= alpha;
                rsum *= alpha;
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
                float rowsum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = fast_exp2(fmaf(s[i], cs, -mn));
                    s[i] = p;
                    rowsum += p;
                }
                lsum += rowsum;
                const frag8 pf0 = acc_to_frag<E>(s, 0), pf1 = acc_to_frag<E>(s, 1);
                rsum = frag_sum<E>(pf1, frag_sum<E>(pf0, rsum));
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
                        oacc[ct] = E::mfma(tr_frag(vc, STRIDE, tr_off, ct, 2 * kt + half), half == 0 ? pf0 : pf1, oacc[ct]);
            }
        }
        if (more) {
            kst.store(kbuf((t + 1) & 1), tid);
            vst.store(vbuf((t + 1) & 1), tid);
        }
        __syncthreads();
    }
}

// (The causal instance carries a per-lane key bound and a few more scalars: it is sized for one
// wavefront per SIMD less than the register file would otherwise hold, which keeps it free of spills.)
template <int D, int NW, typename E, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64, (FwdCfg<D, NW>::WAVES_PER_SIMD - (CAUSAL && FwdCfg<D, NW>::WAVES_PER_SIMD > 3 ? 1 : 0)))
avion_fwd_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                 raw16* __restrict__ o, float* __restrict__ lse, int H, int N, int rs_qkv, int rs_o, int nqb, int nblocks,
                 float cs)
{
    using Cfg = FwdCfg<D, NW>;
    using Ring = typename Cfg::Ring;
    constexpr int BN = Cfg::BN, BM = Cfg::BM, STRIDE = Ring::STRIDE;
    constexpr int KS = D / 16;         // 16-deep steps over the channels
    constexpr int CT = (D + 31) / 32;  // 32-channel tiles of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int logical = xcd_local_id(blockIdx.x, nblocks);
    if (logical < 0) return;
    const int bh = logical / nqb, qb = logical % nqb;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    // token rows of Q, K, V are rs_qkv elements apart, those of O rs_o; a batch entry is N such rows
    const long rs = rs_qkv;
    const long head_off = (long)b * N * rs + (long)h * D;
    const long head_off_o = (long)b * N * rs_o + (long)h * D;
    const SliceView kh(k + head_off, rs, N, D);
    const SliceView vh(v + head_off, rs, N, D);
    const int q0 = qb * BM + wave * 32;  // first query of this wavefront
    const bool wave_active = q0 < N;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    // Keys this lane's query sees: all N, or 0..query for causal attention.  For the whole wavefront:
    // units that start at or beyond wave_key_end are skipped, units that reach beyond mask_from start
    // their scores from the mask; the workgroup streams the tiles up to its last query only.
    const int key_limit = CAUSAL ? min(N, q0 + l32 + 1) : N;
    const int wave_key_end = CAUSAL ? min(N, q0 + 32) : N;
    const int mask_from = CAUSAL ? min(N, q0 + 1) : N;
    const int ntiles = ((CAUSAL ? min(N, qb * BM + BM) : N) + BN - 1) / BN;

    const Ring ring(k + head_off, rs, v + head_off, rs, N, nullptr, 0, ntiles, smem, wave, lane);
    ring.fetch(0);

    // Q fragments stay in registers for the whole kernel
    frag8 qf[KS];
    {
        const int row = min(q0 + l32, N - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = *reinterpret_cast<const frag8*>(q + head_off + (long)row * rs + ks * 16 + g * 8);
    }
    f32x16 oacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) oacc[ct] = f32x16_zero();
    float m_used = 0.f, lsum = 0.f, rsum = 0.f;

    Ring::landed_barrier();  // tile 0 is in LDS (and the Q fragments have arrived)

    // S^T of one unit (32 keys starting at row 32*hk of the K tile); RAGGED units reach past the
    // last key and start from the key mask instead of zero
    auto scores = [&](auto ragged, const char* kt, int hk, int key_base) -> f32x16 {
        constexpr bool RAGGED = decltype(ragged)::value;
        f32x16 s;
        if constexpr (RAGGED) s = key_mask_block(key_base, g, key_limit);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            s = E::mfma(nat_frag(kt, STRIDE, 32 * hk + l32, ks, g), qf[ks], ks == 0 && !RAGGED ? f32x16_zero() : s);
        return s;
    };
    // reference maximum: over the first 32 keys
    if (wave_active) m_used = both_halves_max(max16(scores(std::true_type{}, ring.buf(0), 0, 0))) * cs;

    for (int t = 0; t < ntiles; ++t) {
        ring.fetch(t + 1);  // into the buffer of tile t-1, which nobody reads any more
        if (wave_active) {
            const char* kt = ring.buf(t);
            const char* vt = kt + Ring::OFF_B;
#pragma unroll
            for (int hk = 0; hk < 2; ++hk) {
                const int key_base = t * BN + 32 * hk;
                if (key_base >= wave_key_end) continue;  // past the last key, or (causal) seen by no query of this wavefront
                f32x16 s;
                if (key_base + 32 > mask_from) s = scores(std::true_type{}, kt, hk, key_base);
                else s = scores(std::false_type{}, kt, hk, key_base);
                // the V^T operands are requested before the vector work so that they are there after it
                frag8 vf[2][CT];
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) vf[half][ct] = tr_frag(vt, STRIDE, tr_off, ct, 2 * hk + half);
                u32x4 pf[2];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = fast_exp2(fmaf(s[i], cs, -m_used));
                    s[i] = p;
                    lsum += p;
                    if (i % 2 == 1) {
                        // the second row sum runs over the weights as rounded to the element format, i.e. the
                        // numbers the second contraction multiplies V with; O is divided by it
                        const unsigned wgt = E::pack(s[i - 1], p);
                        pf[i / 8][(i / 2) % 4] = wgt;
                        rsum = E::add_pair(wgt, rsum);
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) oacc[ct] = E::mfma(vf[half][ct], as_frag8(pf[half]), oacc[ct]);
            }
        }
        Ring::landed_barrier();  // tile t+1 has landed; tile t is no longer read
    }

    // overflow of the fixed reference: redo this workgroup's rows with the running maximum
    bool bad = false;
    if (wave_active) bad = !(both_halves_sum(lsum) <= E::kRowSumLimit);
    if (__syncthreads_or(bad ? 1 : 0))
        avion_fwd_safe_pass<D, NW, E>(smem, kh, vh, qf, oacc, m_used, lsum, rsum, N, key_limit, cs, wave_active, tid, l32, g,
                                      tr_off);

    // every wavefront is past its last tile read (barrier above): the tile buffers are free and
    // serve as the per-wavefront staging area of the output rows
    if (!wave_active) return;
    const float l = both_halves_sum(lsum);
    const float inv = 1.0f / both_halves_sum(rsum);
    // each lane scales by its own query's divisor before the rows are transposed
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][i] *= inv;
    RowStore<D, E>::run(smem + wave * RowStore<D, E>::BYTES, oacc, 1.0f, o + head_off_o + (long)q0 * rs_o, rs_o, N - q0, lane_from_exec());
    if (g == 0 && q0 + l32 < N) lse[(long)bh * N + q0 + l32] = (m_used + __builtin_amdgcn_logf(l)) * kLn2;
}
