// Many tiny problems per launch: sequences of at most 32 tokens (Sec. 4.1 compares the plain ViT with a
// divided space/time attention, whose temporal attention runs over N = T = 4..16 frames for every
// spatial position; the text encoder's shortest captions are of this size too).  One (batch, head)
// problem per workgroup would leave almost every lane idle and every load waiting, so here
//
//   * one WAVEFRONT handles a window of 32 consecutive token rows of one head, i.e. G = floor(32 / N)
//     whole problems at once: in the [B, N, H, d] layout the tokens of consecutive batch entries follow
//     each other, so the window is simply rows b0*N .. b0*N + G*N - 1 of the [B*N, H, d] view;
//   * the window is computed as ONE 32 x 32 attention whose score matrix is masked block-diagonally
//     (a query sees the keys of its own problem only; with CAUSAL, only those at or before it).  The
//     masked entries get weight exactly 0, so the problems do not see each other;
//   * the whole window lives in one wavefront -- no workgroup barriers, no cross-wavefront sums.  The
//     backward therefore is truly one pass: S and dP are formed in both orientations (lane = query for
//     dQ, lane = key for dK and dV) from the same register fragments, nothing is exchanged or recomputed
//     from memory, and no workspace is used.  The regime is bound by memory bandwidth (arithmetic
//     intensity N/2 flops per byte), so the doubled contractions cost nothing that matters;
//   * wavefronts walk the windows with a stride and keep the next window's loads in flight while they
//     compute (forward), so that enough bytes are outstanding to cover the memory latency.
//
// Register/LDS layouts and fragment conventions are those of avion_common.h.  Operands whose
// contraction index is a token (V^T, K^T, Q^T, dO^T) are read with transposing LDS loads from a
// per-wavefront tile; everything else goes from global memory straight into MFMA fragments.
// The softmax reference is the exact row maximum (all of a query's keys are in the one unit), so no
// overflow path is needed.
#pragma once
#include "avion_common.h"

template <int D>
struct WinCfg {
    static constexpr int NW = D == 64 ? 4 : 2;  // wavefronts per workgroup (independent of each other)
    static constexpr int NT = NW * 64;
    static constexpr int STRIDE = tile_stride<D>();
    static constexpr int TILE = 32 * STRIDE;  // one 32-row tile
    static constexpr int KS = D / 16, CT = (D + 31) / 32;
    static constexpr int STAGE = 32 * (D * 2 + 16);                  // RowStore's staging area of one wavefront
    static constexpr int FWD_WAVE_BYTES = TILE + STAGE;              // V tile | row-store staging
    static constexpr int BWD_WAVE_BYTES = 3 * TILE + 256 + STAGE;    // Q, K, dO tiles | per-query scalars | staging
    static constexpr int FWD_LDS_BYTES = NW * FWD_WAVE_BYTES;
    static constexpr int BWD_LDS_BYTES = NW * BWD_WAVE_BYTES;
};

// A 32-row window of one tensor and one head as natural MFMA fragments: lane holds row l32, channels
// 16*ks + 8*g .. +7.  Rows at or beyond rows_valid are zeros.
template <int D>
struct RowFrags {
    frag8 f[D / 16];
    DEVINL void load(const raw16* first_row, long rs, int rows_valid, int l32, int g)
    {
        const frag8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            f[ks] = l32 < rows_valid ? *reinterpret_cast<const frag8*>(first_row + (long)l32 * rs + ks * 16 + g * 8) : zero;
    }
    // into a padded LDS tile (row stride tile_stride<D>()); the pad is not written
    DEVINL void to_tile(char* tile, int l32, int g) const
    {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            *reinterpret_cast<frag8*>(tile + l32 * tile_stride<D>() + ks * 32 + g * 16) = f[ks];
    }
};

// the pads of a wavefront's tiles read as zeros (D = 80 reads them as channels 80..95)
template <int D>
DEVINL void win_zero_pads(char* tiles, int ntiles, int lane)
{
    constexpr int STRIDE = tile_stride<D>(), PADW = (STRIDE - D * 2) / 4;
    for (int i = lane; i < ntiles * 32 * PADW; i += 64)
        *reinterpret_cast<unsigned*>(tiles + (i / PADW) * STRIDE + D * 2 + (i % PADW) * 4) = 0u;
}

// Which of the 16 accumulator rows 8*(i/4) + 4*g + i%4 (bit i) this lane's column may be combined
// with: same problem (row / N == col / N) and, for causal attention, key at or before query.
// lane_is_query: the lane's column is a query and the rows are keys (transposed scores), else the
// lane is a key and the rows are queries.
template <bool CAUSAL>
DEVINL unsigned win_allow_bits(int l32, int g, int N, bool lane_is_query)
{
    unsigned bits = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i / 4) + 4 * g + (i % 4);
        bool ok = row / N == l32 / N;
        if (CAUSAL) ok = ok && (lane_is_query ? row % N <= l32 % N : l32 % N <= row % N);
        bits |= ok ? 1u << i : 0u;
    }
    return bits;
}

DEVINL void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// --------------------------------------------------------------------------------------- forward
template <int D, typename E, bool CAUSAL>
__global__ void __launch_bounds__(WinCfg<D>::NT, 2)
avion_win_fwd_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                     raw16* __restrict__ o, float* __restrict__ lse, int B, int H, int N, int rs_qkv, int rs_o, int G,
                     int nitems, float cs)
{
    using Cfg = WinCfg<D>;
    constexpr int STRIDE = Cfg::STRIDE, KS = Cfg::KS, CT = Cfg::CT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    char* vtile = smem + wave * Cfg::FWD_WAVE_BYTES;
    char* stage = vtile + Cfg::TILE;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    const unsigned allow = win_allow_bits<CAUSAL>(l32, g, N, true);
    const long rs = rs_qkv;
    if constexpr (D % 32 != 0) win_zero_pads<D>(vtile, 1, lane);

    struct Window {
        RowFrags<D> q, k, v;
        int item;
    };
    // first row, head and number of valid rows of a window
    auto place = [&](int item, long& row0, int& h, int& rows_valid) {
        const int win = item / H;
        h = item % H;
        const int b0 = win * G;
        row0 = (long)b0 * N;
        rows_valid = min(G, B - b0) * N;
    };
    auto fetch = [&](Window& w, int item) {
        long row0;
        int h, rows_valid;
        place(item, row0, h, rows_valid);
        w.item = item;
        const long off = row0 * rs + (long)h * D;
        w.q.load(q + off, rs, rows_valid, l32, g);
        w.k.load(k + off, rs, rows_valid, l32, g);
        w.v.load(v + off, rs, rows_valid, l32, g);
    };
    auto compute = [&](const Window& w) {
        long row0;
        int h, rows_valid;
        place(w.item, row0, h, rows_valid);
        w.v.to_tile(vtile, l32, g);  // the previous window's reads of this tile are complete (same wavefront, in order)
        // S^T = K Q^T: lane = query, registers = keys
        f32x16 s;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s = E::mfma(w.k.f[ks], w.q.f[ks], ks == 0 ? f32x16_zero() : s);
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = (allow >> i) & 1u ? s[i] : -INFINITY;
        const float m = both_halves_max(max16(s)) * cs;  // finite: a query always sees itself
        float lsum = 0.f, rsum = 0.f;
        u32x4 pf[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = fast_exp2(fmaf(s[i], cs, -m));  // masked: exp2(-inf) = 0 exactly
            s[i] = p;
            lsum += p;
            if (i % 2 == 1) {
                const unsigned wgt = E::pack(s[i - 1], p);
                pf[i / 8][(i / 2) % 4] = wgt;
                rsum = E::add_pair(wgt, rsum);  // O is divided by the sum of the weights as rounded (see avion_fwd.h)
            }
        }
        wave_sync_lds();
        // O^T = V^T P^T
        f32x16 oacc[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) oacc[ct] = f32x16_zero();
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                oacc[ct] = E::mfma(tr_frag(vtile, STRIDE, tr_off, ct, half), as_frag8(pf[half]), oacc[ct]);
        const float l = both_halves_sum(lsum);
        const float inv = 1.0f / both_halves_sum(rsum);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[ct][i] *= inv;
        RowStore<D, E>::run(stage, oacc, 1.0f, o + row0 * rs_o + (long)h * D, rs_o, rows_valid, lane);
        if (g == 0 && l32 < rows_valid) {
            const long b = row0 / N + l32 / N;
            lse[(b * H + h) * N + l32 % N] = (m + __builtin_amdgcn_logf(l)) * kLn2;
        }
    };

    // two windows in registers: the next one is being fetched while the current one is computed
    const int stride = gridDim.x * Cfg::NW;
    int item = blockIdx.x * Cfg::NW + wave;
    if (item >= nitems) return;
    Window a, b;
    fetch(a, item);
    while (true) {
        const int n1 = item + stride;
        if (n1 < nitems) fetch(b, n1);
        compute(a);
        if (n1 >= nitems) break;
        const int n2 = n1 + stride;
        if (n2 < nitems) fetch(a, n2);
        compute(b);
        if (n2 >= nitems) break;
        item = n2;
    }
}

// -------------------------------------------------------------------------------------- backward
// delta_i = sum_c dO_ic O_ic; P = exp(s - LSE); dV = P^T dO; dS = P o (dO V^T - delta);
// dQ = scale dS K; dK = scale dS^T Q -- all of it for one window inside one wavefront.
template <int D, typename E, bool CAUSAL>
__global__ void __launch_bounds__(WinCfg<D>::NT, 2)
avion_win_bwd_kernel(const raw16* __restrict__ q, const raw16* __restrict__ k, const raw16* __restrict__ v,
                     const raw16* __restrict__ o, const raw16* __restrict__ dO, const float* __restrict__ lse,
                     raw16* __restrict__ dq, raw16* __restrict__ dk, raw16* __restrict__ dv, int B, int H, int N, int rs_qkv,
                     int rs_o, int G, int nitems, float cs, float scale)
{
    using Cfg = WinCfg<D>;
    constexpr int STRIDE = Cfg::STRIDE, KS = Cfg::KS, CT = Cfg::CT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, g = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    char* qtile = smem + wave * Cfg::BWD_WAVE_BYTES;
    char* ktile = qtile + Cfg::TILE;
    char* gtile = ktile + Cfg::TILE;
    float* rowsc = reinterpret_cast<float*>(gtile + Cfg::TILE);  // [0..31] LSE*log2e, [32..63] -delta, per query row
    char* stage = reinterpret_cast<char*>(rowsc) + 256;
    const int tr_off = tr_lane_offset(lane, STRIDE);
    const unsigned allow_t = win_allow_bits<CAUSAL>(l32, g, N, true);   // lane = query, rows = keys
    const unsigned allow_n = win_allow_bits<CAUSAL>(l32, g, N, false);  // lane = key, rows = queries
    const long rs = rs_qkv;
    if constexpr (D % 32 != 0) win_zero_pads<D>(qtile, 3, lane);

    for (int item = blockIdx.x * Cfg::NW + wave; item < nitems; item += gridDim.x * Cfg::NW) {
        const int win = item / H, h = item % H, b0 = win * G;
        const long row0 = (long)b0 * N;
        const int rows_valid = min(G, B - b0) * N;
        const long off = row0 * rs + (long)h * D, off_o = row0 * rs_o + (long)h * D;
        RowFrags<D> qf, kf, vf, gf, of;
        qf.load(q + off, rs, rows_valid, l32, g);
        kf.load(k + off, rs, rows_valid, l32, g);
        vf.load(v + off, rs, rows_valid, l32, g);
        gf.load(dO + off_o, rs_o, rows_valid, l32, g);
        of.load(o + off_o, rs_o, rows_valid, l32, g);
        // per-query scalars; rows past the end get LSE = +inf (weight 0) and delta = 0
        float lc = INFINITY;
        if (l32 < rows_valid) lc = lse[((row0 / N + l32 / N) * H + h) * N + l32 % N] * kLog2e;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf(E::widen(of.f[ks], e), E::widen(gf.f[ks], e), part);
        const float dl = both_halves_sum(part);
        // tiles for the transposed operands, scalars for the key-stationary orientation
        qf.to_tile(qtile, l32, g);
        kf.to_tile(ktile, l32, g);
        gf.to_tile(gtile, l32, g);
        if (g == 0) {
            rowsc[l32] = lc;
            rowsc[32 + l32] = -dl;
        }
        wave_sync_lds();

        // ---- lane = query: S^T = K Q^T, dP^T = V dO^T, dS^T, dQ^T = K^T dS^T
        {
            f32x16 s, dp;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = E::mfma(kf.f[ks], qf.f[ks], ks == 0 ? f32x16_zero() : s);
                dp = E::mfma(vf.f[ks], gf.f[ks], ks == 0 ? f32x16_zero() : dp);
            }
            u32x4 df[2];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float t = (allow_t >> i) & 1u ? fmaf(s[i], cs, -lc) : -INFINITY;
                s[i] = fast_exp2(t) * (dp[i] - dl);
                if (i % 2 == 1) df[i / 8][(i / 2) % 4] = E::pack(s[i - 1], s[i]);
            }
            f32x16 acc[CT];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x16_zero();
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[ct] = E::mfma(tr_frag(ktile, STRIDE, tr_off, ct, half), as_frag8(df[half]), acc[ct]);
            RowStore<D, E>::run(stage, acc, scale, dq + off, rs, rows_valid, lane);
        }
        // ---- lane = key: S = Q K^T, dP = dO V^T - delta, P, dS, dV^T = dO^T P, dK^T = Q^T dS
        {
            const float* rowv = rowsc + 4 * g;
            f32x16 s, dp;
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(rowv + 32 + 8 * a4);
#pragma unroll
                for (int e = 0; e < 4; ++e) dp[4 * a4 + e] = d4[e];
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = E::mfma(qf.f[ks], kf.f[ks], ks == 0 ? f32x16_zero() : s);
                dp = E::mfma(gf.f[ks], vf.f[ks], dp);
            }
            f32x4 l4[4];
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) l4[a4] = *reinterpret_cast<const f32x4*>(rowv + 8 * a4);
            u32x4 pf[2], df[2];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float t = (allow_n >> i) & 1u ? fmaf(s[i], cs, -l4[i / 4][i % 4]) : -INFINITY;
                const float pe = fast_exp2(t);
                s[i] = pe;
                dp[i] = pe * dp[i];
                if (i % 2 == 1) {
                    pf[i / 8][(i / 2) % 4] = E::pack(s[i - 1], s[i]);
                    df[i / 8][(i / 2) % 4] = E::pack(dp[i - 1], dp[i]);
                }
            }
            f32x16 dka[CT], dva[CT];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                dka[ct] = f32x16_zero();
                dva[ct] = f32x16_zero();
            }
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    dva[ct] = E::mfma(tr_frag(gtile, STRIDE, tr_off, ct, half), as_frag8(pf[half]), dva[ct]);
                    dka[ct] = E::mfma(tr_frag(qtile, STRIDE, tr_off, ct, half), as_frag8(df[half]), dka[ct]);
                }
            RowStore<D, E>::run(stage, dka, scale, dk + off, rs, rows_valid, lane);
            RowStore<D, E>::run(stage, dva, 1.0f, dv + off, rs, rows_valid, lane);
        }
        wave_sync_lds();  // the tiles are rewritten by the next window
    }
}
