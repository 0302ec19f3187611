// Device-side building blocks shared by the attention kernels (gfx950 / CDNA4 only).
//
// Register and LDS layouts used throughout
// ----------------------------------------
// All contractions use v_mfma_f32_32x32x16_bf16 (one wavefront, 32x32 output tile, 16 deep):
//   A operand (32 x 16): lane l holds row  l%32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   B operand (16 x 32): lane l holds col  l%32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   accumulator (32x32): lane l holds col  l%32; register v (0..15) holds row
//                        8*(v/4) + 4*(l/32) + v%4
// Only "slot t of lane group g of A meets slot t of lane group g of B" matters for correctness of
// a contraction, so operands whose contraction index is a channel are read straight from memory
// rows (8 consecutive channels per lane), and operands whose contraction index is a token are read
// from a transposed LDS tile whose token positions are permuted to match the accumulator rows.
//
// Natural LDS tile   : R token rows of D bf16, row stride D*2+16 bytes (the 16-byte pad makes the
//                      16-byte fragment reads of 16 consecutive lanes hit distinct banks).
// Transposed LDS tile: one row per channel, R token slots of bf16 per row, stride R*2+16 bytes.
//                      Token r of the tile sits at slot 16*(r/16) + 8*g + 4*a + e where
//                      r%16 = 8*a + 4*g + e.  Lane group g of an MFMA then reads its 8 slots of
//                      a 16-token step as one 16-byte unit, and slot t = 4*a + e is the token that
//                      accumulator register 8*step + t of the same lane group belongs to.
//                      The 16-byte unit index within a row is XORed with (row/16)%4, which spreads
//                      the 8-byte writes of the staging threads over all banks.
#pragma once
#include <hip/hip_runtime.h>

#define DEVINL __device__ __forceinline__

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

DEVINL f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

DEVINL bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

// max of three without the NaN-quieting moves the generic fmaxf lowering adds in front
DEVINL float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// Exchange between the two halves of the wavefront (lane l <-> lane l^32) with v_permlane32_swap.
// The instruction swaps the upper half of its first register with the lower half of its second;
// fed with two copies of x it leaves, in every lane, the lower-half lane's value in the first
// result and the upper-half lane's value in the second.  The empty asm pins both results as
// separate integer registers before they are reinterpreted as floats (without it this compiler
// folds the two results into one register once they are bit-cast).
DEVINL void halves(float x, float& lower, float& upper)
{
    const unsigned a = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    lower = __builtin_bit_cast(float, r0);
    upper = __builtin_bit_cast(float, r1);
}
DEVINL float both_halves_max(float x)
{
    float lo, hi;
    halves(x, lo, hi);
    return max3(lo, hi, hi);
}
DEVINL float both_halves_sum(float x)
{
    float lo, hi;
    halves(x, lo, hi);
    return lo + hi;
}

DEVINL float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

DEVINL float max16(const f32x16& s)
{
    float m = max3(s[0], s[1], s[2]);
    m = max3(m, s[3], s[4]);
    m = max3(m, s[5], s[6]);
    m = max3(m, s[7], s[8]);
    m = max3(m, s[9], s[10]);
    m = max3(m, s[11], s[12]);
    m = max3(m, s[13], s[14]);
    return max3(m, s[15], s[15]);
}

// two fp32 -> packed bf16 pair (round to nearest even), low half = a
DEVINL unsigned pack_bf16(float a, float b)
{
    bf16x2 p;
    p[0] = (bf16)a;
    p[1] = (bf16)b;
    return __builtin_bit_cast(unsigned, p);
}

// accumulator registers 8*half .. 8*half+7 -> bf16 B-operand fragment of one 16-deep step
DEVINL bf16x8 acc_to_frag(const f32x16& s, int half)
{
    u32x4 r;
    const int b = 8 * half;
    r[0] = pack_bf16(s[b + 0], s[b + 1]);
    r[1] = pack_bf16(s[b + 2], s[b + 3]);
    r[2] = pack_bf16(s[b + 4], s[b + 5]);
    r[3] = pack_bf16(s[b + 6], s[b + 7]);
    return as_bf16x8(r);
}

// acc + sum of the 8 bf16 values of a fragment (fp32 accumulation, v_dot2 with a vector of ones)
DEVINL float frag_sum(bf16x8 f, float acc)
{
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16x2 pr;
        pr[0] = f[2 * i];
        pr[1] = f[2 * i + 1];
        acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
    }
    return acc;
}

// ---------------------------------------------------------------------------------------------
// Global memory view of one (batch, head) slice [N rows, row stride rs elements, D channels] as a
// buffer resource: loads whose byte offset lies beyond the last row return zeros in hardware, so
// tiles that hang over the end of the sequence need no branches.
// ---------------------------------------------------------------------------------------------
struct SliceView {
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned row_bytes;  // rs * 2
    DEVINL SliceView(const bf16* base, long rs, int N, int D)
    {
        const unsigned bytes = (unsigned)(((long)(N - 1) * rs + D) * 2);
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(base), 0, (int)bytes, 0x00020000);
        row_bytes = (unsigned)(rs * 2);
    }
    DEVINL u32x4 load16(unsigned byte_off) const { return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0); }
    DEVINL u32x2 load8(unsigned byte_off) const { return __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_off, 0, 0); }
};
constexpr unsigned kOutOfRange = 0x7fffffffu;  // a byte offset no slice reaches

// 16-byte fragment of a natural LDS tile: row `row`, 16-deep step `step`, lane group g
DEVINL bf16x8 nat_frag(const char* tile, int stride, int row, int step, int g)
{
    return *reinterpret_cast<const bf16x8*>(tile + row * stride + step * 32 + g * 16);
}
// 16-byte fragment of a transposed LDS tile (unit index swizzled by the row)
DEVINL bf16x8 tr_frag(const char* tile, int stride, int row, int step, int g)
{
    const int unit = (2 * step + g) ^ ((row >> 4) & 3);
    return *reinterpret_cast<const bf16x8*>(tile + row * stride + unit * 16);
}

// ---------------------------------------------------------------------------------------------
// Staging of a tile of R token rows x D channels from global memory into LDS through registers,
// so that the global loads of the next tile are in flight while the current one is computed on.
// Rows at or beyond N come back as zeros.  NT = threads of the workgroup.
// ---------------------------------------------------------------------------------------------
template <int D, int R, int NT>
struct NatStage {
    static constexpr int CH = D / 8;  // 16-byte chunks per row
    static constexpr int TOTAL = R * CH;
    static constexpr int PER = (TOTAL + NT - 1) / NT;
    static constexpr int STRIDE = D * 2 + 16;
    static constexpr int BYTES = R * STRIDE;
    u32x4 r[PER];

    DEVINL void load(const SliceView& src, int r0, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = tid + i * NT;
            const int row = idx / CH, ch = idx % CH;
            unsigned off = (unsigned)(r0 + row) * src.row_bytes + ch * 16;
            if (TOTAL % NT != 0 && idx >= TOTAL) off = kOutOfRange;
            r[i] = src.load16(off);
        }
    }
    DEVINL void store(char* tile, int tid) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = tid + i * NT;
            const int row = idx / CH, ch = idx % CH;
            if (TOTAL % NT == 0 || idx < TOTAL) *reinterpret_cast<u32x4*>(tile + row * STRIDE + ch * 16) = r[i];
        }
    }
};

template <int D, int R, int NT>
struct TrStage {
    static constexpr int CQ = D / 4;  // channel quads
    static constexpr int TQ = R / 4;  // token quads
    static constexpr int TOTAL = CQ * TQ;
    static constexpr int PER = (TOTAL + NT - 1) / NT;
    static constexpr int STRIDE = R * 2 + 16;
    static constexpr int ROWS = ((D + 31) / 32) * 32;  // channel rows incl. zero padding
    static constexpr int BYTES = ROWS * STRIDE;
    u32x2 r[PER][4];

    // thread idx -> (channel quad, token quad); the two low bits of the token quad are swapped so
    // that the 32 lanes of one LDS write phase land in distinct banks
    DEVINL static void split(int idx, int& cq, int& tq)
    {
        cq = idx % CQ;
        const int t = idx / CQ;
        tq = (t & ~3) | ((t & 1) << 1) | ((t >> 1) & 1);
    }
    DEVINL void load(const SliceView& src, int r0, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = tid + i * NT;
            int cq, tq;
            split(idx, cq, tq);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned off = (unsigned)(r0 + 4 * tq + e) * src.row_bytes + cq * 8;
                if (TOTAL % NT != 0 && idx >= TOTAL) off = kOutOfRange;
                r[i][e] = src.load8(off);
            }
        }
    }
    // 4x4 transpose of 16-bit values in registers, then four 8-byte LDS writes (one per channel)
    DEVINL void store(char* tile, int tid) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = tid + i * NT;
            int cq, tq;
            split(idx, cq, tq);
            const int grp = tq / 4, w4 = tq % 4;
            const int slot = 16 * grp + 8 * (w4 % 2) + 4 * (w4 / 2);
            const int unit = (slot >> 3) ^ ((cq >> 2) & 3);  // rows 4cq..4cq+3 share (row/16)%4
            const int byte = unit * 16 + (slot & 7) * 2;
            if (TOTAL % NT == 0 || idx < TOTAL) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int d = c / 2;
                    u32x2 w;
                    if (c % 2 == 0) {
                        w[0] = (r[i][0][d] & 0xffffu) | (r[i][1][d] << 16);
                        w[1] = (r[i][2][d] & 0xffffu) | (r[i][3][d] << 16);
                    } else {
                        w[0] = (r[i][0][d] >> 16) | (r[i][1][d] & 0xffff0000u);
                        w[1] = (r[i][2][d] >> 16) | (r[i][3][d] & 0xffff0000u);
                    }
                    *reinterpret_cast<u32x2*>(tile + (4 * cq + c) * STRIDE + byte) = w;
                }
            }
        }
    }
    // rows D..ROWS-1 (present when D is not a multiple of 32) must read as zeros
    DEVINL static void zero_pad_rows(char* tile, int tid)
    {
        if constexpr (ROWS > D) {
            constexpr int WORDS = (ROWS - D) * STRIDE / 4;
            for (int i = tid; i < WORDS; i += NT) reinterpret_cast<unsigned*>(tile + D * STRIDE)[i] = 0u;
        }
    }
};

// Workgroup id -> logical tile id such that tiles with consecutive logical ids run on the same XCD
// (workgroups are dealt to the 8 XCDs round robin, and each XCD has its own L2): tiles of one
// (batch, head) then share the K/V (or Q/dO) lines they all read.  Returns -1 for the padding ids.
DEVINL int xcd_local_id(int block, int nblocks)
{
    const int chunk = (nblocks + 7) / 8;
    const int logical = (block % 8) * chunk + block / 8;
    return logical < nblocks ? logical : -1;
}

// store 4 consecutive channels (fp32 -> bf16) of one token
DEVINL void store_bf16x4(bf16* dst, float a, float b, float c, float d)
{
    u32x2 w;
    w[0] = pack_bf16(a, b);
    w[1] = pack_bf16(c, d);
    *reinterpret_cast<u32x2*>(dst) = w;
}
