// Device-side building blocks shared by the attention kernels (gfx950 / CDNA4 only).
//
// Register and LDS layouts used throughout
// ----------------------------------------
// All contractions use v_mfma_f32_32x32x16_bf16 or _f16 (one wavefront, 32x32 output tile, 16 deep):
//   A operand (32 x 16): lane l holds row  l%32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   B operand (16 x 32): lane l holds col  l%32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   accumulator (32x32): lane l holds col  l%32; register v (0..15) holds row
//                        8*(v/4) + 4*(l/32) + v%4
// Only "slot t of lane group g of A meets slot t of lane group g of B" matters for correctness of
// a contraction, so operands whose contraction index is a channel are read straight from memory
// rows (8 consecutive channels per lane), and operands whose contraction index is a token are read
// from a transposed LDS tile whose token positions are permuted to match the accumulator rows.
//
// LDS tile: R token rows of D two-byte elements in their natural order, row stride D*2+16 bytes for D = 64 and
// D*2+48 for D = 80 (an odd multiple of 16 bytes, so the 16-byte fragment reads of 16 consecutive
// lanes hit distinct banks; for D = 80 the zeroed pad also covers the reads of the channel tile
// that reaches past channel 79).
//   natural fragment   : lane = token row, 8 consecutive channels -> one ds_read_b128.
//   transposed fragment: lane = channel, 8 tokens.  Read from the same tile with two
//                        ds_read_b64_tr_b16.  Within a group of 16 lanes that instruction hands
//                        lane i, as element e, element i%4 of the 8 bytes addressed by lane
//                        i/4 + 4e; lane j therefore addresses token 4g + j/4 (+8 for the second
//                        read), channels c0 + 4(j%4).., and lane i receives channel c0 + i of
//                        tokens 4g..4g+3, i.e. exactly the tokens that accumulator registers
//                        8*step + 4a + e of lane group g belong to (a = 0 first read, 1 second).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#define DEVINL __device__ __forceinline__

typedef unsigned short raw16;  // one tensor element of either format, as bits
// 16 bytes = 8 elements: the unit every MFMA operand fragment is moved and held in
typedef __attribute__((ext_vector_type(8))) short frag8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

DEVINL f32x16 f32x16_zero()
{
    const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    return z;
}

DEVINL frag8 as_frag8(u32x4 x) { return __builtin_bit_cast(frag8, x); }

// ---------------------------------------------------------------------------------------------
// Element formats of the tensors.  Both are two bytes wide, so tiles, fragments and addressing are
// the same; only the contraction instruction, the roundings (nearest even in both) and the
// conversions differ.  kRowSumLimit is the forward pass's bound on a row sum of weights taken
// against the fixed reference (see avion_fwd.h): every weight is at most the sum, so the bound also
// keeps each weight representable in the format it is rounded to.
// ---------------------------------------------------------------------------------------------
struct Bf16 {
    typedef __attribute__((ext_vector_type(8))) __bf16 v8;
    typedef __attribute__((ext_vector_type(2))) __bf16 v2;
    static constexpr float kRowSumLimit = 7.9e28f;  // 2^96; bf16 has the exponent range of fp32
    DEVINL static f32x16 mfma(frag8 a, frag8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
    }
    // two fp32 -> packed pair, low half = a
    DEVINL static unsigned pack(float a, float b)
    {
        v2 p;
        p[0] = (__bf16)a;
        p[1] = (__bf16)b;
        return __builtin_bit_cast(unsigned, p);
    }
    // acc + both elements of a packed pair (fp32 accumulation, v_dot2 with a vector of ones)
    DEVINL static float add_pair(unsigned pair, float acc)
    {
        const v2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2, pair), ones, acc, false);
    }
    DEVINL static float widen(frag8 f, int e) { return (float)__builtin_bit_cast(v8, f)[e]; }
};
struct F16 {
    typedef __attribute__((ext_vector_type(8))) _Float16 v8;
    typedef __attribute__((ext_vector_type(2))) _Float16 v2;
    static constexpr float kRowSumLimit = 32768.0f;  // 2^15 < 65504, the largest fp16
    DEVINL static f32x16 mfma(frag8 a, frag8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8, a), __builtin_bit_cast(v8, b), c, 0, 0, 0);
    }
    DEVINL static unsigned pack(float a, float b)
    {
        v2 p;
        p[0] = (_Float16)a;
        p[1] = (_Float16)b;
        return __builtin_bit_cast(unsigned, p);
    }
    DEVINL static float add_pair(unsigned pair, float acc)
    {
        const v2 ones = {(_Float16)1.0f, (_Float16)1.0f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(v2, pair), ones, acc, false);
    }
    DEVINL static float widen(frag8 f, int e) { return (float)__builtin_bit_cast(v8, f)[e]; }
};

// Max of three.  Deliberately plain fmaxf, not inline assembly: the compiler inserts the wait states
// that a vector instruction needs before it may read an MFMA result (or feed a lane permute) only
// around instructions it knows, and an opaque asm statement reading an accumulator right after the
// MFMA that produces it picks up stale registers every now and then.  Only used outside hot loops.
DEVINL float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
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

// Wait until every outstanding global/buffer load of this wavefront has returned (vmcnt(0)).
// Placed once before a main loop so that loads issued in the prologue are not waited for again
// inside the loop, where the same counter also covers the tile prefetch that should stay in flight.
// lane index from the execution mask: costs two instructions where it is used and keeps no register alive before that
DEVINL int lane_from_exec() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

DEVINL void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

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

// accumulator registers 8*half .. 8*half+7 -> B-operand fragment of one 16-deep step
template <typename E>
DEVINL frag8 acc_to_frag(const f32x16& s, int half)
{
    u32x4 r;
    const int b = 8 * half;
    r[0] = E::pack(s[b + 0], s[b + 1]);
    r[1] = E::pack(s[b + 2], s[b + 3]);
    r[2] = E::pack(s[b + 4], s[b + 5]);
    r[3] = E::pack(s[b + 6], s[b + 7]);
    return as_frag8(r);
}

// acc + sum of the 8 values of a fragment (fp32 accumulation)
template <typename E>
DEVINL float frag_sum(frag8 f, float acc)
{
    const u32x4 w = __builtin_bit_cast(u32x4, f);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = E::add_pair(w[i], acc);
    return acc;
}

// ---------------------------------------------------------------------------------------------
// Global memory view of one (batch, head) slice [N rows, row stride rs elements, D channels] as a
// buffer resource: loads whose byte offset lies beyond the last row return zeros in hardware, so
// tiles that hang over the end of the sequence need no branches.
// ---------------------------------------------------------------------------------------------
DEVINL unsigned slice_bytes(long rs, int N, int D) { return (unsigned)(((long)(N - 1) * rs + D) * 2); }
struct SliceView {
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned row_bytes;  // rs * 2
    unsigned bytes;      // extent of the slice
    DEVINL SliceView(const raw16* base, long rs, int N, int D)
    {
        bytes = slice_bytes(rs, N, D);
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<raw16*>(base), 0, (int)bytes, 0x00020000);
        row_bytes = (unsigned)(rs * 2);
    }
    DEVINL u32x4 load16(unsigned byte_off) const { return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0); }
    DEVINL u32x2 load8(unsigned byte_off) const { return __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_off, 0, 0); }
};
constexpr unsigned kOutOfRange = 0x7fffffffu;  // a byte offset no slice reaches
// Same, for offsets that a tile base (< 2^31) is still added to: the sum stays in [2^31, 2^32).
constexpr unsigned kOutOfRangeBase = 0x80000000u;

// Global -> LDS without passing through registers (buffer_load_dwordx4 ... lds): the 16 bytes that
// lane i fetches from byte offset `voff` of the buffer land at LDS address lds_addr + 16*i, so one
// instruction fills 1 KB of LDS; lds_addr (it travels in M0) must be the same in all lanes.
// Offsets beyond the buffer deposit zeros.  Completion is tracked by the vector-memory counter
// (s_waitcnt vmcnt) for the fetch and by lgkmcnt for the write into LDS.
// Written as inline assembly on purpose: told that an instruction writes LDS asynchronously, the
// compiler makes every later LDS read wait for ALL outstanding loads, which would serialise the
// prefetch; here the ordering is established by hand (vmcnt waits + workgroup barriers).
struct RawBuffer {
    u32x4 words;  // base[31:0] | base[47:32] | bytes | flags: raw buffer, offsets beyond `bytes` are out of range
    DEVINL RawBuffer(const void* base, unsigned bytes)
    {
        const unsigned long a = (unsigned long)base;
        words[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
        words[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32) & 0xffffu);
        words[2] = __builtin_amdgcn_readfirstlane(bytes);
        words[3] = 0x00020000u;
    }
    DEVINL explicit RawBuffer(u32x4 w) : words(w) {}
};
DEVINL unsigned lds_address(const char* p) { return (unsigned)(unsigned long)(const lds_char*)p; }
// one of two / three descriptors, chosen by a wavefront-uniform condition; the result is moved to
// scalar registers explicitly because the compiler may have kept the selection in vector registers
DEVINL RawBuffer pick(bool first, const RawBuffer& a, const RawBuffer& b)
{
    RawBuffer r = first ? a : b;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.words[i] = __builtin_amdgcn_readfirstlane(r.words[i]);
    return r;
}
// Wait states: the compiler's hazard recogniser does not look inside the statement.  M0 must be
// written at least one wait state before the load that reads it, and a scalar register that a
// vector instruction (v_readfirstlane) has just produced -- the descriptor words or lds_addr may be
// such registers -- needs five wait states before a vector-memory instruction reads it.  s_mov plus
// s_nop 4 (five wait states) puts six between anything before the statement and the load.
DEVINL void load_to_lds16(const RawBuffer& buf, unsigned lds_addr, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(buf.words)
                 : "memory", "m0");
}

// Byte offset, relative to the tile's first row, that `lane` fetches for 1 KB block `blk` of a padded
// LDS tile (row stride tile_stride<D>(), D/8 data chunks of 16 bytes per row, the rest padding): the
// block holds chunks 64*blk .. 64*blk+63 of the tile in row-major order.  Lanes that land on a pad
// chunk get an offset beyond any buffer, so that zeros are deposited there.
template <int D>
DEVINL unsigned padded_block_voff(int blk, int lane, unsigned row_bytes);

// row stride of an LDS tile in bytes
template <int D>
constexpr int tile_stride()
{
    return D == 64 ? 144 : D * 2 + 48;
}

template <int D>
DEVINL unsigned padded_block_voff(int blk, int lane, unsigned row_bytes)
{
    constexpr int CPR = tile_stride<D>() / 16, DCH = D / 8;
    const int c = 64 * blk + lane, row = c / CPR, pos = c % CPR;
    return pos < DCH ? (unsigned)row * row_bytes + pos * 16 : kOutOfRangeBase;
}

// natural fragment: row `row`, 16-deep channel step `step`, lane group g
DEVINL frag8 nat_frag(const char* tile, int stride, int row, int step, int g)
{
    return *reinterpret_cast<const frag8*>(tile + row * stride + step * 32 + g * 16);
}

// per-lane byte offset for transposed fragment reads (see the layout notes at the top)
DEVINL int tr_lane_offset(int lane, int stride)
{
    const int G = lane >> 4, j = lane & 15;
    return (4 * (G >> 1) + (j >> 2)) * stride + (16 * (G & 1) + 4 * (j & 3)) * 2;
}
// transposed fragment: channel tile ct (32 channels), 16-token step `step`
DEVINL frag8 tr_frag(const char* tile, int stride, int lane_off, int ct, int step)
{
    const lds_char* p = (const lds_char*)tile + lane_off + step * 16 * stride + ct * 64;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * stride));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    const u32x4 r = {l2[0], l2[1], h2[0], h2[1]};
    return as_frag8(r);
}

// ---------------------------------------------------------------------------------------------
// Staging of a tile of R token rows x D channels from global memory into LDS through registers,
// so that the global loads of the next tile are in flight while the current one is computed on.
// Rows at or beyond N come back as zeros.  NT = threads of the workgroup.
// ---------------------------------------------------------------------------------------------
template <int D, int R, int NT>
struct TileStage {
    static constexpr int CH = D / 8;  // 16-byte chunks per row
    static constexpr int TOTAL = R * CH;
    static constexpr int PER = (TOTAL + NT - 1) / NT;
    static constexpr int STRIDE = tile_stride<D>();
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
    // the pad of every row reads as zeros (only D = 80 ever reads it)
    DEVINL static void zero_pad(char* tile, int tid)
    {
        constexpr int PADW = (STRIDE - D * 2) / 4;
        for (int i = tid; i < R * PADW; i += NT)
            *reinterpret_cast<unsigned*>(tile + (i / PADW) * STRIDE + D * 2 + (i % PADW) * 4) = 0u;
    }
};

// Initial value of a transposed score accumulator (lane = query, register i = key
// key_base + 8*(i/4) + 4*g + i%4) that removes keys at or beyond N from the softmax: 0 for valid
// keys, a huge negative number otherwise.  Those keys are zero rows in LDS, so the contraction adds
// nothing to it, and exp2 of it is exactly 0: weight 0, dS 0, no inf * 0.
DEVINL f32x16 key_mask_block(int key_base, int g, int N)
{
    f32x16 r;
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = key_base + 8 * (i / 4) + 4 * g + (i % 4) < N ? 0.f : -1.0e30f;
    return r;
}
// Causal attention (query i sees keys 0..i): the same with a per-lane bound.  In the query-stationary
// kernels the lane is a query and passes N = min(N, query + 1) to key_mask_block above.  In the
// key-stationary kernel the lane is a key and the registers are queries
// query_base + 8*(i/4) + 4*g + i%4: a query below the lane's key must not see it.
DEVINL f32x16 query_mask_block(int query_base, int g, int key)
{
    f32x16 r;
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = query_base + 8 * (i / 4) + 4 * g + (i % 4) >= key ? 0.f : -1.0e30f;
    return r;
}

// ---------------------------------------------------------------------------------------------
// Ring of NBUF buffers in LDS, each holding an A tile and a B tile of 64 token rows in the padded
// row layout above (K and V, or Q and dO) and, with SCALARS, one more 1 KB block with x[64] then
// y[64] floats, where x and y are two arrays of `npad` floats stored one after the other in global
// memory (LSE*log2e and -delta as the dQ pass leaves them).  Buffers are filled straight from
// global memory by LDS-direct loads: a buffer is a sequence of 1 KB blocks (A blocks, B blocks,
// scalars), each filled by one load of one wavefront; a block of a tile holds 64 consecutive
// 16-byte chunks of its padded rows, and lanes that land on a pad chunk deposit zeros.  Blocks are
// dealt round robin: wavefront w issues blocks w, w+NW, ...  Tiles past the end of the sequence
// arrive as zero rows.
// ---------------------------------------------------------------------------------------------
template <int D, int NW, int NBUF, bool SCALARS>
struct TileRing {
    static constexpr int ROWS = 64;
    static constexpr int STRIDE = tile_stride<D>();
    static constexpr int TILE_BYTES = ROWS * STRIDE;
    static_assert(TILE_BYTES % 1024 == 0, "a tile must be a whole number of 1 KB blocks");
    static_assert((NBUF & (NBUF - 1)) == 0, "ring size must be a power of two");
    static constexpr int NTI = TILE_BYTES / 1024, NBLK = 2 * NTI + (SCALARS ? 1 : 0), NPW = (NBLK + NW - 1) / NW;
    static constexpr int OFF_B = TILE_BYTES, OFF_SCALARS = 2 * TILE_BYTES;
    static constexpr int BUF_BYTES = NBLK * 1024;
    static constexpr int LDS_BYTES = NBUF * BUF_BYTES;

    char* smem;
    unsigned smem_addr;
    int ntiles, wave;
    // per load j of this wavefront (block wave + NW*j, if there is one):
    bool has[NPW];        // the block exists
    bool is_scalars[NPW];
    unsigned voff[NPW];   // this lane's byte offset for tile 0
    unsigned vstep[NPW];  // what a step to the next tile adds to it
    u32x4 desc[NPW];      // descriptor of the array the block comes from

    // a, b: first rows of the two [N, D] slices, whose rows are rs_a and rs_b elements apart
    DEVINL TileRing(const raw16* a, long rs_a, const raw16* b, long rs_b, int N, const float* scalars, int npad,
                    int ntiles_, char* smem_, int wave_, int lane)
        : smem(smem_), smem_addr(lds_address(smem_)), ntiles(ntiles_), wave(wave_)
    {
        const RawBuffer a_buf(a, slice_bytes(rs_a, N, D)), b_buf(b, slice_bytes(rs_b, N, D)),
            s_buf(scalars, SCALARS ? 2u * npad * 4u : 0u);
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
            const int blk = wave + NW * j;
            has[j] = blk < NBLK;
            const int kind = blk < NTI ? 0 : blk < 2 * NTI ? 1 : 2;
            is_scalars[j] = SCALARS && kind == 2;
            if (is_scalars[j]) {
                voff[j] = lane < 16 ? (unsigned)lane * 16 : lane < 32 ? (unsigned)(npad * 4 + (lane - 16) * 16) : kOutOfRangeBase;
                vstep[j] = ROWS * 4;
            } else {
                const unsigned row_bytes = (unsigned)((kind == 0 ? rs_a : rs_b) * 2);
                voff[j] = padded_block_voff<D>(blk - kind * NTI, lane, row_bytes);
                vstep[j] = ROWS * row_bytes;
            }
            desc[j] = pick(kind == 0, a_buf, pick(kind == 1, b_buf, s_buf)).words;
        }
    }
    DEVINL const char* buf(int ti) const { return smem + (ti & (NBUF - 1)) * BUF_BYTES; }
    // request tile `ti` (this wavefront's share of its blocks)
    DEVINL void fetch(int ti) const
    {
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
            if (!has[j]) continue;
            const unsigned dst = smem_addr + (ti & (NBUF - 1)) * BUF_BYTES + (wave + NW * j) * 1024;
            // the two scalar arrays follow one another, so running past the first would read the second
            const bool past_end = is_scalars[j] && ti >= ntiles;
            load_to_lds16(RawBuffer(desc[j]), dst, past_end ? kOutOfRangeBase : voff[j] + (unsigned)ti * vstep[j]);
        }
    }
    // Wait for all of this wavefront's requests, then meet the other wavefronts: after it every
    // requested tile is in LDS, and every wavefront is past the code before the barrier.  An
    // LDS-direct load counts in both counters -- vmcnt for the fetch, then lgkmcnt for the deposit
    // into LDS, hence two waits in this order -- and only when both have drained is the data visible
    // to other wavefronts.  (Plain
    // instructions: to the compiler the loads above are opaque, so no fence would wait for them.)
    DEVINL static void landed_barrier()
    {
        asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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

// Epilogue store of one wavefront's 32 x D result tile held as transposed accumulators
// (lane = token row l32 of the tile, register v of channel tile ct = channel
// 32*ct + 8*(v/4) + 4*g + v%4).  Written straight from that layout every lane would store 8-byte
// pieces of 32 different rows; instead the tile is rounded to the element format, laid out row-major in a
// per-wavefront LDS region and read back so that 8 (D=64) or 10 (D=80) consecutive lanes store one
// full row with 16-byte pieces.  `region` must not be in use by any other wavefront; LDS
// operations of one wavefront execute in order, so no barrier is needed in between.
template <int D, typename E>
struct RowStore {
    static constexpr int CT = (D + 31) / 32;
    static constexpr int STRIDE = D * 2 + 16;
    static constexpr int BYTES = 32 * STRIDE;  // per wavefront
    static constexpr int CH = D / 8;           // 16-byte chunks per row

    DEVINL static void run(char* region, const f32x16 (&acc)[CT], float mul, raw16* dst, long rs, int rows_valid, int lane)
    {
        const int l32 = lane % 32, g = lane / 32;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
                const int c0 = 32 * ct + 8 * a4 + 4 * g;
                if (c0 < D) {
                    u32x2 w;
                    w[0] = E::pack(acc[ct][4 * a4 + 0] * mul, acc[ct][4 * a4 + 1] * mul);
                    w[1] = E::pack(acc[ct][4 * a4 + 2] * mul, acc[ct][4 * a4 + 3] * mul);
                    *reinterpret_cast<u32x2*>(region + l32 * STRIDE + c0 * 2) = w;
                }
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int TOTAL = 32 * CH;
#pragma unroll
        for (int i = 0; i < (TOTAL + 63) / 64; ++i) {
            const int idx = lane + 64 * i;
            const int row = idx / CH, ch = idx % CH;
            if (idx < TOTAL && row < rows_valid) {
                const u32x4 val = *reinterpret_cast<const u32x4*>(region + row * STRIDE + ch * 16);
                *reinterpret_cast<u32x4*>(dst + (long)row * rs + ch * 8) = val;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
};
