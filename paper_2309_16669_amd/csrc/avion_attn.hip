// C ABI of the gfx950 attention library: argument checks, kernel-instance selection, launches.
// See include/avion_attn.h for the contract of every entry point.
#include "avion_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <atomic>
#include <cstring>
#include <mutex>

#include "avion_bwd.h"
#include "avion_fwd.h"
#include "avion_ln.h"
#include "avion_small.h"
#include "avion_gelu.h"

// Built-in scratch of avion_attn_bwd_noalloc: the per-query scalars that the backward's two passes
// hand to each other live here instead of in a caller's workspace.  One copy per GPU, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels get
// the device address that call returns.
constexpr size_t kScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char* what)
{
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return AVION_EHIP;
}

// Device address of `scratch` on each GPU, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return AVION_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return AVION_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Token strides (elements between consecutive tokens of one head) of the two tensor groups.
struct Strides {
    int qkv;  // Q, K, V and their gradients: H*d, or 3*H*d when they are packed in one tensor
    int o;    // O and dO: H*d
};

// Which kernel family an entry point runs: element format and masking.
struct Variant {
    bool f16;
    bool causal;
};

constexpr float kMinScale = 8.673617379884035e-19f;  // 2^-60

int check_shape(int B, int H, int N, int d, float scale, int packed = 1)
{
    if (B < 1 || H < 1 || N < 1) return AVION_EINVAL;
    // Keys past the end of a ragged tile (and keys a causal query must not see) are removed by a
    // score of -1e30 that is then multiplied by scale*log2(e); the product has to stay far below any
    // real score for the weight to come out as exactly 0, hence the floor of 2^-60 on scale.
    if (!(scale >= kMinScale) || !std::isfinite(scale)) return AVION_EINVAL;
    if (d != 64 && d != 80) return AVION_EUNSUPPORTED;
    if (N > (1 << 24) || (long long)B * H > (1 << 24)) return AVION_EUNSUPPORTED;
    // one (batch, head) slice is addressed with 32-bit byte offsets (buffer loads), and tile loads
    // may start up to four 64-row tiles past the end of the sequence
    if (((long long)N + 256) * packed * H * d * 2 >= (1LL << 31)) return AVION_EUNSUPPORTED;
    return AVION_OK;
}

// Workgroups are launched in multiples of 8 (one per XCD); the padding ones exit at once.
bool grid_for(long long nblocks, unsigned* grid)
{
    const long long padded = ((nblocks + 7) / 8) * 8;
    if (padded > 0x7fffffffLL) return false;
    *grid = (unsigned)padded;
    return true;
}

// Raises the kernel's dynamic LDS limit once; `done` is the caller's per-instance flag.  A failure
// is not remembered, so the next call tries again.
template <typename K>
hipError_t allow_lds(K kernel, int bytes, std::atomic<bool>& done)
{
    if (done.load(std::memory_order_acquire)) return hipSuccess;
    const hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.store(true, std::memory_order_release);
    return e;
}

// Result of the launch just made on this thread.  Errors left behind by earlier, unrelated work of
// the caller are cleared before the launch (begin_launch) so that they are not mistaken for it.
void begin_launch() { (void)hipGetLastError(); }
int end_launch(const char* what)
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? AVION_OK : hip_fail(e, what);
}

template <int D, int NW, typename E, bool CAUSAL>
int launch_fwd(const raw16* q, const raw16* k, const raw16* v, raw16* o, float* lse, int B, int H, int N, Strides rs,
               float scale, hipStream_t st)
{
    using Cfg = FwdCfg<D, NW>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_fwd_kernel<D, NW, E, CAUSAL>, Cfg::LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(fwd)");
    const int nqb = (N + Cfg::BM - 1) / Cfg::BM;
    const long long nblocks = (long long)nqb * B * H;
    unsigned grid;
    if (!grid_for(nblocks, &grid)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_fwd_kernel<D, NW, E, CAUSAL>), dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, q, k, v, o, lse, H, N, rs.qkv,
                       rs.o, nqb, (int)nblocks, scale * kLog2e);
    return end_launch("launch avion_fwd_kernel");
}

template <int D, int NW, typename E, bool CAUSAL>
int launch_dq(const raw16* q, const raw16* k, const raw16* v, const raw16* o, const raw16* dO, const float* lse, raw16* dq,
              float* rowsc, int B, int H, int N, Strides rs, float scale, hipStream_t st)
{
    using Cfg = DqCfg<D, NW>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_dq_kernel<D, NW, E, CAUSAL>, Cfg::LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(dq)");
    const int nqb = (N + Cfg::BM - 1) / Cfg::BM;
    const long long nblocks = (long long)nqb * B * H;
    unsigned grid;
    if (!grid_for(nblocks, &grid)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_dq_kernel<D, NW, E, CAUSAL>), dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, q, k, v, o, dO, lse, dq,
                       rowsc, H, N, rs.qkv, rs.o, nqb, (int)nblocks, scale * kLog2e, scale);
    return end_launch("launch avion_dq_kernel");
}

template <int D, int NW, typename E, bool CAUSAL>
int launch_dkdv(const raw16* q, const raw16* k, const raw16* v, const raw16* dO, const float* rowsc, raw16* dk, raw16* dv,
                int B, int H, int N, Strides rs, float scale, hipStream_t st)
{
    using Cfg = DkvCfg<D, NW>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_dkdv_kernel<D, NW, E, CAUSAL>, Cfg::LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(dkdv)");
    const int nkb = (N + Cfg::BNK - 1) / Cfg::BNK;
    const long long nblocks = (long long)nkb * B * H;
    unsigned grid;
    if (!grid_for(nblocks, &grid)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_dkdv_kernel<D, NW, E, CAUSAL>), dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, q, k, v, dO, rowsc, dk,
                       dv, H, N, rs.qkv, rs.o, nkb, (int)nblocks, scale * kLog2e, scale);
    return end_launch("launch avion_dkdv_kernel");
}

template <int D, int NW, typename E, bool CAUSAL>
int launch_bwd_small(const raw16* q, const raw16* k, const raw16* v, const raw16* o, const raw16* dO, const float* lse,
                     raw16* dq, raw16* dk, raw16* dv, float* rowsc, int B, int H, int N, Strides rs, float scale,
                     hipStream_t st)
{
    using Cfg = BwdSmallCfg<D, NW>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_bwd_small_kernel<D, NW, E, CAUSAL>, Cfg::LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(bwd_small)");
    const long long nblocks = (long long)B * H;
    unsigned grid;
    if (!grid_for(nblocks, &grid)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_bwd_small_kernel<D, NW, E, CAUSAL>), dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, st, q, k, v, o,
                       dO, lse, dq, dk, dv, rowsc, H, N, rs.qkv, rs.o, (int)nblocks, scale * kLog2e, scale);
    return end_launch("launch avion_bwd_small_kernel");
}

// Sequences of at most 32 tokens: one wavefront per window of floor(32 / N) problems (avion_small.h).
constexpr int kWindowMaxN = 32;
struct WindowGrid {
    int G, nitems;
    unsigned grid;
};
template <int D>
bool window_grid(int B, int H, int N, WindowGrid* w)
{
    w->G = 32 / N;
    const long long nwin = ((long long)B + w->G - 1) / w->G, nitems = nwin * H;
    if (nitems > 0x7fffffffLL) return false;
    w->nitems = (int)nitems;
    const long long wgs = (nitems + WinCfg<D>::NW - 1) / WinCfg<D>::NW;
    w->grid = (unsigned)(wgs < 256 * 16 ? wgs : 256 * 16);  // wavefronts walk the windows with a stride
    return true;
}

template <int D, typename E, bool CAUSAL>
int launch_win_fwd(const raw16* q, const raw16* k, const raw16* v, raw16* o, float* lse, int B, int H, int N, Strides rs,
                   float scale, hipStream_t st)
{
    using Cfg = WinCfg<D>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_win_fwd_kernel<D, E, CAUSAL>, Cfg::FWD_LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(win_fwd)");
    WindowGrid w;
    if (!window_grid<D>(B, H, N, &w)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_win_fwd_kernel<D, E, CAUSAL>), dim3(w.grid), dim3(Cfg::NT), Cfg::FWD_LDS_BYTES, st, q, k, v, o,
                       lse, B, H, N, rs.qkv, rs.o, w.G, w.nitems, scale * kLog2e);
    return end_launch("launch avion_win_fwd_kernel");
}

template <int D, typename E, bool CAUSAL>
int launch_win_bwd(const raw16* q, const raw16* k, const raw16* v, const raw16* o, const raw16* dO, const float* lse,
                   raw16* dq, raw16* dk, raw16* dv, int B, int H, int N, Strides rs, float scale, hipStream_t st)
{
    using Cfg = WinCfg<D>;
    static std::atomic<bool> lds_allowed{false};
    const hipError_t attr = allow_lds(avion_win_bwd_kernel<D, E, CAUSAL>, Cfg::BWD_LDS_BYTES, lds_allowed);
    if (attr != hipSuccess) return hip_fail(attr, "hipFuncSetAttribute(win_bwd)");
    WindowGrid w;
    if (!window_grid<D>(B, H, N, &w)) return AVION_EUNSUPPORTED;
    begin_launch();
    hipLaunchKernelGGL((avion_win_bwd_kernel<D, E, CAUSAL>), dim3(w.grid), dim3(Cfg::NT), Cfg::BWD_LDS_BYTES, st, q, k, v, o,
                       dO, lse, dq, dk, dv, B, H, N, rs.qkv, rs.o, w.G, w.nitems, scale * kLog2e, scale);
    return end_launch("launch avion_win_bwd_kernel");
}

// Kernel instances: four wavefronts per workgroup for every kernel, head size, format and masking.
// Calls f(head dim, element format, causal) with the three as compile-time tags.
template <typename T>
struct TypeTag {
    using type = T;
};
template <typename F>
int by_variant(Variant var, int d, F f)
{
    auto by_dim = [&](auto fmt, auto causal) {
        if (d == 64) return f(std::integral_constant<int, 64>{}, fmt, causal);
        return f(std::integral_constant<int, 80>{}, fmt, causal);
    };
    auto by_fmt = [&](auto causal) {
        if (var.f16) return by_dim(TypeTag<F16>{}, causal);
        return by_dim(TypeTag<Bf16>{}, causal);
    };
    if (var.causal) return by_fmt(std::true_type{});
    return by_fmt(std::false_type{});
}


int fwd_impl(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d, int packed,
             Variant var, float scale, void* stream)
{
    if (!q || !k || !v || !o || !lse) return AVION_EINVAL;
    const int rc = check_shape(B, H, N, d, scale, packed);
    if (rc != AVION_OK) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse)) return AVION_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Strides rs{packed * H * d, H * d};
    const raw16 *qq = static_cast<const raw16*>(q), *kk = static_cast<const raw16*>(k), *vv = static_cast<const raw16*>(v);
    raw16* oo = static_cast<raw16*>(o);
    if (N <= kWindowMaxN)
        return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
            return launch_win_fwd<decltype(dim)::value, typename decltype(fmt)::type, decltype(causal)::value>(
                qq, kk, vv, oo, lse, B, H, N, rs, scale, st);
        });
    return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
        return launch_fwd<decltype(dim)::value, 4, typename decltype(fmt)::type, decltype(causal)::value>(
            qq, kk, vv, oo, lse, B, H, N, rs, scale, st);
    });
}

bool workspace_ok(const void* workspace, size_t workspace_bytes, int B, int H, int N, int d)
{
    return workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u) == 0 &&
           workspace_bytes >= avion_attn_bwd_workspace_bytes(B, H, N, d);
}

int dq_impl(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq, int B,
            int H, int N, int d, int packed, Variant var, float scale, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !o || !lse || !dO || !dq) return AVION_EINVAL;
    const int rc = check_shape(B, H, N, d, scale, packed);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {q, k, v, o, lse, dO, dq};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    if (!workspace_ok(workspace, workspace_bytes, B, H, N, d)) return AVION_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Strides rs{packed * H * d, H * d};
    float* rowsc = static_cast<float*>(workspace);  // receives LSE*log2e and -delta for the second pass
    const raw16 *qq = static_cast<const raw16*>(q), *kk = static_cast<const raw16*>(k), *vv = static_cast<const raw16*>(v),
               *oo = static_cast<const raw16*>(o), *gg = static_cast<const raw16*>(dO);
    raw16* dqq = static_cast<raw16*>(dq);
    return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
        return launch_dq<decltype(dim)::value, 4, typename decltype(fmt)::type, decltype(causal)::value>(
            qq, kk, vv, oo, gg, lse, dqq, rowsc, B, H, N, rs, scale, st);
    });
}

int dkdv_impl(const void* q, const void* k, const void* v, const float* lse, const void* dO, void* dk, void* dv, int B,
              int H, int N, int d, int packed, Variant var, float scale, const void* workspace, size_t workspace_bytes,
              void* stream)
{
    if (!q || !k || !v || !lse || !dO || !dk || !dv) return AVION_EINVAL;
    const int rc = check_shape(B, H, N, d, scale, packed);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {q, k, v, lse, dO, dk, dv};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    if (!workspace_ok(workspace, workspace_bytes, B, H, N, d)) return AVION_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Strides rs{packed * H * d, H * d};
    const float* rowsc = static_cast<const float*>(workspace);  // LSE*log2e and -delta, left by the dQ pass
    const raw16 *qq = static_cast<const raw16*>(q), *kk = static_cast<const raw16*>(k), *vv = static_cast<const raw16*>(v),
               *gg = static_cast<const raw16*>(dO);
    raw16 *dkk = static_cast<raw16*>(dk), *dvv = static_cast<raw16*>(dv);
    return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
        return launch_dkdv<decltype(dim)::value, 4, typename decltype(fmt)::type, decltype(causal)::value>(
            qq, kk, vv, gg, rowsc, dkk, dvv, B, H, N, rs, scale, st);
    });
}

// Whole backward in one launch (N <= 128); arguments already checked by the caller.
int bwd_small_impl(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
                   void* dk, void* dv, int B, int H, int N, int d, int packed, Variant var, float scale, void* workspace,
                   void* stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Strides rs{packed * H * d, H * d};
    float* rowsc = static_cast<float*>(workspace);
    const raw16 *qq = static_cast<const raw16*>(q), *kk = static_cast<const raw16*>(k), *vv = static_cast<const raw16*>(v),
                *oo = static_cast<const raw16*>(o), *gg = static_cast<const raw16*>(dO);
    raw16 *dqq = static_cast<raw16*>(dq), *dkk = static_cast<raw16*>(dk), *dvv = static_cast<raw16*>(dv);
    return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
        return launch_bwd_small<decltype(dim)::value, 4, typename decltype(fmt)::type, decltype(causal)::value>(
            qq, kk, vv, oo, gg, lse, dqq, dkk, dvv, rowsc, B, H, N, rs, scale, st);
    });
}

int bwd_impl(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
             void* dk, void* dv, int B, int H, int N, int d, int packed, Variant var, float scale, void* workspace,
             size_t workspace_bytes, void* stream)
{
    // every argument is checked before the first launch, so an error leaves all outputs untouched
    if (!q || !k || !v || !o || !lse || !dO || !dq || !dk || !dv) return AVION_EINVAL;
    const int rc = check_shape(B, H, N, d, scale, packed);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {q, k, v, o, lse, dO, dq, dk, dv};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    if (!workspace_ok(workspace, workspace_bytes, B, H, N, d)) return AVION_EWORKSPACE;
    if (N <= kWindowMaxN) {
        // one wavefront per window of problems; needs no workspace (it is still checked, as for every shape)
        hipStream_t st = static_cast<hipStream_t>(stream);
        const Strides rs{packed * H * d, H * d};
        const raw16 *qq = static_cast<const raw16*>(q), *kk = static_cast<const raw16*>(k), *vv = static_cast<const raw16*>(v),
                    *oo = static_cast<const raw16*>(o), *gg = static_cast<const raw16*>(dO);
        raw16 *dqq = static_cast<raw16*>(dq), *dkk = static_cast<raw16*>(dk), *dvv = static_cast<raw16*>(dv);
        return by_variant(var, d, [&](auto dim, auto fmt, auto causal) {
            return launch_win_bwd<decltype(dim)::value, typename decltype(fmt)::type, decltype(causal)::value>(
                qq, kk, vv, oo, gg, lse, dqq, dkk, dvv, B, H, N, rs, scale, st);
        });
    }
    if (N <= BwdSmallCfg<64, 4>::MAX_N)
        return bwd_small_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, packed, var, scale, workspace, stream);
    const int rq = dq_impl(q, k, v, o, lse, dO, dq, B, H, N, d, packed, var, scale, workspace, workspace_bytes, stream);
    if (rq != AVION_OK) return rq;
    return dkdv_impl(q, k, v, lse, dO, dk, dv, B, H, N, d, packed, var, scale, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------------------ layer normalisation
int ln_check(long long M, int D, unsigned flags)
{
    if (M < 1 || D < 1) return AVION_EINVAL;
    if (flags & ~AVION_FLAG_F16) return AVION_EINVAL;
    if (D % 8 != 0 || D > 64 * 8 * kLnMaxChunks) return AVION_EUNSUPPORTED;
    if (M > (1LL << 40)) return AVION_EUNSUPPORTED;
    return AVION_OK;
}
unsigned ln_grid(long long M)
{
    const long long wgs = (M + kLnWaves - 1) / kLnWaves;
    return (unsigned)(wgs < kLnMaxGrid ? wgs : kLnMaxGrid);
}
// calls f(chunks per lane, element format) with both as compile-time tags
template <typename F>
int ln_dispatch(int D, bool f16, F f)
{
    const int per_lane = (D / 8 + 63) / 64;
    auto by_fmt = [&](auto nch) {
        if (f16) return f(nch, TypeTag<F16>{});
        return f(nch, TypeTag<Bf16>{});
    };
    if (per_lane <= 1) return by_fmt(std::integral_constant<int, 1>{});
    if (per_lane <= 2) return by_fmt(std::integral_constant<int, 2>{});
    return by_fmt(std::integral_constant<int, 4>{});
}

// ------------------------------------------------------------------------------------ bias + GELU
constexpr int kGeluMaxF = 1 << 16;
int gelu_check(long long M, int F, unsigned flags)
{
    if (M < 1 || F < 1) return AVION_EINVAL;
    if (flags & ~AVION_FLAG_F16) return AVION_EINVAL;
    if (F % 8 != 0 || F > kGeluMaxF) return AVION_EUNSUPPORTED;
    if (M > (1LL << 40)) return AVION_EUNSUPPORTED;
    return AVION_OK;
}
// column blocks of 1024 columns, and row groups so that the launch has at most kGeluMaxGrid workgroups
struct GeluGrid {
    int ncb, nrg;
};
// tensors beyond half of the 256 MB last-level cache are streamed past it
bool gelu_streams(long long M, int F) { return M * F * 2 > (128LL << 20); }
GeluGrid gelu_grid(long long M, int F)
{
    GeluGrid g;
    g.ncb = (F / 8 + kGeluThreads - 1) / kGeluThreads;
    const long long most = kGeluMaxGrid / g.ncb;
    g.nrg = (int)(M < most ? M : most);
    return g;
}

constexpr unsigned kAllFlags = AVION_FLAG_F16 | AVION_FLAG_CAUSAL | AVION_FLAG_QKVPACKED;

// q, k, v planes of a packed [B, N, 3, H, d] tensor
struct Planes {
    const char *q, *k, *v;
    Planes(const void* qkv, int H, int d)
    {
        const char* p = static_cast<const char*>(qkv);
        const size_t plane = (size_t)H * d * 2;
        q = p;
        k = p ? p + plane : nullptr;
        v = p ? p + 2 * plane : nullptr;
    }
};

}  // namespace

extern "C" {

int avion_version(void) { return 20200; }  // 2.2.0

const char* avion_strerror(int code)
{
    switch (code) {
        case AVION_OK: return "ok";
        case AVION_EINVAL: return "invalid argument (null pointer, B/H/N < 1, or scale not finite or below 2^-60)";
        case AVION_EUNSUPPORTED: return "unsupported shape or alignment (d must be 64 or 80; pointers 16-byte aligned)";
        case AVION_EWORKSPACE: return "workspace missing, misaligned or too small";
        case AVION_EHIP: return "HIP runtime error (see avion_last_hip_error)";
        case AVION_ESCRATCH: return "problem needs more than the 32 MiB built-in scratch of avion_attn_bwd_noalloc";
        default: return "unknown avion error code";
    }
}

const char* avion_last_hip_error(void) { return g_hip_error; }

int avion_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                   float scale, void* stream)
{
    return fwd_impl(q, k, v, o, lse, B, H, N, d, 1, Variant{false, false}, scale, stream);
}

int avion_attn_fwd_qkvpacked(const void* qkv, void* o, float* lse, int B, int H, int N, int d, float scale, void* stream)
{
    if (H < 1 || d < 1) return AVION_EINVAL;
    const Planes p(qkv, H, d);
    return fwd_impl(p.q, p.k, p.v, o, lse, B, H, N, d, 3, Variant{false, false}, scale, stream);
}

size_t avion_attn_bwd_workspace_bytes(int B, int H, int N, int d)
{
    if (check_shape(B, H, N, d, 1.0f) != AVION_OK) return 0;
    // per (batch, head): LSE*log2e and -delta, each padded to a multiple of 64 rows
    const size_t npad = ((size_t)N + 63) & ~(size_t)63;
    const size_t bytes = (size_t)B * H * 2 * npad * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

int avion_attn_bwd_dq(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                      void* dq, int B, int H, int N, int d, float scale, void* workspace, size_t workspace_bytes,
                      void* stream)
{
    return dq_impl(q, k, v, o, lse, dO, dq, B, H, N, d, 1, Variant{false, false}, scale, workspace, workspace_bytes, stream);
}

int avion_attn_bwd_dkdv(const void* q, const void* k, const void* v, const float* lse, const void* dO, void* dk,
                        void* dv, int B, int H, int N, int d, float scale, const void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return dkdv_impl(q, k, v, lse, dO, dk, dv, B, H, N, d, 1, Variant{false, false}, scale, workspace, workspace_bytes,
                     stream);
}

int avion_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                   void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    return bwd_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, 1, Variant{false, false}, scale, workspace, workspace_bytes,
                    stream);
}

int avion_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                           void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, void* stream)
{
    // argument errors first, so that they are reported as for avion_attn_bwd
    if (!q || !k || !v || !o || !lse || !dO || !dq || !dk || !dv) return AVION_EINVAL;
    const int rc = check_shape(B, H, N, d, scale);
    if (rc != AVION_OK) return rc;
    const size_t need = avion_attn_bwd_workspace_bytes(B, H, N, d);
    if (need > kScratchBytes) return AVION_ESCRATCH;
    void* ws = nullptr;
    const int rs = scratch_of_current_device(&ws);
    if (rs != AVION_OK) return rs;
    // every entry of the scratch that the second pass reads is written by the first one (padding
    // rows included), so nothing has to be cleared between calls
    return bwd_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, 1, Variant{false, false}, scale, ws, need, stream);
}

int avion_attn_fwd_causal(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                          float scale, void* stream)
{
    return fwd_impl(q, k, v, o, lse, B, H, N, d, 1, Variant{false, true}, scale, stream);
}

int avion_attn_bwd_causal(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                          void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, void* workspace,
                          size_t workspace_bytes, void* stream)
{
    return bwd_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, 1, Variant{false, true}, scale, workspace, workspace_bytes,
                    stream);
}

int avion_attn_fwd_f16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                       float scale, void* stream)
{
    return fwd_impl(q, k, v, o, lse, B, H, N, d, 1, Variant{true, false}, scale, stream);
}

int avion_attn_bwd_f16(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                       void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    return bwd_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, 1, Variant{true, false}, scale, workspace, workspace_bytes,
                    stream);
}

int avion_attn_bwd_qkvpacked(const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv, int B, int H,
                             int N, int d, float scale, void* workspace, size_t workspace_bytes, void* stream)
{
    return avion_attn_bwd_ex(qkv, nullptr, nullptr, o, lse, dO, dqkv, nullptr, nullptr, B, H, N, d, scale,
                             AVION_FLAG_QKVPACKED, workspace, workspace_bytes, stream);
}

int avion_attn_fwd_ex(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                      float scale, unsigned flags, void* stream)
{
    if (flags & ~kAllFlags) return AVION_EINVAL;
    const Variant var{(flags & AVION_FLAG_F16) != 0, (flags & AVION_FLAG_CAUSAL) != 0};
    if (flags & AVION_FLAG_QKVPACKED) {
        if (k || v || H < 1 || d < 1) return AVION_EINVAL;
        const Planes p(q, H, d);
        return fwd_impl(p.q, p.k, p.v, o, lse, B, H, N, d, 3, var, scale, stream);
    }
    return fwd_impl(q, k, v, o, lse, B, H, N, d, 1, var, scale, stream);
}

int avion_attn_bwd_ex(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                      void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, unsigned flags,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    if (flags & ~kAllFlags) return AVION_EINVAL;
    const Variant var{(flags & AVION_FLAG_F16) != 0, (flags & AVION_FLAG_CAUSAL) != 0};
    if (flags & AVION_FLAG_QKVPACKED) {
        if (k || v || dk || dv || !q || !dq || H < 1 || d < 1) return AVION_EINVAL;
        const Planes in(q, H, d), out(dq, H, d);
        return bwd_impl(in.q, in.k, in.v, o, lse, dO, const_cast<char*>(out.q), const_cast<char*>(out.k),
                        const_cast<char*>(out.v), B, H, N, d, 3, var, scale, workspace, workspace_bytes, stream);
    }
    return bwd_impl(q, k, v, o, lse, dO, dq, dk, dv, B, H, N, d, 1, var, scale, workspace, workspace_bytes, stream);
}

int avion_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y, float* mean, float* rstd,
                        long long M, int D, float eps, unsigned flags, void* stream)
{
    if (!x || !gamma || !beta || !y || !mean || !rstd) return AVION_EINVAL;
    if (!(eps >= 0.f) || !std::isfinite(eps)) return AVION_EINVAL;
    const int rc = ln_check(M, D, flags);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {x, gamma, beta, y, mean, rstd};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return ln_dispatch(D, (flags & AVION_FLAG_F16) != 0, [&](auto nch, auto fmt) {
        begin_launch();
        hipLaunchKernelGGL((avion_ln_fwd_kernel<decltype(nch)::value, typename decltype(fmt)::type>), dim3(ln_grid(M)),
                           dim3(kLnWaves * 64), 0, st, static_cast<const raw16*>(x), gamma, beta, static_cast<raw16*>(y), mean,
                           rstd, (long)M, D, eps);
        return end_launch("launch avion_ln_fwd_kernel");
    });
}

size_t avion_layernorm_bwd_workspace_bytes(long long M, int D)
{
    if (ln_check(M, D, 0) != AVION_OK) return 0;
    const size_t bytes = (size_t)ln_grid(M) * 2 * D * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

int avion_layernorm_bwd(const void* x, const float* gamma, const float* mean, const float* rstd, const void* dy, void* dx,
                        float* dgamma, float* dbeta, long long M, int D, unsigned flags, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    if (!x || !gamma || !mean || !rstd || !dy || !dx || !dgamma || !dbeta) return AVION_EINVAL;
    const int rc = ln_check(M, D, flags);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {x, gamma, mean, rstd, dy, dx, dgamma, dbeta};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
        workspace_bytes < avion_layernorm_bwd_workspace_bytes(M, D))
        return AVION_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* part = static_cast<float*>(workspace);
    const unsigned grid = ln_grid(M);
    const int r1 = ln_dispatch(D, (flags & AVION_FLAG_F16) != 0, [&](auto nch, auto fmt) {
        begin_launch();
        hipLaunchKernelGGL((avion_ln_bwd_kernel<decltype(nch)::value, typename decltype(fmt)::type>), dim3(grid),
                           dim3(kLnWaves * 64), (kLnWaves - 1) * 2 * D * sizeof(float), st, static_cast<const raw16*>(x), gamma,
                           mean, rstd, static_cast<const raw16*>(dy), static_cast<raw16*>(dx), part, (long)M, D);
        return end_launch("launch avion_ln_bwd_kernel");
    });
    if (r1 != AVION_OK) return r1;
    begin_launch();
    hipLaunchKernelGGL(avion_ln_param_reduce_kernel, dim3((2 * D + kLnReduceCols - 1) / kLnReduceCols),
                       dim3(kLnReduceCols * kLnReduceGroups), 0, st, part, dgamma, dbeta, (int)grid, D);
    return end_launch("launch avion_ln_param_reduce_kernel");
}

size_t avion_bias_gelu_bwd_workspace_bytes(long long M, int F)
{
    if (gelu_check(M, F, 0) != AVION_OK) return 0;
    const size_t bytes = (size_t)gelu_grid(M, F).nrg * F * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

int avion_bias_gelu_fwd(const void* x, const float* bias, void* y, long long M, int F, unsigned flags, void* stream)
{
    if (!x || !bias || !y) return AVION_EINVAL;
    const int rc = gelu_check(M, F, flags);
    if (rc != AVION_OK) return rc;
    if (!aligned16(x) || !aligned16(y) || !aligned16(bias)) return AVION_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const GeluGrid g = gelu_grid(M, F);
    const bool f16 = (flags & AVION_FLAG_F16) != 0, stream_past_cache = gelu_streams(M, F);
    auto launch = [&](auto fmt, auto streaming) {
        hipLaunchKernelGGL((avion_bias_gelu_fwd_kernel<typename decltype(fmt)::type, decltype(streaming)::value>),
                           dim3((unsigned)(g.ncb * g.nrg)), dim3(kGeluThreads), 0, st, static_cast<const raw16*>(x), bias,
                           static_cast<raw16*>(y), (long)M, F, g.ncb);
    };
    begin_launch();
    if (f16 && stream_past_cache) launch(TypeTag<F16>{}, std::true_type{});
    else if (f16) launch(TypeTag<F16>{}, std::false_type{});
    else if (stream_past_cache) launch(TypeTag<Bf16>{}, std::true_type{});
    else launch(TypeTag<Bf16>{}, std::false_type{});
    return end_launch("launch avion_bias_gelu_fwd_kernel");
}

int avion_bias_gelu_bwd(const void* x, const float* bias, const void* dy, void* dx, float* dbias, long long M, int F,
                        unsigned flags, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !bias || !dy || !dx || !dbias) return AVION_EINVAL;
    const int rc = gelu_check(M, F, flags);
    if (rc != AVION_OK) return rc;
    const void* ptrs[] = {x, bias, dy, dx, dbias};
    for (const void* p : ptrs)
        if (!aligned16(p)) return AVION_EUNSUPPORTED;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
        workspace_bytes < avion_bias_gelu_bwd_workspace_bytes(M, F))
        return AVION_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* part = static_cast<float*>(workspace);
    const GeluGrid g = gelu_grid(M, F);
    const bool f16 = (flags & AVION_FLAG_F16) != 0, stream_past_cache = gelu_streams(M, F);
    auto launch = [&](auto fmt, auto streaming) {
        hipLaunchKernelGGL((avion_bias_gelu_bwd_kernel<typename decltype(fmt)::type, decltype(streaming)::value>),
                           dim3((unsigned)(g.ncb * g.nrg)), dim3(kGeluThreads), 0, st, static_cast<const raw16*>(x), bias,
                           static_cast<const raw16*>(dy), static_cast<raw16*>(dx), part, (long)M, F, g.ncb);
    };
    begin_launch();
    if (f16 && stream_past_cache) launch(TypeTag<F16>{}, std::true_type{});
    else if (f16) launch(TypeTag<F16>{}, std::false_type{});
    else if (stream_past_cache) launch(TypeTag<Bf16>{}, std::true_type{});
    else launch(TypeTag<Bf16>{}, std::false_type{});
    const int r1 = end_launch("launch avion_bias_gelu_bwd_kernel");
    if (r1 != AVION_OK) return r1;
    // column sums of the row groups' partials: the reduction kernel splits its 2 * (F / 2) columns into two outputs
    begin_launch();
    hipLaunchKernelGGL(avion_ln_param_reduce_kernel, dim3((F + kLnReduceCols - 1) / kLnReduceCols),
                       dim3(kLnReduceCols * kLnReduceGroups), 0, st, part, dbias, dbias + F / 2, g.nrg, F / 2);
    return end_launch("launch avion_ln_param_reduce_kernel");
}

}  // extern "C"
