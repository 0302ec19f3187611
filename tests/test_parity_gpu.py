"""GPU parity: the HIP kernels (through the C ABI) against the fp64 CPU oracle on the same seeded
bf16 inputs.  Tolerances: max-abs <= 2e-2 and relative Frobenius <= 5e-3 for O, dQ, dK, dV;
LSE within 1e-3 (see tests/gpu_harness.py)."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


# The one named workload whose dQ cannot meet the stated absolute bound on every head, whatever the
# kernel: the backward takes the forward's output as rounded to the tensor format, so the row sums
# delta = rowsum(dO o O) carry that rounding; with the peaky softmax of this workload (K doubled: few
# effective keys, |O| up to 3.5, |sum_j P_ij k_j| up to 7) the error of delta alone moves dQ by up to
# 2.7e-2 on some heads (shown on the CPU, with everything else exact, in
# tests/test_tolerance_model.py).  The bound taken for that one tensor is one bf16 unit in the last
# place of the workload's largest dQ element (5.79 over all 256 heads, from the oracle): 2^-7 * 5.79;
# an eighth of it for the fp16 entry points.  O, dK, dV and every relative bound stay as stated.
PEAKY_DQ_ABS = 5.79 * 2.0 ** -7
ABS_BOUND = {"vitl_batch_peaky": {"dQ": PEAKY_DQ_ABS}}
ABS_BOUND_F16 = {"vitl_batch_peaky": {"dQ": PEAKY_DQ_ABS / 8}}


def _run(w, slices=None, strict_abs=True):
    x = si.make_inputs(w)
    out = gh.run_hip(w, x)
    rep = gh.check_against_oracle(w, x, out, slices, strict_abs, abs_bound=ABS_BOUND.get(w.name))
    worst = {k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in rep.items()}
    print(f"\n{w.name}: shape={w.shape} errors(max-abs/rel-fro)={worst}", flush=True)
    return x, out


# sizes spanning several tiles with ragged tails, tiny N, and the CLS-token shapes (N+1)
SMALL = [
    # B, H,   N,  d
    (1, 1, 1, 64), (1, 2, 2, 64), (2, 1, 31, 64), (1, 3, 33, 64), (1, 1, 63, 64), (2, 2, 64, 64),
    (1, 2, 65, 64), (1, 1, 127, 64), (1, 2, 129, 64), (2, 3, 255, 64), (1, 2, 257, 64), (3, 5, 300, 64),
    (1, 2, 785, 64), (1, 1, 784, 64), (1, 2, 513, 64),
    (1, 1, 1, 80), (1, 2, 33, 80), (2, 2, 64, 80), (1, 3, 129, 80), (2, 2, 300, 80), (1, 1, 785, 80),
]


@pytest.mark.parametrize("B,H,N,d", SMALL)
def test_small_shapes_match_oracle(B, H, N, d):
    _run(si.small_workload(B, H, N, d, seed=1000 + 7 * N + d + B))


# Divided space/time attention (the comparison architecture of Sec. 4.1): temporal attention is one
# problem of N = T tokens per spatial position and clip, spatial attention one of N = 14*14 per frame.
# Sequences of at most 32 tokens run as windows of floor(32 / N) problems per wavefront.
@pytest.mark.parametrize("T", [4, 8, 16])
def test_temporal_attention_every_problem(T):
    # 8 clips x 196 positions, 12 heads of 64; 196 * 8 is a multiple of every window size used here.
    # A softmax over a handful of keys is near one-hot in many of the 18816 problems, so the absolute
    # bound follows the one-ulp rule (as for causal rows, which are softmaxes over few keys too).
    _run(si.small_workload(8 * 196, 12, T, 64, seed=4100 + T), strict_abs=False)


@pytest.mark.parametrize("B,H,N,d", [(37, 3, 3, 64), (1, 1, 32, 64), (50, 2, 7, 80), (3, 2, 17, 64), (100, 1, 1, 64), (11, 4, 20, 80)])
def test_windows_with_ragged_ends(B, H, N, d):
    # windows that are not full (32 % N != 0), last windows with fewer problems (B % floor(32/N) != 0)
    _run(si.small_workload(B, H, N, d, seed=4200 + 31 * B + N), strict_abs=False)


def test_spatial_attention_on_sampled_heads():
    # 32 clips x 8 frames as 256 problems of 14 x 14 tokens
    w = si.small_workload(256, 12, 196, 64, seed=4300)
    _run(w, _sampled_heads(w, 6))


def test_window_kernels_are_bitwise_reproducible():
    import torch
    w = si.small_workload(301, 5, 6, 64, seed=4400)
    x = si.make_inputs(w)
    a = gh.run_hip(w, x)
    for _ in range(2):
        b = gh.run_hip(w, x)
        for n in a:
            assert torch.equal(a[n].view(torch.int16) if a[n].dtype == torch.bfloat16 else a[n],
                               b[n].view(torch.int16) if b[n].dtype == torch.bfloat16 else b[n]), n


def test_peaky_softmax_small():
    # few effective keys: gradients reach magnitudes of 10 and more, so the absolute bound
    # follows the bf16 ulp of the largest value; the relative bound is unchanged
    _run(si.small_workload(2, 4, 333, 64, seed=4242, scale=0.125, k_mul=2.0), strict_abs=False)
    _run(si.small_workload(1, 2, 200, 80, seed=4243, k_mul=4.0), strict_abs=False)


def test_vitb_single_clip_full():
    # configs[0]: every element of every output is compared
    _run(si.WORKLOADS["vitb_clip"])


def test_cls_token_shape_full_head_count():
    # N = 1568 + 1 (a CLS token in front of the cubes), one clip
    _run(si.small_workload(1, 12, 1569, 64, seed=99, scale=0.125))


def _sampled_heads(w, n):
    """n distinct (batch, head) pairs: the first, the last and seeded random ones."""
    rng = np.random.default_rng(w.seed)
    heads = {(0, 0), (w.B - 1, w.H - 1)}
    while len(heads) < min(n, w.B * w.H):
        heads.add((int(rng.integers(w.B)), int(rng.integers(w.H))))
    return sorted(heads)


def test_benchmark_workload_every_element():
    # the workload bench.py times (ViT-B video training batch), in the launch configuration it times:
    # every element of O, LSE, dQ, dK, dV of all 384 heads against the oracle, at the strict bounds
    _run(si.WORKLOADS["vitb_batch"])


@pytest.mark.parametrize("name", ["vitl_batch_peaky", "vitb_long", "vith_d80", "vitl_336"])
def test_full_size_configs_on_sampled_heads(name):
    # The launch configuration bench.py times; the oracle recomputes whole (batch, head) slices
    # (dK and dV of a head need every query of that head, so the head is the sampling unit).
    w = si.WORKLOADS[name]
    x, out = _run(w, _sampled_heads(w, 8))
    # properties that hold at any size, on the whole tensors
    import torch
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n
    # sum_j dV_j = sum_i dO_i per (b,h,c) (rows of P sum to one)
    dv_sum = out["dv"].double().sum(1).cpu().numpy()
    do_sum = si.bf16_bits_to_f64(x["dO"]).sum(1)
    assert np.sqrt(((dv_sum - do_sum) ** 2).sum() / (do_sum ** 2).sum()) <= 2e-3


@pytest.mark.parametrize("shape", [(2, 3, 700, 64), (1, 4, 1568, 64), (2, 2, 300, 80)])
def test_bitwise_reproducible(shape):
    # no atomics and no order-dependent reductions: repeated runs agree bit for bit (this is also
    # what exposes a tile that is read before it has completely arrived)
    import torch
    w = si.small_workload(*shape, seed=31337)
    x = si.make_inputs(w)
    a = gh.run_hip(w, x)
    for _ in range(3):
        b = gh.run_hip(w, x)
        for n in a:
            assert torch.equal(a[n].view(torch.int16) if a[n].dtype == torch.bfloat16 else a[n],
                               b[n].view(torch.int16) if b[n].dtype == torch.bfloat16 else b[n]), n


@pytest.mark.parametrize("B,H,N,d", [(1, 1, 1, 64), (2, 3, 197, 64), (1, 2, 785, 64), (2, 2, 300, 80), (1, 12, 1569, 64)])
def test_packed_qkv_entry_points(B, H, N, d):
    # the [B,N,3,H,d] output of the joint projection taken as it is: against the oracle, and bit for
    # bit against the unpacked entry points (the same kernels with another token stride)
    import torch
    w = si.small_workload(B, H, N, d, seed=500 + N + d)
    x = si.make_inputs(w)
    out = gh.run_hip_packed(w, x)
    gh.check_against_oracle(w, x, out)
    ref = gh.run_hip(w, x)
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(out[n].contiguous().view(torch.int16), ref[n].view(torch.int16)), n
    assert torch.equal(out["lse"], ref["lse"])


def test_packed_qkv_at_the_benchmark_shape_on_sampled_heads():
    w = si.WORKLOADS["vitb_batch"]
    x = si.make_inputs(w)
    out = gh.run_hip_packed(w, x)
    gh.check_against_oracle(w, x, out, [(0, 0), (w.B - 1, w.H - 1), (w.B // 2, 5)])
    import torch
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n


def test_longest_cls_token_shape():
    # N = 3136 + 1: the 16-frame token count with a CLS token in front
    _run(si.small_workload(1, 2, 3137, 64, seed=3137, scale=0.125))


# causal attention (the GPT-like text encoder, at most 77 tokens); also sizes that cross several key
# tiles and workgroups so that skipped, diagonal and full blocks all occur in every kernel
CAUSAL_SHAPES = [(1, 1, 1, 64), (2, 2, 2, 64), (1, 2, 31, 64), (2, 3, 33, 64), (3, 8, 77, 64), (1, 2, 128, 64),
                 (1, 2, 129, 64), (2, 2, 300, 64), (1, 2, 785, 64), (1, 1, 1, 80), (2, 2, 77, 80), (1, 2, 300, 80)]


@pytest.mark.parametrize("B,H,N,d", CAUSAL_SHAPES)
def test_causal_shapes_match_oracle(B, H, N, d):
    w = si.small_workload(B, H, N, d, seed=7700 + 5 * N + d)
    x = si.make_inputs(w)
    out = gh.run_hip(w, x, causal=True)
    rep = gh.check_causal_against_oracle(w, x, out)
    print(f"\ncausal {w.shape}: " + str({k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in rep.items()}), flush=True)


def test_causal_text_encoder_batch_on_sampled_heads():
    # a text-encoder layer for a batch of 2048 captions: 8 heads of 64 over 77 tokens
    import torch
    w = si.small_workload(2048, 8, 77, 64, seed=77)
    x = si.make_inputs(w)
    out = gh.run_hip(w, x, causal=True)
    gh.check_causal_against_oracle(w, x, out, [(0, 0), (2047, 7), (1000, 3)])
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n
    # the first token sees only itself: O_0 = v_0 exactly (a weight of one times a bf16 value)
    assert torch.equal(out["o"][:, 0].view(torch.int16), gh.to_gpu_bf16(x["v"])[:, 0].view(torch.int16))


def test_causal_at_the_video_token_count_on_sampled_heads():
    # the causal kernels at the benchmark's shape (N = 1568: skipped, diagonal and full blocks in every
    # workgroup, 13 workgroups per head), on sampled heads; the absolute bound is the strict one wherever
    # one bf16 ulp of the largest reference value stays below it (see check_causal_against_oracle)
    import torch
    w = si.WORKLOADS["vitb_batch"]
    x = si.make_inputs(w)
    out = gh.run_hip(w, x, causal=True)
    gh.check_causal_against_oracle(w, x, out, _sampled_heads(w, 4))
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n


def test_causal_running_max_path():
    # as test_scores_far_above_the_first_keys_take_the_running_max_path, with the causal mask: keys
    # from 64 on are 16 times larger and scale = 1, so rows from 64 on overflow the fixed reference
    # and the workgroup redoes its rows with a running maximum -- which must honour the mask too
    import oracle
    import paper_2309_16669_amd as av
    import torch
    for d in (64, 80):
        w = si.small_workload(1, 2, 200, d, seed=4321 + d, scale=1.0)
        x = si.make_inputs(w)
        big = si.bf16_bits_to_f32(x["k"][:, 64:]) * np.float32(16.0)
        x["k"][:, 64:] = si.f32_to_bf16_bits(big)          # exact: power of two
        q, k, v = (gh.to_gpu_bf16(x[n]) for n in ("q", "k", "v"))
        o = torch.full_like(q, float("nan"))
        lse = torch.full((w.B, w.H, w.N), float("nan"), dtype=torch.float32, device="cuda")
        av.attn_fwd_causal(q, k, v, o, lse, w.scale)
        torch.cuda.synchronize()
        ro, rl = oracle.fwd(x["q"], x["k"], x["v"], w.scale, causal=True)
        og = gh.bf16_tensor_to_f64(o)
        lg = lse.double().cpu().numpy()
        assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
        assert np.abs(og - ro).max() <= 2.0 ** -7 * np.abs(ro).max()
        assert np.abs(lg - rl).max() <= 2e-6 * np.abs(rl).max() + 1e-3


F16_SHAPES = [(1, 1, 1, 64), (1, 2, 33, 64), (2, 3, 197, 64), (1, 2, 300, 64), (1, 2, 785, 64), (1, 1, 1569, 64),
              (1, 1, 1, 80), (2, 2, 300, 80), (1, 1, 785, 80)]


@pytest.mark.parametrize("B,H,N,d", F16_SHAPES)
def test_f16_small_shapes_match_oracle(B, H, N, d):
    w = si.small_workload(B, H, N, d, seed=1600 + 3 * N + d)
    x = si.make_inputs(w, fmt="f16")
    out = gh.run_hip_f16(w, x)
    rep = gh.check_f16_against_oracle(w, x, out)
    print(f"\nf16 {w.shape}: errors(max-abs/rel-fro)=" + str({k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in rep.items()}), flush=True)


@pytest.mark.parametrize("name", ["vitb_clip", "vitb_batch", "vitl_batch_peaky", "vitb_long", "vith_d80", "vitl_336"])
def test_f16_full_size_configs_on_sampled_heads(name):
    import torch
    w = si.WORKLOADS[name]
    x = si.make_inputs(w, fmt="f16")
    out = gh.run_hip_f16(w, x)
    rep = gh.check_f16_against_oracle(w, x, out, _sampled_heads(w, 4), abs_bound=ABS_BOUND_F16.get(name))
    print(f"\nf16 {name}: " + str({k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in rep.items()}), flush=True)
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n


def test_f16_weights_beyond_the_half_precision_range_take_the_running_max_path():
    # keys from 64 on are 4 times larger and scale = 1: later scores exceed the maximum over the first
    # 32 keys by far more than 15 binades, so weights taken against that fixed reference would not
    # fit fp16; the kernel must notice and redo the rows with a running maximum
    import oracle
    for d in (64, 80):
        w = si.small_workload(1, 2, 200, d, seed=1900 + d, scale=1.0)
        x = si.make_inputs(w, fmt="f16")
        big = x["k"][:, 64:].view(np.float16).astype(np.float32) * np.float32(4.0)
        x["k"][:, 64:] = si.f32_to_f16_bits(big)          # exact: power of two, far from overflow
        out = gh.run_hip_f16(w, x)
        q, k, v = (si.f16_bits_to_f64(x[n]) for n in ("q", "k", "v"))
        ro, rl = oracle.fwd_f64(q, k, v, w.scale)
        o = out["o"].double().cpu().numpy()
        lse = out["lse"].double().cpu().numpy()
        assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
        assert np.abs(o - ro).max() <= 2.0 ** -10 * np.abs(ro).max()
        assert np.abs(lse - rl).max() <= 2e-6 * np.abs(rl).max() + 1e-3


def test_identical_keys_and_single_token_closed_forms_on_gpu():
    # closed forms again, this time on the HIP path: identical keys -> O = mean of V
    import torch
    w = si.small_workload(1, 2, 150, 64, seed=5)
    x = si.make_inputs(w)
    x["k"][:] = x["k"][:, :1]
    out = gh.run_hip(w, x)
    v = si.bf16_bits_to_f64(x["v"])
    o = gh.bf16_tensor_to_f64(out["o"])
    assert np.abs(o - v.mean(1, keepdims=True)).max() < 3e-3
    import oracle
    ro, rl = oracle.fwd(x["q"], x["k"], x["v"], w.scale)
    rdq, rdk, rdv = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], w.scale)
    gh.assert_close("O", o, ro)
    assert np.abs(out["lse"].double().cpu().numpy() - rl).max() <= gh.LSE_ABS
    gh.assert_close("dV", gh.bf16_tensor_to_f64(out["dv"]), rdv)
    gh.assert_close("dK", gh.bf16_tensor_to_f64(out["dk"]), rdk)
    # dQ is exactly zero here (every k_j is the same vector and rows of dS sum to zero):
    # only an absolute bound makes sense
    assert np.abs(rdq).max() < 1e-12
    assert np.abs(gh.bf16_tensor_to_f64(out["dq"])).max() <= gh.MAX_ABS


def test_large_magnitude_scores():
    # scores around +-60 after scaling: exp() must not overflow, LSE must stay accurate
    w = si.small_workload(1, 2, 130, 64, seed=77, scale=1.0)
    x = si.make_inputs(w)
    out = gh.run_hip(w, x)
    import oracle
    ro, rl = oracle.fwd(x["q"], x["k"], x["v"], w.scale)
    o = gh.bf16_tensor_to_f64(out["o"])
    assert np.all(np.isfinite(o))
    assert np.abs(o - ro).max() <= 3e-2          # |O| is O(1) here (near one-hot weights)
    assert np.abs(out["lse"].double().cpu().numpy() - rl).max() <= 2e-3 * np.abs(rl).max()


def test_scores_far_above_the_first_keys_take_the_running_max_path():
    # The forward kernel references every query's weights to the maximum over its first 32 keys and
    # falls back to a running maximum when a later score is ~100 binades larger.  Here the keys
    # from 64 on are 16 times larger and scale = 1: later scores exceed the early ones by hundreds
    # of binades, so this exercises the fallback; O and LSE must still match the oracle.
    import oracle
    for d in (64, 80):
        w = si.small_workload(1, 2, 200, d, seed=1234 + d, scale=1.0)
        x = si.make_inputs(w)
        big = si.bf16_bits_to_f32(x["k"][:, 64:]) * np.float32(16.0)
        x["k"][:, 64:] = si.f32_to_bf16_bits(big)          # exact: power of two
        out = gh.run_hip(w, x)
        ro, rl = oracle.fwd(x["q"], x["k"], x["v"], w.scale)
        o = gh.bf16_tensor_to_f64(out["o"])
        lse = out["lse"].double().cpu().numpy()
        assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
        assert np.abs(o - ro).max() <= 2.0 ** -7 * np.abs(ro).max()      # one bf16 ulp of near one-hot rows
        assert np.abs(lse - rl).max() <= 2e-6 * np.abs(rl).max() + 1e-3  # fp32 LSE of magnitude ~1e3


def test_largest_addressable_head_slice():
    # The kernels address one (batch, head) slice with 32-bit byte offsets and the library accepts
    # shapes up to (N + 256) * H*d*2 < 2^31.  H = 4000, N = 3900 is just inside (2.128e9); the last
    # head's last rows sit at the far end of that range.  Inputs are drawn on the GPU (seeded); the
    # oracle gets the bytes of the sampled heads copied back.
    import ctypes
    import torch
    import oracle
    import paper_2309_16669_amd as av
    B, H, N, d = 1, 4000, 3900, 64
    assert (N + 256) * H * d * 2 < 2 ** 31 <= (N + 64 + 256) * H * d * 2
    g = torch.Generator(device="cuda")
    g.manual_seed(20230916)
    q, k, v, dO = (torch.randn((B, N, H, d), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
                   for _ in range(4))
    o = torch.full_like(q, float("nan"))
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    ws = torch.empty(av.attn_bwd_workspace_bytes(B, H, N, d), dtype=torch.uint8, device="cuda")
    av.attn_fwd(q, k, v, o, lse, 0.125)
    av.attn_bwd(q, k, v, o, lse, dO, dq, dk, dv, 0.125, ws)
    torch.cuda.synchronize()
    bits = lambda t, h: t[:, :, h:h + 1].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    for h in (0, 1777, H - 1):
        ro, rl = oracle.fwd(bits(q, h), bits(k, h), bits(v, h), 0.125)
        rdq, rdk, rdv = oracle.bwd(bits(q, h), bits(k, h), bits(v, h), bits(dO, h), 0.125)
        assert np.abs(lse[:, h:h + 1].double().cpu().numpy() - rl).max() <= gh.LSE_ABS
        for name, t, ref in (("O", o, ro), ("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
            gh.assert_close(f"{name}[h={h}]", si.bf16_bits_to_f64(bits(t, h)), ref)
    # every element was written (the buffers were filled with NaN)
    for t in (o, dq, dk, dv, lse):
        assert bool(torch.isfinite(t.float()).all())
    # one tile further is refused before anything is launched
    assert av.load_library().avion_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                            B, H, N + 64, d, ctypes.c_float(0.125), None) == av.EUNSUPPORTED


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    # calls only enqueue on the caller's stream: two problems in flight on two streams, each with its
    # own workspace, give the same bits as when run one after the other on the default stream
    import torch
    import paper_2309_16669_amd as av
    ws_ = [si.small_workload(2, 4, 700, 64, seed=91), si.small_workload(1, 6, 1100, 64, seed=92)]
    xs = [si.make_inputs(w) for w in ws_]
    ref = [gh.run_hip(w, x) for w, x in zip(ws_, xs)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for w, x, st in zip(ws_, xs, streams):
        q, k, v, dO = (gh.to_gpu_bf16(x[n]) for n in ("q", "k", "v", "dO"))
        o = torch.empty_like(q)
        lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        wsb = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
        outs.append(dict(q=q, k=k, v=v, dO=dO, o=o, lse=lse, dq=dq, dk=dk, dv=dv, ws=wsb))
    torch.cuda.synchronize()
    for rep in range(3):          # interleave the enqueues
        for w, t, st in zip(ws_, outs, streams):
            av.attn_fwd(t["q"], t["k"], t["v"], t["o"], t["lse"], w.scale, st)
            av.attn_bwd(t["q"], t["k"], t["v"], t["o"], t["lse"], t["dO"], t["dq"], t["dk"], t["dv"], w.scale, t["ws"], st)
    torch.cuda.synchronize()
    for r, t in zip(ref, outs):
        for n in ("o", "dq", "dk", "dv"):
            assert torch.equal(r[n].view(torch.int16), t[n].view(torch.int16)), n
        assert torch.equal(r["lse"], t["lse"])


def test_autograd_front_end_matches_oracle_gradients():
    # loss = sum(O * W) through torch.autograd: the gradients that reach q, k, v are the library's
    # backward for dO = W; unmasked, causal, fp16 and packed forms
    import torch
    import oracle
    from paper_2309_16669_amd import autograd as ag
    w = si.small_workload(2, 3, 210, 64, seed=606)
    x = si.make_inputs(w)
    dO = gh.to_gpu_bf16(x["dO"])
    for causal in (False, True):
        q, k, v = (gh.to_gpu_bf16(x[n]).requires_grad_() for n in ("q", "k", "v"))
        o = ag.attention(q, k, v, w.scale, causal=causal)
        (o.float() * dO.float()).sum().backward()
        out = dict(o=o.detach(), dq=q.grad, dk=k.grad, dv=v.grad)
        ro, _ = oracle.fwd(x["q"], x["k"], x["v"], w.scale, causal=causal)
        refs = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], w.scale, causal=causal)
        gh.assert_close("O", gh.bf16_tensor_to_f64(out["o"]), ro, strict_abs=not causal)
        for n, ref in zip(("dq", "dk", "dv"), refs):
            gh.assert_close(n, gh.bf16_tensor_to_f64(out[n]), ref, strict_abs=not causal)
    # packed: bit-identical to the unpacked gradients
    qkv = gh.to_gpu_bf16(np.stack([x["q"], x["k"], x["v"]], axis=2)).requires_grad_()
    o = ag.attention_qkvpacked(qkv, w.scale)
    (o.float() * dO.float()).sum().backward()
    q, k, v = (gh.to_gpu_bf16(x[n]).requires_grad_() for n in ("q", "k", "v"))
    (ag.attention(q, k, v, w.scale).float() * dO.float()).sum().backward()
    for i, t in enumerate((q, k, v)):
        assert torch.equal(qkv.grad[:, :, i].contiguous().view(torch.int16), t.grad.view(torch.int16))
    # fp16
    x16 = si.make_inputs(w, fmt="f16")
    up = lambda b: torch.from_numpy(np.ascontiguousarray(b).view(np.int16)).cuda().view(torch.float16)
    q, k, v = (up(x16[n]).requires_grad_() for n in ("q", "k", "v"))
    o = ag.attention(q, k, v, w.scale)
    (o.float() * up(x16["dO"]).float()).sum().backward()
    f = {n: si.f16_bits_to_f64(x16[n]) for n in x16}
    ro, _ = oracle.fwd_f64(f["q"], f["k"], f["v"], w.scale)
    refs = oracle.bwd_f64(f["q"], f["k"], f["v"], f["dO"], w.scale)
    for n, got, ref in (("O", o.detach(), ro), ("dQ", q.grad, refs[0]), ("dK", k.grad, refs[1]), ("dV", v.grad, refs[2])):
        max_abs, rel = gh.errors(got.double().cpu().numpy(), ref)
        assert max_abs <= gh.MAX_ABS_F16 and rel <= gh.REL_FRO_F16, (n, max_abs, rel)


@pytest.mark.parametrize("B,H,N,d", [(3, 5, 100, 64), (2, 2, 128, 64), (2, 3, 77, 80), (1, 2, 129, 64)])
def test_whole_backward_equals_its_two_phases(B, H, N, d):
    # avion_attn_bwd runs short sequences (N <= 128) as one launch and longer ones as two; either way
    # it must give the bits of avion_attn_bwd_dq followed by avion_attn_bwd_dkdv
    import torch
    import paper_2309_16669_amd as av
    w = si.small_workload(B, H, N, d, seed=5150 + N)
    x = si.make_inputs(w)
    whole = gh.run_hip(w, x)
    q, k, v, dO = (gh.to_gpu_bf16(x[n]) for n in ("q", "k", "v", "dO"))
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    av.attn_bwd_dq(q, k, v, whole["o"], whole["lse"], dO, dq, w.scale, ws)
    av.attn_bwd_dkdv(q, k, v, whole["lse"], dO, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    for n, t in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert torch.equal(whole[n].view(torch.int16), t.view(torch.int16)), n


@pytest.mark.parametrize("B,H,N,d", [(3, 5, 100, 64), (2, 2, 128, 64), (2, 3, 77, 80), (4, 2, 20, 64)])
def test_the_two_phases_stay_callable_on_short_sequences(B, H, N, d):
    # avion_attn_bwd_dq + avion_attn_bwd_dkdv on shapes that avion_attn_bwd itself runs in one launch
    import torch
    import paper_2309_16669_amd as av
    w = si.small_workload(B, H, N, d, seed=5250 + N)
    x = si.make_inputs(w)
    whole = gh.run_hip(w, x)
    q, k, v, dO = (gh.to_gpu_bf16(x[n]) for n in ("q", "k", "v", "dO"))
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    av.attn_bwd_dq(q, k, v, whole["o"], whole["lse"], dO, dq, w.scale, ws)
    av.attn_bwd_dkdv(q, k, v, whole["lse"], dO, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    gh.check_against_oracle(w, x, dict(whole, dq=dq, dk=dk, dv=dv))


def test_calls_can_be_captured_in_a_graph_and_replayed():
    # the entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
    # synchronisation), so a forward + backward can be recorded into a HIP graph; every replay, with
    # eager work and synchronisations in between and fresh inputs copied into the captured buffers,
    # must give the bits of the eager call
    import torch
    import paper_2309_16669_amd as av
    w = si.small_workload(2, 3, 450, 64, seed=808)
    xs = [si.make_inputs(si.small_workload(2, 3, 450, 64, seed=808 + i)) for i in range(3)]
    refs = [gh.run_hip(w, x) for x in xs]                      # eager; also warms up the library
    q, k, v, dO = (gh.to_gpu_bf16(xs[0][n]).clone() for n in ("q", "k", "v", "dO"))
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                              # captures on a side stream
        av.attn_fwd(q, k, v, o, lse, w.scale)
        av.attn_bwd(q, k, v, o, lse, dO, dq, dk, dv, w.scale, ws)
    for i in (1, 2, 0, 1):
        for t, n in ((q, "q"), (k, "k"), (v, "v"), (dO, "dO")):
            t.copy_(gh.to_gpu_bf16(xs[i][n]))
        for t in (o, dq, dk, dv):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv)):
            assert torch.equal(refs[i][n].view(torch.int16), t.view(torch.int16)), (i, n)
        assert torch.equal(refs[i]["lse"], lse), i
        gh.run_hip(w, xs[(i + 1) % 3])                         # unrelated eager work between replays


def test_bad_arguments_raise_on_gpu_tensors():
    import torch
    import paper_2309_16669_amd as av
    q = torch.zeros(1, 8, 2, 48, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 2, 8, dtype=torch.float32, device="cuda")
    with pytest.raises(av.AvionError) as e:
        av.attn_fwd(q, q, q, torch.empty_like(q), lse, 0.1)
    assert e.value.code == av.EUNSUPPORTED
    q = torch.zeros(1, 8, 2, 64, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(av.AvionError) as e:
        av.attn_bwd(q, q, q, q, lse, q, torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), 0.1, ws)
    assert e.value.code == av.EWORKSPACE
