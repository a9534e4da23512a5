"""Pins for tests/rounded_chain.py, the control of the bf16 parity tests: with its roundings switched off it must be
the oracle's layer to fp64 rounding, and with them on it must sit at a bf16-sized distance from it."""
import dataclasses
import numpy as np

from oracle import share as oshare
from oracle import layout as olayout
from oracle.precision import round_to_bf16
from tests import rounded_chain as rc
from tests.harness import rel_errors
from workloads import CONFIGS, draw_layer_params, draw_activations


def small_case(causal):
    cfg = dataclasses.replace(CONFIGS["c2"], hidden=64, heads=4, mlp=256, seq=40, micro_batch=2, n_micro=2, causal=causal)
    t = draw_layer_params(cfg, perturbed=True)
    flat = round_to_bf16(olayout.flatten_layer(t, cfg.hidden, cfg.mlp, dtype=np.float32))
    x, dy = draw_activations(cfg)
    return cfg, flat, x.astype(np.float64), dy.astype(np.float64)


def test_chain_without_roundings_is_the_oracle(monkeypatch):
    monkeypatch.setattr(rc, "rb", lambda a: np.asarray(a, dtype=np.float64))
    monkeypatch.setattr(rc, "rh", lambda a: np.asarray(a, dtype=np.float64))
    for causal in (False, True):
        cfg, flat, x, dy = small_case(causal)
        ref = oshare.share_layer_step(flat, x, dy, cfg.hidden, cfg.mlp, cfg.heads, causal, cfg.micro_batch, scale=0.75)
        got = rc.share_layer_step(flat, x, dy, cfg.hidden, cfg.mlp, cfg.heads, causal, cfg.micro_batch, scale=0.75)
        for a, b in zip(got, ref):
            assert np.max(np.abs(a - b)) <= 1e-11 * np.max(np.abs(b))


def test_chain_with_roundings_is_a_bf16_distance_away():
    cfg, flat, x, dy = small_case(True)
    ref = oshare.share_layer_step(flat, x, dy, cfg.hidden, cfg.mlp, cfg.heads, True, cfg.micro_batch)
    got = rc.share_layer_step(flat, x, dy, cfg.hidden, cfg.mlp, cfg.heads, True, cfg.micro_batch)
    for a, b in zip(got, ref):
        mx, mean = rel_errors(a, b)
        assert 1e-5 < mean < 5e-3 and mx < 2e-2, (mx, mean)       # one to a dozen roundings of 2^-9 relative each
    assert np.array_equal(rc.rb(np.float32([1.00390625])), [1.0])             # ties to even, as the oracle's rounding
    assert rc.rh(np.float64([1.0 + 2.0 ** -12]))[0] == 1.0                      # half: 11 significand bits
