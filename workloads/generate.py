"""Seeded draws of the synthetic tensors.  Values only; nothing here knows how they are used.

Each named tensor is drawn from its own Philox stream keyed by (seed, crc32(name)), so a
tensor's values do not depend on the order or on which other tensors are drawn.
All results are float32 (token ids: int32) numpy arrays on the host.
"""
import zlib
import numpy as np

LAYER_TENSORS = (
    # name, shape as a function of (H, F), kind
    ("ln1_g", lambda H, F: (H,), "gamma"),
    ("ln1_b", lambda H, F: (H,), "zero"),
    ("w_qkv", lambda H, F: (3 * H, H), "weight"),
    ("b_qkv", lambda H, F: (3 * H,), "zero"),
    ("w_o", lambda H, F: (H, H), "weight"),
    ("b_o", lambda H, F: (H,), "zero"),
    ("ln2_g", lambda H, F: (H,), "gamma"),
    ("ln2_b", lambda H, F: (H,), "zero"),
    ("w_fc1", lambda H, F: (F, H), "weight"),
    ("b_fc1", lambda H, F: (F,), "zero"),
    ("w_fc2", lambda H, F: (H, F), "weight"),
    ("b_fc2", lambda H, F: (H,), "zero"),
)


LLAMA_TENSORS = (
    ("rms1_g", lambda H, F: (H,), "gamma"),
    ("w_qkv", lambda H, F: (3 * H, H), "weight"),
    ("w_o", lambda H, F: (H, H), "weight"),
    ("rms2_g", lambda H, F: (H,), "gamma"),
    ("w_gu", lambda H, F: (2 * F, H), "weight"),
    ("w_down", lambda H, F: (H, F), "weight"),
)


def _rng(seed, name):
    return np.random.Generator(np.random.Philox(key=[seed, zlib.crc32(name.encode())]))


def _normal(seed, name, shape, std, chunk=1 << 24):
    rng = _rng(seed, name)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = rng.standard_normal(e - s, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out.reshape(shape)


def draw_layer_params(cfg, layer_index=0, perturbed=False):
    """dict name -> float32 array.  Weights N(0, cfg.init_std^2) (0.02 unless the config says otherwise); biases 0; LN gamma 1, beta 0.

    perturbed=True shifts biases, gamma and beta by N(0, 0.02^2) draws so that a test
    can tell tensors (and their rows) apart; the plain form hides indexing mistakes.
    """
    H, F = cfg.hidden, cfg.mlp
    out = {}
    for name, shp, kind in (LLAMA_TENSORS if getattr(cfg, "kind", "gpt") == "llama" else LAYER_TENSORS):
        shape = shp(H, F)
        tag = "L%d.%s" % (layer_index, name)
        if kind == "weight":
            t = _normal(cfg.seed, tag, shape, getattr(cfg, "init_std", 0.02))
        else:
            t = np.zeros(shape, dtype=np.float32)
            if kind == "gamma":
                t += np.float32(1.0)
            if perturbed:
                t += _normal(cfg.seed, tag, shape, 0.02)
        out[name] = t
    return out


def draw_stack_params(cfg, perturbed=False):
    """Parameters of a full stack: wte [V,H], wpe [S,H], per-layer dicts, final LN (Llama-style: wte, layers, final
    RMSNorm gamma, w_head [V,H])."""
    H = cfg.hidden
    if getattr(cfg, "kind", "gpt") == "llama":          # token embedding, layers, final RMSNorm, a head of its own
        out = {
            "wte": _normal(cfg.seed, "wte", (cfg.vocab, H), 0.02),
            "layers": [draw_layer_params(cfg, i, perturbed) for i in range(cfg.layers)],
            "normf_g": np.ones((H,), dtype=np.float32),
            "w_head": _normal(cfg.seed, "w_head", (cfg.vocab, H), 0.02),
        }
        if perturbed:
            out["normf_g"] += _normal(cfg.seed, "normf_g", (H,), 0.02)
        return out
    out = {
        "wte": _normal(cfg.seed, "wte", (cfg.vocab, H), 0.02),
        "wpe": _normal(cfg.seed, "wpe", (cfg.seq, H), 0.02),
        "layers": [draw_layer_params(cfg, i, perturbed) for i in range(cfg.layers)],
        "lnf_g": np.ones((H,), dtype=np.float32),
        "lnf_b": np.zeros((H,), dtype=np.float32),
    }
    if perturbed:
        out["lnf_g"] += _normal(cfg.seed, "lnf_g", (H,), 0.02)
        out["lnf_b"] += _normal(cfg.seed, "lnf_b", (H,), 0.02)
    return out


def draw_activations(cfg, batch=None):
    """x and the upstream gradient dy, each N(0,1), shape [batch, S, H] (default: the whole share)."""
    b = cfg.batch_share if batch is None else batch
    shape = (b, cfg.seq, cfg.hidden)
    return _normal(cfg.seed, "x", shape, 1.0), _normal(cfg.seed, "dy", shape, 1.0)


def draw_token_ids(cfg, batch=None):
    """Input ids and target ids, uniform over the vocabulary, int32 [batch, S] each."""
    b = cfg.batch_share if batch is None else batch
    ids = _rng(cfg.seed, "ids").integers(0, cfg.vocab, size=(b, cfg.seq), dtype=np.int32)
    tgt = _rng(cfg.seed, "targets").integers(0, cfg.vocab, size=(b, cfg.seq), dtype=np.int32)
    return ids, tgt


def draw_adam_state(cfg, n, chunk=1 << 24):
    """Non-trivial Adam inputs for a mid-training step: gradient g ~ N(0, 1e-2^2),
    first moment m ~ N(0, 1e-2^2), second moment v = (1e-2 * N(0,1))^2 >= 0, each [n] float32."""
    g = _normal(cfg.seed, "adam_g", (n,), 1e-2, chunk)
    m = _normal(cfg.seed, "adam_m", (n,), 1e-2, chunk)
    v = _normal(cfg.seed, "adam_v", (n,), 1e-2, chunk)
    np.square(v, out=v)
    return g, m, v
