"""Flat layout of an FSDP unit (Sec. 3.1: a unit's parameters are managed as one buffer).

The paper does not give the order inside a unit.  The order used here, per transformer
layer, with every matrix stored [out_features, in_features] row-major and no padding:

    ln1.gamma[H] ln1.beta[H] W_qkv[3H,H] b_qkv[3H] W_o[H,H] b_o[H]
    ln2.gamma[H] ln2.beta[H] W_fc1[F,H] b_fc1[F] W_fc2[H,F] b_fc2[H]

A full stack is  wte[V,H]  wpe[S,H]  layer 0 .. layer L-1  lnf.gamma[H]  lnf.beta[H].
A shard [offset, offset+len) may begin and end anywhere, including inside a matrix.
"""
import numpy as np

LAYER_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def layer_shapes(H, F):
    return {"ln1_g": (H,), "ln1_b": (H,), "w_qkv": (3 * H, H), "b_qkv": (3 * H,),
            "w_o": (H, H), "b_o": (H,), "ln2_g": (H,), "ln2_b": (H,),
            "w_fc1": (F, H), "b_fc1": (F,), "w_fc2": (H, F), "b_fc2": (H,)}


def layer_param_count(H, F):
    return sum(int(np.prod(s)) for s in layer_shapes(H, F).values())


def layer_offsets(H, F):
    """name -> (start, shape) inside one layer's flat buffer."""
    shapes, out, pos = layer_shapes(H, F), {}, 0
    for name in LAYER_ORDER:
        out[name] = (pos, shapes[name])
        pos += int(np.prod(shapes[name]))
    return out


def flatten_layer(tensors, H, F, dtype=np.float64):
    flat = np.empty(layer_param_count(H, F), dtype=dtype)
    for name, (start, shape) in layer_offsets(H, F).items():
        n = int(np.prod(shape))
        flat[start:start + n] = np.asarray(tensors[name], dtype=dtype).reshape(-1)
    return flat


def unflatten_layer(flat, H, F):
    out = {}
    for name, (start, shape) in layer_offsets(H, F).items():
        n = int(np.prod(shape))
        out[name] = flat[start:start + n].reshape(shape)
    return out


def stack_param_count(H, F, S, V, L):
    return V * H + S * H + L * layer_param_count(H, F) + 2 * H


def stack_offsets(H, F, S, V, L):
    """Ordered list of (name, start, shape); layer tensors are named 'L<i>.<tensor>'."""
    out, pos = [], 0
    out.append(("wte", pos, (V, H))); pos += V * H
    out.append(("wpe", pos, (S, H))); pos += S * H
    for i in range(L):
        for name, (start, shape) in layer_offsets(H, F).items():
            out.append(("L%d.%s" % (i, name), pos + start, shape))
        pos += layer_param_count(H, F)
    out.append(("lnf_g", pos, (H,))); pos += H
    out.append(("lnf_b", pos, (H,))); pos += H
    return out


def flatten_stack(params, H, F, S, V, L, dtype=np.float64):
    flat = np.empty(stack_param_count(H, F, S, V, L), dtype=dtype)
    for name, start, shape in stack_offsets(H, F, S, V, L):
        n = int(np.prod(shape))
        if name.startswith("L"):
            li, tn = name.split(".")
            src = params["layers"][int(li[1:])][tn]
        else:
            src = params[name]
        flat[start:start + n] = np.asarray(src, dtype=dtype).reshape(-1)
    return flat


def state_bytes(n_elements):
    """Training-state bytes of n fp32 parameters under Adam: 4 (param) + 4 (grad) + 8 (two
    moments) per element (Sec. 3.3, memory utilization model)."""
    return 16 * n_elements
