"""Oracle-side execution of a layer plan: the CPU oracle per conv, numpy for the elementwise steps.

Activations are rounded to the I/O dtype at the same two points as on the GPU (after the
convolution, after bias/residual/ReLU), so the two runs differ only by accumulation order.
Nothing here touches the GPU library.
"""
import numpy as np

import oracle


def level_coords(coords, top):
    levels = {0: np.asarray(coords, np.int32)}
    for level in range(top):
        levels[level + 1] = oracle.out_coords(levels[level], 2, 2)
    return levels


def run_plan(ops, output, params, coords, feats, dtype=np.float16, hook=None):
    top = max(op["map"][1] + (1 if op["map"][0] in ("down", "up") else 0) for k, op in ops if k == "conv")
    levels = level_coords(coords, top)
    t = {"input": np.asarray(feats, dtype)}
    for kind, op in ops:
        if kind == "concat":
            t[op["dst"]] = np.concatenate([t[op["a"]], t[op["b"]]], axis=1)
        else:
            w, b = params[op["name"]]
            mk, level = op["map"]
            x = t[op["src"]]
            if mk == "sub":
                _, y = oracle.conv(levels[level], x, w, 3, 1)
            elif mk == "id":
                _, y = oracle.conv(levels[level], x, w, 1, 1)
            elif mk == "down":
                _, y = oracle.conv(levels[level], x, w, 2, 2)
            else:
                _, y = oracle.conv_transposed(levels[level], x, w, 2, 2)
            y = y.astype(dtype).astype(np.float64)                 # the conv kernel stores in the I/O dtype
            y = y + b.astype(np.float64)[None, :]
            if op["residual"]:
                y = y + t[op["residual"]].astype(np.float64)
            if op["relu"]:
                y = np.maximum(y, 0.0)
            t[op["dst"]] = y.astype(dtype)
        if hook:
            hook(op["dst"], t[op["dst"]])
    return t[output], levels
