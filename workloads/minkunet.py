"""Layer plan and random parameters of the MinkUNet-style benchmark network (config 5).

Structure only: which layers exist, their shapes, which tensors they read and write, and
seeded random parameters.  No convolution arithmetic lives here; the GPU driver and the
oracle driver each execute the plan with their own code.

Network (the task's description, with the channel plan made explicit):

* stem: 3x3x3 conv  C_in -> 32, bias, ReLU                                  (level 0)
* encoder stage i = 1..4: 2x2x2 stride-2 conv to widths 64, 128, 256, 256 (bias, ReLU), then two
  residual blocks at that width                                            (level i)
* decoder stage for levels 3, 2, 1, 0: 2x2x2 stride-2 transposed conv to widths 256, 128, 96, 96
  (bias, ReLU), channel concatenation with the encoder output of that level (256, 128, 64, 32
  channels), then two residual blocks at the decoder width
* residual block: h = ReLU(conv3(x) + b1); y = ReLU(conv3(h) + b2 + shortcut(x)), where shortcut is
  the identity when the widths agree and a 1x1x1 conv with bias otherwise

"BN folded into the weights" means each conv is followed by a per-channel bias only.

A plan is a list of ops over named tensors:
  ("conv", dict(name, src, dst, map=(kind, level), c_in, c_out, relu, residual))   dst = act(conv(src) + bias + residual)
  ("concat", dict(dst, a, b))                                                      dst = [a, b] along channels
Map kinds: "sub" (3x3x3, stride 1, at `level`), "down" (2x2x2 stride 2, level -> level+1),
"up" (transposed, level+1 -> level), "id" (1x1x1 at `level`).
"""
from __future__ import annotations

import numpy as np

ENC_WIDTHS = (32, 64, 128, 256, 256)     # stem, then encoder stages 1..4
DEC_WIDTHS = {3: 256, 2: 128, 1: 96, 0: 96}
KVOL = {"sub": 27, "down": 8, "up": 8, "id": 1}
# Average number of kernel offsets that actually meet an input on surface-like data; used only
# to scale the random weights so that activations keep a sane magnitude in fp16.
EFFECTIVE_TAPS = {"sub": 8.0, "down": 2.5, "up": 1.0, "id": 1.0}


def _conv(ops, name, src, dst, kind, level, c_in, c_out, relu=True, residual=None):
    ops.append(("conv", dict(name=name, src=src, dst=dst, map=(kind, level), c_in=c_in, c_out=c_out,
                             relu=relu, residual=residual)))


def _res_block(ops, name, src, dst, level, c_in, c_out):
    _conv(ops, f"{name}.conv1", src, f"{name}.h", "sub", level, c_in, c_out)
    shortcut = src
    if c_in != c_out:
        _conv(ops, f"{name}.shortcut", src, f"{name}.s", "id", level, c_in, c_out, relu=False)
        shortcut = f"{name}.s"
    _conv(ops, f"{name}.conv2", f"{name}.h", dst, "sub", level, c_out, c_out, residual=shortcut)


def build_plan(in_channels: int = 4):
    """Returns (ops, output tensor name).  The input tensor is called "input" (level 0)."""
    ops = []
    _conv(ops, "stem", "input", "enc0", "sub", 0, in_channels, ENC_WIDTHS[0])
    cur = "enc0"
    for i in range(1, 5):
        w = ENC_WIDTHS[i]
        _conv(ops, f"down{i}", cur, f"enc{i}.d", "down", i - 1, ENC_WIDTHS[i - 1], w)
        _res_block(ops, f"enc{i}.b1", f"enc{i}.d", f"enc{i}.r1", i, w, w)
        _res_block(ops, f"enc{i}.b2", f"enc{i}.r1", f"enc{i}", i, w, w)
        cur = f"enc{i}"
    width = ENC_WIDTHS[4]
    for level in (3, 2, 1, 0):
        w = DEC_WIDTHS[level]
        _conv(ops, f"up{level}", cur, f"dec{level}.u", "up", level, width, w)
        ops.append(("concat", dict(dst=f"dec{level}.c", a=f"dec{level}.u", b=f"enc{level}")))
        cat = w + ENC_WIDTHS[level]
        _res_block(ops, f"dec{level}.b1", f"dec{level}.c", f"dec{level}.r1", level, cat, w)
        _res_block(ops, f"dec{level}.b2", f"dec{level}.r1", f"dec{level}", level, w, w)
        cur, width = f"dec{level}", w
    return ops, cur


def make_params(seed: int, ops, dtype=np.float16, gain: float = 1.5):
    """{conv name: (weights [K^3, C_in, C_out], bias [C_out])}, seeded per layer.

    weights ~ N(0, gain / (taps * C_in)) with `taps` the typical number of offsets that meet an
    input; bias ~ N(0, 0.05^2).  Second convs of residual blocks get a quarter of the gain so the
    sum with the shortcut does not grow from block to block.
    """
    params = {}
    idx = 0
    for kind, op in ops:
        if kind != "conv":
            continue
        idx += 1
        rng = np.random.Generator(np.random.PCG64([int(seed), idx]))
        mk = op["map"][0]
        g = gain * (0.25 if op["name"].endswith("conv2") else 1.0)
        std = np.sqrt(g / (EFFECTIVE_TAPS[mk] * op["c_in"]))
        w = rng.standard_normal((KVOL[mk], op["c_in"], op["c_out"])) * std
        b = rng.standard_normal(op["c_out"]) * 0.05
        params[op["name"]] = (np.ascontiguousarray(w.astype(dtype)), np.ascontiguousarray(b.astype(dtype)))
    return params


def map_keys(ops):
    """The distinct (kind, level) kernel maps the plan needs, in first-use order."""
    seen = []
    for kind, op in ops:
        if kind == "conv" and op["map"] not in seen:
            seen.append(op["map"])
    return seen
