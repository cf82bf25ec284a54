"""Runs a layer plan (see ``workloads/minkunet.py``) on the GPU through the C-ABI binding.

Only sequencing lives here: kernel maps per resolution level, one ``ts_sparse_conv_prepared`` per conv op,
bias / residual / ReLU in the layer kernel's epilogue.  A skip connection's concatenation is not formed:
the layers that take it read its two parts in place (``ts_sparse_conv_prepared2``); ``ts_concat_cols`` runs
only if something other than a conv asks for the concatenated tensor (a hook, the network's output).  Maps are
built once per (kind, level) and reused by every layer that needs them (the paper builds maps
per downsampling block, Sec. 2.3).
"""
from __future__ import annotations

import torch

from . import binding as ts


class SparseNet:
    def __init__(self, ops, output, params):
        """ops/output from the plan; params: {name: (weights, bias)} as device tensors."""
        self.ops, self.output, self.params = ops, output, params
        # weights do not change between passes: repack them for the kernels once
        self.prepared = {name: ts.ts_weights_prepare(w) for name, (w, _) in params.items()}

    def build_maps(self, coords: torch.Tensor, sort_rows: bool = False, box=None):
        """Kernel maps for every (kind, level) of the plan, plus the coordinates of each level.
        With ``sort_rows`` the 3x3x3 maps, which serve 4 to 9 layers each, get their output rows
        ordered by offset bitmask (``ts_kmap_sort_rows``).  ``box`` = (lo[3], hi[3], batches), the
        voxel grid the coordinates were quantised to, if the caller knows it: every build then
        searches through the coordinate grid (Sec. 4.4) over the box of its level (halved per
        level), and the strided builds need not measure theirs."""
        kinds = []
        for k, op in self.ops:
            if k == "conv" and op["map"] not in kinds:
                kinds.append(op["map"])
        levels = {0: coords}
        boxes = {0: box}
        maps = {}
        top = max(level for _, level in kinds)
        hint = None     # where a level's points can lie, as the strided build of the level above bounded them
        for level in range(top + 1):
            if ("down", level) in kinds or ("up", level) in kinds:
                down = ts.ts_build_kmap(levels[level], 2, 2, False, wait=False, grid=boxes[level],
                                        box=hint if boxes[level] is None else None)
                maps[("down", level)] = down
                levels[level + 1] = down.out_coords()
                hint = down.out_box()     # the next strided build need not measure its box
                b = boxes[level]
                boxes[level + 1] = None if b is None else (tuple(v // 2 for v in b[0]), tuple(v // 2 for v in b[1]), b[2])
        for kind, level in kinds:
            if kind == "sub":
                maps[(kind, level)] = ts.ts_build_kmap(levels[level], 3, 1, False, wait=False, grid=boxes.get(level))
                if sort_rows:
                    maps[(kind, level)].sort_rows()
            elif kind == "id":
                # a 1x1x1 convolution takes input k to output k whatever the coordinates are; that the points of
                # the level are distinct is checked by the other builds on them
                maps[(kind, level)] = ts.ts_identity_kmap(levels[level].shape[0])
            elif kind == "up":
                maps[(kind, level)] = maps[("down", level)].transpose()
        for m in maps.values():
            # The put-off part of a build gives the fetch-on-demand dataflow its per-offset counts and ranks
            # (wide layers on small maps) and the fused kernel its tile order, longest tiles first, which is
            # worth 5 to 12 % of a layer on the full-resolution maps: these maps serve 4 to 9 layers each.
            m.prepare()
        for m in maps.values():
            m.status()      # builds did not wait one by one; bad coordinates are reported here
        return maps, levels

    def forward(self, maps, feats: torch.Tensor, hook=None):
        """Executes the plan; ``hook(name, tensor)`` (optional) sees every tensor written (and makes every
        concatenation materialise, since it asks for the tensor)."""
        t = {"input": feats}
        parts = {}          # name of a concatenation -> its two source tensors; formed only on demand

        def whole(name):
            if name not in t:
                a, b = parts[name]
                t[name] = ts.ts_concat_cols(a, b)
            return t[name]

        for kind, op in self.ops:
            if kind == "concat":
                parts[op["dst"]] = (whole(op["a"]), whole(op["b"]))
            else:
                _, b = self.params[op["name"]]
                res = whole(op["residual"]) if op["residual"] else None
                if op["src"] in parts and op["src"] not in t:
                    xa, xb = parts[op["src"]]
                    t[op["dst"]] = ts.ts_sparse_conv_prepared2(xa, xb, self.prepared[op["name"]], maps[op["map"]], b, res,
                                                               op["relu"])
                else:
                    t[op["dst"]] = ts.ts_sparse_conv_prepared(whole(op["src"]), self.prepared[op["name"]], maps[op["map"]],
                                                              b, res, op["relu"])
            if hook:
                hook(op["dst"], whole(op["dst"]))
        return whole(self.output)

    def capture(self, maps, feats: torch.Tensor):
        """Records one forward pass into a HIP graph and returns (graph, input buffer, output).

        The forward pass is a fixed sequence of launches with no host synchronisation, so the
        host cost of ~50 library calls per pass (it exceeds the device time on the coarse
        levels) is paid once.  One eager pass runs first so that every scratch area of the
        library has its final size: nothing may allocate while the stream is being captured.
        Replay with ``graph.replay()`` after copying new features into the input buffer.
        """
        static_in = feats.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.forward(maps, static_in)          # sizes the library's scratch areas
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            static_out = self.forward(maps, static_in)
        return graph, static_in, static_out

    @staticmethod
    def free_maps(maps):
        for m in maps.values():
            m.free()
