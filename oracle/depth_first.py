"""Depth-first replay of a layer stack on the CPU -- TEST INFRASTRUCTURE.

Figure 3 of the paper: instead of finishing a layer over the whole tensor, a
sub-region of the *final* output is chosen, the input region it depends on is
found by walking the layers backwards, and that region alone is pushed through
all layers.  The paper states (Sections 1, 3, 6) that this re-ordering leaves
the results unchanged.  This module replays that order with small Python loops
so that the claim can be checked bit for bit against the breadth-first runner
for arbitrary tile sizes, including the padding and overlap cases of
Section 5.1 (overlapping windows make neighbouring tiles recompute a halo).

Rules the replay follows:
  * a pooling window's cells that fall outside the layer's own input plane are
    padding: never a max candidate, and contribute nothing to an average's sum
    -- whatever earlier layers would have made of a zero there;
  * cells are visited in row-major window order (first maximum wins; the
    average's float32 sum runs in that order and is then multiplied by the
    float32 reciprocal of the divisor).
It is slow by design: use it on tensors of a few thousand elements.
"""
from __future__ import annotations

import numpy as np

from . import layers as L


def _regions(layers, h_in, w_in, rows, cols):
    """Walk backwards from the final-output tile (rows=[a,b), cols=[c,d)) and return,
    for every layer boundary 0..len(layers), the in-image region needed there,
    together with the plane size at that boundary."""
    sizes = [(h_in, w_in)]
    for l in layers:
        h, w = sizes[-1]
        if l["kind"] in ("maxpool", "avgpool"):
            h = L.pool_out(h, l["k"][0], l["s"][0], l["p"][0], l.get("ceil_mode", False))
            w = L.pool_out(w, l["k"][1], l["s"][1], l["p"][1], l.get("ceil_mode", False))
        sizes.append((h, w))
    need = [None] * (len(layers) + 1)
    need[len(layers)] = (rows, cols)
    for i in range(len(layers) - 1, -1, -1):
        (a, b), (c, d) = need[i + 1]
        l = layers[i]
        if l["kind"] in ("maxpool", "avgpool"):
            h, w = sizes[i]
            a, b = max(0, a * l["s"][0] - l["p"][0]), min(h, (b - 1) * l["s"][0] - l["p"][0] + l["k"][0])
            c, d = max(0, c * l["s"][1] - l["p"][1]), min(w, (d - 1) * l["s"][1] - l["p"][1] + l["k"][1])
        need[i] = ((a, b), (c, d))
    return need, sizes


def _pool_region(kind, layer, src, src_rows, src_cols, plane_hw, out_rows, out_cols):
    """Pool the cached region `src` (covering src_rows x src_cols of a plane of size
    plane_hw) into the output region out_rows x out_cols.  Returns (values, flat indices)."""
    (kh, kw), (sh, sw), (ph, pw) = layer["k"], layer["s"], layer["p"]
    h, w = plane_hw
    n, c = src.shape[:2]
    oh0, oh1 = out_rows
    ow0, ow1 = out_cols
    out = np.empty((n, c, oh1 - oh0, ow1 - ow0), np.float32)
    idx = np.empty(out.shape, np.int32)
    for oh in range(oh0, oh1):
        for ow in range(ow0, ow1):
            cells = [(ih, iw)
                     for ih in range(oh * sh - ph, oh * sh - ph + kh) if 0 <= ih < h
                     for iw in range(ow * sw - pw, ow * sw - pw + kw) if 0 <= iw < w]
            for (ih, iw) in cells:
                if not (src_rows[0] <= ih < src_rows[1] and src_cols[0] <= iw < src_cols[1]):
                    raise AssertionError("halo region does not cover the window")
            vals = [src[:, :, ih - src_rows[0], iw - src_cols[0]] for (ih, iw) in cells]
            if kind == "maxpool":
                best = np.full((n, c), -np.inf, np.float32)
                bidx = np.full((n, c), cells[0][0] * w + cells[0][1], np.int32)
                for (ih, iw), v in zip(cells, vals):
                    m = v > best
                    best = np.where(m, v, best)
                    bidx = np.where(m, np.int32(ih * w + iw), bidx)
                out[:, :, oh - oh0, ow - ow0] = best
                idx[:, :, oh - oh0, ow - ow0] = bidx
            else:
                acc = np.zeros((n, c), np.float32)
                for v in vals:
                    acc = (acc + v).astype(np.float32)
                # count_include_pad: the window cells inside the padded plane (kh*kw in floor mode)
                hp = min(oh * sh - ph + kh, h + ph) - (oh * sh - ph)
                wp = min(ow * sw - pw + kw, w + pw) - (ow * sw - pw)
                div = hp * wp if layer.get("count_include_pad", True) else len(cells)
                inv = np.float32(1.0) / np.float32(div)
                out[:, :, oh - oh0, ow - ow0] = (acc * inv).astype(np.float32)
    return out, idx


def run_stack_tiled(layers, x, residuals=(), dtype="f32", tile=(1, 1)):
    """Depth-first execution with final-output tiles of `tile` = (rows, cols).

    Returns (out, indices) shaped like the breadth-first runner's results.
    Index tensors are written by whichever tile computes a cell; every tile that
    recomputes a halo cell must produce the same value (asserted)."""
    x = np.ascontiguousarray(x, np.float32)
    n, c, h_in, w_in = x.shape
    _, sizes = _regions(layers, h_in, w_in, (0, 1), (0, 1))
    h_out, w_out = sizes[-1]
    out = np.full((n, c, h_out, w_out), np.nan, np.float32)
    idx_out = {i: np.full((n, c) + sizes[i + 1], -1, np.int32)
               for i, l in enumerate(layers) if l["kind"] == "maxpool" and l.get("return_indices")}
    th, tw = tile
    for r0 in range(0, h_out, th):
        for c0 in range(0, w_out, tw):
            rows, cols = (r0, min(h_out, r0 + th)), (c0, min(w_out, c0 + tw))
            need, _ = _regions(layers, h_in, w_in, rows, cols)
            (a, b), (cc, d) = need[0]
            cur = x[:, :, a:b, cc:d].copy()
            cur_rows, cur_cols = (a, b), (cc, d)
            res_i = 0
            for i, l in enumerate(layers):
                kind = l["kind"]
                if kind == "bn":
                    cur = L.batchnorm(cur, l["gamma"], l["beta"], l["mean"], l["var"], l["eps"])
                elif kind == "relu":
                    cur = L.relu(cur)
                elif kind == "leaky_relu":
                    cur = L.leaky_relu(cur, l["slope"])
                elif kind == "clamp":
                    cur = L.clamp(cur, l["lo"], l["hi"])
                elif kind == "add":
                    r = np.ascontiguousarray(residuals[res_i], np.float32)
                    res_i += 1
                    cur = L.add(cur, r[:, :, cur_rows[0]:cur_rows[1], cur_cols[0]:cur_cols[1]])
                else:
                    nrows, ncols = need[i + 1]
                    cur, idx = _pool_region(kind, l, cur, cur_rows, cur_cols, sizes[i], nrows, ncols)
                    cur_rows, cur_cols = nrows, ncols
                    if i in idx_out:
                        dst = idx_out[i][:, :, nrows[0]:nrows[1], ncols[0]:ncols[1]]
                        seen = dst >= 0
                        if not np.array_equal(dst[seen], idx[seen]):
                            raise AssertionError("halo recompute produced a different argmax")
                        dst[...] = idx
                cur = L.round_to(cur, dtype)
            out[:, :, rows[0]:rows[1], cols[0]:cols[1]] = cur
    return out, [idx_out[i] for i in sorted(idx_out)]
