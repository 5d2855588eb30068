"""Plain CPU definition of the middle-submodel forward.  TEST INFRASTRUCTURE.

What is computed (paper Sec. 2.1 "General Inference Process of LLMs": a stack
of identical decoder layers, each a self-attention module followed by a
feed-forward network, with the keys/values of already processed tokens kept in
a KV cache; Sec. 3.1 / Fig. 3: the cloud runs the layers between the device's
shallow layers and the device's head, hidden states in, deep hidden states
out).  Chunked prefill (Sec. 2.1, Sec. 3.3) and single-step verification of a
draft sequence (Sec. 3.4) are re-schedulings of that same causal evaluation, so
the oracle is the ordinary definition evaluated per device:

    a segment of n rows starting at absolute position p attends, row t, to the
    device's keys 0 .. p+t (prefix from earlier steps + the rows up to itself).

The paper does not spell out the layer internals; the workload configurations
name them (LLaMA-style: pre-RMSNorm, rotary embedding with rotate-half pairing,
multi-head attention with as many KV heads as query heads, SwiGLU feed-forward,
no biases, residual after each sub-block).

Arithmetic is numpy in float64 by default (inputs are the bf16-representable
values the harness generated, widened); `dtype=np.float32` gives the fp32
variant.  numpy's matmul is the only library primitive used; there is no
blocking, fusion or online softmax here.

Tree verification (Sec. 2.2 "Speculative Decoding", last paragraph; Sec. 4.1:
the tree-verifying comparison system uses trees of 8 candidates): the candidate
tokens of one step form a tree whose every root-to-node path is a possible
continuation, all verified in one step.  The paper gives no more than that, so
the definition here is the one that sentence fixes: a node is evaluated exactly
as if its path alone had been submitted as a chain -- position = start + depth,
visible keys = the prefix, its ancestors and itself.  Nodes are given in an
order with parents first; `masks[i]` has bit j set when node j is node i or one
of its ancestors.  Node i's keys/values are stored at cache row start + i; once
a path has been accepted, `OracleMiddle.compact` moves its rows to the front of
that range and drops the rest, after which the cache is what the chain would
have left.

Pins: tests/test_oracle_*.py (brute-force scalar loops, closed forms,
chunk-split / verify-vs-sequential / batch-independence / rollback / RoPE-shift
invariants, torch-CPU third opinions; for trees: a chain-shaped tree equals the
chain, every path of a tree equals that path submitted alone, compaction equals
the chain's cache).  The paper prints no numeric worked example for this path,
so no value here is pinned to a printed figure.
"""
from __future__ import annotations

import numpy as np


def rmsnorm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain, row-wise (eps inside the root)."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope_rotate_half(x, positions, theta):
    """Rotary embedding, rotate-half pairing.

    x: [n, H, hd]; positions: [n] absolute positions.  For i < hd/2 the pair
    (x_i, x_{i+hd/2}) is rotated by the angle pos * theta**(-2i/hd).
    Angles are formed in float64 whatever the dtype of x.
    """
    n, H, hd = x.shape
    half = hd // 2
    inv_freq = np.float64(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]   # [n, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def prefix_causal_attention(q, K, V, start):
    """softmax(q K^T / sqrt(hd)) V with the prefix-causal mask.

    q: [n, H, hd] rows at absolute positions start .. start+n-1.
    K, V: [len, H, hd] with len >= start + n (the device's cache after append).
    Row t sees keys 0 .. start+t.  Two-pass softmax (subtract the row max).
    """
    n, H, hd = q.shape
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(np.float64(hd))
    for t in range(n):
        last = start + t                      # index of the last visible key
        for h in range(H):
            s = (K[: last + 1, h, :] @ q[t, h, :]) * scale
            w = np.exp(s - s.max())
            w = w / w.sum()
            out[t, h, :] = w @ V[: last + 1, h, :]
    return out


def check_tree(masks):
    """True if `masks` describes a forest in parents-first order: node i sees
    itself, nothing after itself, and exactly the nodes on one path to it."""
    for i, m in enumerate(masks):
        m = int(m)
        if m < 0 or (m >> i) != 1:            # own bit set, no later node
            return False
        anc = [j for j in range(i) if (m >> j) & 1]
        seen = 0
        for j in anc:                         # the ancestors form a path: each one's
            if int(masks[j]) != (seen | (1 << j)):   # own mask = the ancestors before it + itself
                return False
            seen |= 1 << j
    return True


def tree_depths(masks):
    """Depth of every node (a root has depth 0) = number of its ancestors."""
    return np.array([bin(int(m)).count("1") - 1 for m in masks], dtype=np.int64)


def tree_attention(q, K, V, start, masks):
    """Attention of tree nodes: node t sees keys 0 .. start-1 (the prefix) and
    the cache rows start + j of the nodes j on its path (bit j of masks[t]).

    q: [n, H, hd]; K, V: [len, H, hd] with len >= start + n.
    """
    n, H, hd = q.shape
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(np.float64(hd))
    for t in range(n):
        rows = list(range(start)) + [start + j for j in range(n) if (int(masks[t]) >> j) & 1]
        for h in range(H):
            s = (K[rows, h, :] @ q[t, h, :]) * scale
            w = np.exp(s - s.max())
            w = w / w.sum()
            out[t, h, :] = w @ V[rows, h, :]
    return out


def silu(z):
    return z / (1.0 + np.exp(-z))


def decoder_layer(x, start, w, kv, cfg, masks=None):
    """One decoder layer on one device's segment.

    x: [n, d] rows at positions start..start+n-1; w: dict of this layer's
    weights (linear weights stored [out, in]); kv: [K, V] lists of this
    device/layer, each [len, H, hd] with len == start on entry; they are
    extended in place (returned as new arrays in the list).
    masks: None for consecutive rows (a chunk or a chain of draft tokens), or
    the tree masks of the n rows (then row i is at position start + depth(i)).
    """
    n, d = x.shape
    H, hd = cfg["n_heads"], cfg["head_dim"]
    eps, theta = cfg["rms_eps"], cfg["rope_theta"]
    pos = np.arange(start, start + n) if masks is None else start + tree_depths(masks)

    xn = rmsnorm(x, w["attn_norm"], eps)
    q = (xn @ w["wq"].T).reshape(n, H, hd)
    k = (xn @ w["wk"].T).reshape(n, H, hd)
    v = (xn @ w["wv"].T).reshape(n, H, hd)
    q = rope_rotate_half(q, pos, theta)
    k = rope_rotate_half(k, pos, theta)
    kv[0] = np.concatenate([kv[0], k], axis=0)
    kv[1] = np.concatenate([kv[1], v], axis=0)
    if masks is None:
        o = prefix_causal_attention(q, kv[0], kv[1], start).reshape(n, d)
    else:
        o = tree_attention(q, kv[0], kv[1], start, masks).reshape(n, d)
    h = x + o @ w["wo"].T
    hn = rmsnorm(h, w["ffn_norm"], eps)
    a = silu(hn @ w["w_gate"].T) * (hn @ w["w_up"].T)
    return h + a @ w["w_down"].T


class OracleMiddle:
    """The middle submodel with one KV cache per device.

    cfg: dict with n_layers, d_model, n_heads, head_dim, d_ffn, rms_eps,
    rope_theta.  layers: a list of weight dicts, or a callable l -> dict so a
    large model's weights can be produced one layer at a time.
    """

    def __init__(self, cfg, layers, dtype=np.float64):
        self.cfg = dict(cfg)
        self.dtype = dtype
        self._layers = layers
        self._converted = {}    # layers given as a list are widened to `dtype` once
        self.kv = {}            # device -> list over layers of [K, V]

    def _layer(self, l):
        if callable(self._layers):
            return {k: np.asarray(v, dtype=self.dtype) for k, v in self._layers(l).items()}
        if l not in self._converted:
            self._converted[l] = {k: np.asarray(v, dtype=self.dtype) for k, v in self._layers[l].items()}
        return self._converted[l]

    def kv_len(self, device):
        if device not in self.kv:
            return 0
        return self.kv[device][0][0].shape[0]

    def _ensure(self, device):
        if device not in self.kv:
            H, hd = self.cfg["n_heads"], self.cfg["head_dim"]
            self.kv[device] = [[np.zeros((0, H, hd), self.dtype), np.zeros((0, H, hd), self.dtype)]
                               for _ in range(self.cfg["n_layers"])]

    def import_kv(self, device, layer, pos0, k, v):
        """Install synthetic cache rows (k taken as already rotated) at pos0.."""
        self._ensure(device)
        K, V = self.kv[device][layer]
        assert K.shape[0] == pos0, "import must extend the cache contiguously"
        self.kv[device][layer][0] = np.concatenate([K, np.asarray(k, self.dtype)], axis=0)
        self.kv[device][layer][1] = np.concatenate([V, np.asarray(v, self.dtype)], axis=0)

    def release(self, device):
        self.kv.pop(device, None)

    def compact(self, device, base, keep):
        """After a tree step at `base`: keep the nodes `keep` (indices into the
        tree, one path from a root, ascending) as rows base .. base+len(keep)-1
        and drop everything behind them."""
        keep = [int(k) for k in keep]
        if any(b <= a for a, b in zip(keep, keep[1:])) or (keep and keep[0] < 0):
            raise ValueError("kept nodes must ascend")
        if base < 0 or base + (keep[-1] + 1 if keep else 0) > self.kv_len(device):
            raise ValueError("kept node beyond the cache")
        self._ensure(device)
        rows = list(range(base)) + [base + k for k in keep]
        for l in range(self.cfg["n_layers"]):
            self.kv[device][l][0] = self.kv[device][l][0][rows]
            self.kv[device][l][1] = self.kv[device][l][1][rows]

    def forward(self, segments):
        """segments: list of (device, start_pos, X[n, d]) or, for a tree of
        candidates, (device, start_pos, X[n, d], masks).  Returns list of [n, d].

        start_pos < cache length rolls the cache back to start_pos first (the
        rows of rejected draft tokens are dropped); start_pos > length is an
        error.  One device may appear once per step.
        """
        seen = set()
        segments = [tuple(sg) + (None,) * (4 - len(sg)) for sg in segments]
        for dev, start, x, masks in segments:
            if dev in seen:
                raise ValueError("device appears twice in one step")
            seen.add(dev)
            if start > self.kv_len(dev):
                raise ValueError("start position leaves a gap in the cache")
            if masks is not None and (len(masks) != len(x) or not check_tree(masks)):
                raise ValueError("masks do not describe a tree in parents-first order")
        xs = []
        for dev, start, x, masks in segments:
            self._ensure(dev)
            for l in range(self.cfg["n_layers"]):
                self.kv[dev][l][0] = self.kv[dev][l][0][:start]
                self.kv[dev][l][1] = self.kv[dev][l][1][:start]
            xs.append(np.asarray(x, dtype=self.dtype))
        # layer-outer order so that a lazily generated layer is built once per
        # step; segments never interact, so this equals device-by-device order.
        for l in range(self.cfg["n_layers"]):
            w = self._layer(l)
            for i, (dev, start, _, masks) in enumerate(segments):
                xs[i] = decoder_layer(xs[i], start, w, self.kv[dev][l], self.cfg, masks)
        return xs
