"""Seeded synthetic inputs shared by the oracle tests, the GPU tests and bench.py.

Holds no arithmetic of the method: only model shapes, random draws, the bf16
rounding used to make inputs representable on both sides, and the segment
schedules of the synthetic workloads.  The workloads stand in for the paper's
SpecBench / CNN-DailyMail runs with Vicuna-7B/13B (Sec. 4.1, Table 2/3): same
layer shapes, 30 devices, prompt lengths of hundreds to thousands of tokens,
draft length about 5 with about 2 accepted (Table 4), 64-step runs (Sec. 2.3).
"""
from __future__ import annotations

import numpy as np

PAGE = 16
MAX_VERIFY = 8
CHUNK, VERIFY = 0, 1

# ----------------------------------------------------------------------------
# model shapes (the middle submodel: all layers except the device's first m
# and the head, paper Sec. 2.4 / 4.1)
# ----------------------------------------------------------------------------
TINY = dict(name="tiny", n_layers=1, d_model=256, n_heads=4, head_dim=64, d_ffn=688,
            rms_eps=1e-6, rope_theta=1e4)
MID7B = dict(name="7b-mid", n_layers=30, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008,
             rms_eps=1e-6, rope_theta=1e4)
MID13B = dict(name="13b-mid", n_layers=38, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824,
              rms_eps=1e-6, rope_theta=1e4)


def with_layers(cfg, n_layers):
    c = dict(cfg)
    c["n_layers"] = n_layers
    return c


# ----------------------------------------------------------------------------
# bf16 helpers (round-to-nearest-even), numpy only
# ----------------------------------------------------------------------------
def bf16_bits(x):
    """float32 array -> uint16 array of bf16 bit patterns (RNE)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x):
    """float32 array -> float32 array holding bf16-representable values."""
    return bf16_to_f32(bf16_bits(x))


# ----------------------------------------------------------------------------
# seeded draws
# ----------------------------------------------------------------------------
def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(k) for k in key])))


WEIGHT_NAMES = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def layer_weights(cfg, layer, seed, gain_jitter=0.0, round_bf16=True, std=0.02):
    """One layer's weights as float32 arrays (bf16-representable if round_bf16).

    Linear weights ~ N(0, std^2), stored [out, in].  RMSNorm gains are 1
    (+ gain_jitter * N(0,1) for tests that must notice an ignored gain).
    """
    d, F = cfg["d_model"], cfg["d_ffn"]
    r = _rng(seed, 7, layer)
    shapes = dict(wq=(d, d), wk=(d, d), wv=(d, d), wo=(d, d), w_gate=(F, d), w_up=(F, d), w_down=(d, F))
    w = {}
    for name in WEIGHT_NAMES:
        if name.endswith("norm"):
            g = np.ones(d, np.float32)
            if gain_jitter:
                g = g + np.float32(gain_jitter) * r.standard_normal(d, dtype=np.float32)
            w[name] = g
        else:
            a = r.standard_normal(shapes[name], dtype=np.float32)
            a *= np.float32(std)
            w[name] = a
    if round_bf16:
        w = {k: bf16_round(v) for k, v in w.items()}
    return w


def hidden_rows(n, d, seed, *key, round_bf16=True):
    """n rows of hidden states ~ N(0,1)."""
    x = _rng(seed, 11, *key).standard_normal((n, d), dtype=np.float32)
    return bf16_round(x) if round_bf16 else x


def kv_prefix(n, H, hd, seed, *key, std=1.28):
    """Synthetic cache rows for import: K (taken as already rotated) and V,
    ~ N(0, std^2); std 1.28 is what unit-RMS inputs times N(0, 0.02^2) weights
    give at d = 4096.  bf16-representable."""
    r = _rng(seed, 13, *key)
    k = r.standard_normal((n, H, hd), dtype=np.float32) * np.float32(std)
    v = r.standard_normal((n, H, hd), dtype=np.float32) * np.float32(std)
    return bf16_round(k), bf16_round(v)


# ----------------------------------------------------------------------------
# workload schedules: lists of steps, each a list of (device, kind, start, n)
# ----------------------------------------------------------------------------
def tiny_schedule():
    """Config 1: 64-row prompt as 4 chunks of 16, then 3 verify segments of 4
    draft rows with accepted counts 2, 4 (the third is not followed)."""
    steps = [[(0, CHUNK, 16 * i, 16)] for i in range(4)]
    steps += [[(0, VERIFY, 64, 4)], [(0, VERIFY, 66, 4)], [(0, VERIFY, 70, 4)]]
    return steps


def single_prompt_schedule(prompt=2048, chunk=256, device=0):
    """Config 2: one device, the prompt fed as equal chunks."""
    return [[(device, CHUNK, s, min(chunk, prompt - s))] for s in range(0, prompt, chunk)]


def mixed_prefixes(seed, n_devices=30, lo=256, hi=4096):
    """Config 3: per-device prefix length, uniform in [lo, hi]."""
    return _rng(seed, 17).integers(lo, hi + 1, size=n_devices).tolist()


def mixed_step(seed, step, lengths, n_chunk=10, k=5, chunk_sizes=(128, 256, 512)):
    """Config 3, one step: n_chunk devices (rotating with the step) submit a
    prompt chunk, the rest a k-row verify segment.  `lengths` = current cache
    lengths; returns the step's segments (cache grows by n for everyone)."""
    n_dev = len(lengths)
    r = _rng(seed, 19, step)
    first = (step * n_chunk) % n_dev
    chunkers = {(first + i) % n_dev for i in range(n_chunk)}
    segs = []
    for dev in range(n_dev):
        if dev in chunkers:
            segs.append((dev, CHUNK, lengths[dev], int(r.choice(chunk_sizes))))
        else:
            segs.append((dev, VERIFY, lengths[dev], k))
    return segs


def verify_lengths(seed, n_devices=30, lo=1024, hi=8192):
    """Config 4: per-device cache length, uniform in [lo, hi]."""
    return _rng(seed, 23).integers(lo, hi + 1, size=n_devices).tolist()


ACCEPT_P = (0.40, 0.30, 0.15, 0.10, 0.05)      # accepted rows 1..5, mean 2.1 (paper Table 4: about 2)


def verify_schedule(seed, lengths, steps=64, k=5, rollback=True):
    """Config 4: every device verifies k rows per step; before the next step
    each device rolls back to start + a, a drawn from ACCEPT_P (or keeps all k
    rows when rollback is False)."""
    r = _rng(seed, 29)
    cur = list(lengths)
    out = []
    for _ in range(steps):
        out.append([(dev, VERIFY, cur[dev], k) for dev in range(len(cur))])
        for dev in range(len(cur)):
            a = int(r.choice(np.arange(1, 6), p=ACCEPT_P)) if rollback else k
            cur[dev] += min(a, k)
    return out


def random_tree(seed, n, *key):
    """A seeded forest of n candidate nodes in parents-first order (the shape of a
    tree-verification step, paper Sec. 2.2; size 8 in Sec. 4.1): parents[i] in
    {-1 (hangs off the last committed token), 0 .. i-1}."""
    r = _rng(seed, 23, n, *key)
    return [-1] + [int(r.integers(-1, i)) for i in range(1, n)]


def tree_masks(parents):
    """parents -> per-node bit masks (bit j: node j is the node itself or an ancestor)."""
    masks = []
    for i, p in enumerate(parents):
        masks.append((1 << i) | (masks[p] if p >= 0 else 0))
    return masks


def tree_path(parents, node):
    """Indices from the root down to `node`."""
    path = []
    while node >= 0:
        path.append(node)
        node = parents[node]
    return path[::-1]


MEDUSA_LIKE_TREE = [-1, 0, 0, 1, 1, 2, 3, -1]   # a fixed 8-node shape: two first candidates, branching below


def sweep_schedule(chunk, prompt=8192, n_devices=8, batched=True):
    """Config 5: n_devices prompts of `prompt` rows fed in chunks of `chunk`;
    batched: all devices submit their j-th chunk in the same step."""
    steps = []
    if batched:
        for s in range(0, prompt, chunk):
            steps.append([(dev, CHUNK, s, min(chunk, prompt - s)) for dev in range(n_devices)])
    else:
        for dev in range(n_devices):
            for s in range(0, prompt, chunk):
                steps.append([(dev, CHUNK, s, min(chunk, prompt - s))])
    return steps
