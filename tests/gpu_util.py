"""Helpers for the GPU parity tests: move seeded inputs to the device, run the
same step list through the HIP library and through the oracle."""
import numpy as np

import hat_inputs as hi


def rel_err(got, ref):
    """max |got - ref| / max |ref|   (the tolerance of the parity bar is stated on this)."""
    ref = np.asarray(ref, np.float64)
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def rel_l2(got, ref):
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / max(np.linalg.norm(ref), 1e-30))


def to_dev_bf16(x):
    import torch
    return torch.from_numpy(hi.bf16_bits(np.ascontiguousarray(x, np.float32)).view(np.int16)).view(torch.bfloat16).cuda()


def dev_weights(w):
    return {k: to_dev_bf16(v) for k, v in w.items()}


def to_np(t):
    return t.detach().float().cpu().numpy()


class Pair:
    """The library and the oracle side by side on the same weights."""

    def __init__(self, cfg, seed, n_pages, gain_jitter=0.1, io_dtype="bf16", **kw):
        from oracle import OracleMiddle, PageModel
        from paper_2503_18989_amd import HatMid
        self.cfg, self.seed = cfg, seed
        self.weights = [hi.layer_weights(cfg, l, seed, gain_jitter=gain_jitter) for l in range(cfg["n_layers"])]
        self.gpu = HatMid(cfg, [dev_weights(w) for w in self.weights], n_pages=n_pages, io_dtype=io_dtype, **kw)
        self.ref = OracleMiddle(cfg, self.weights)
        self.pages = PageModel(n_pages, 16, kw.get("max_devices", 64), kw.get("max_step_tokens", 8192),
                               kw.get("max_pos", 16384))
        self.io_dtype = io_dtype
        self.counter = 0

    def step(self, segs, inputs=None):
        """segs: list of (device, kind, start, n) or (device, kind, start, n, tree masks).
        Returns (gpu outs, oracle outs) as numpy."""
        import torch
        from paper_2503_18989_amd import Segment
        masks = [sg[4] if len(sg) > 4 else None for sg in segs]
        segs = [tuple(sg[:4]) for sg in segs]
        xs = []
        for i, (dev, kind, start, n) in enumerate(segs):
            x = inputs[i] if inputs is not None else hi.hidden_rows(n, self.cfg["d_model"], self.seed, self.counter, dev)
            xs.append(x)
        self.counter += 1
        gsegs = []
        for (dev, kind, start, n), x, m in zip(segs, xs, masks):
            xd = to_dev_bf16(x) if self.io_dtype == "bf16" else torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
            gsegs.append(Segment(dev, kind, start, xd, tree_mask=m))
        outs = self.gpu.forward(gsegs)
        torch.cuda.synchronize()
        refs = self.ref.forward([(dev, start, x, m) for (dev, kind, start, n), x, m in zip(segs, xs, masks)])
        self.pages.step(segs)
        return [to_np(o) for o in outs], refs

    def compact(self, dev, base, keep):
        """Keeps tree nodes `keep` of the step that started at `base`, on all three sides."""
        import torch
        self.gpu.kv_compact(dev, base, keep)
        torch.cuda.synchronize()
        self.ref.compact(dev, base, keep)
        self.pages.compact(dev, base, keep)

    def check_pages(self, devices):
        for d in devices:
            assert self.gpu.kv_query(d) == self.pages.query(d), "page table of device %d differs" % d

    def close(self):
        self.gpu.close()
