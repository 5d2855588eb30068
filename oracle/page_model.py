"""Integer model of the paged KV bookkeeping.  TEST INFRASTRUCTURE.

The paper only says the cloud keeps a KV cache per request and batches
requests that join and leave between steps (Sec. 2.1), served through paged
attention (Sec. 4.1 implementation paragraph).  Many page assignments would be
valid; to make page ids comparable bit for bit the library follows one fixed
policy, and this file is an independent model of that policy:

  * pages are ids 0 .. n_pages-1; an allocation takes the lowest free id;
  * a segment (device, start, n) first rolls the device back to `start`
    (pages wholly beyond ceil(start/page) are freed), then appends n tokens;
  * within a step all rollback frees happen first, for all segments in array
    order; then segments allocate in array order, each in ascending position;
  * token at position q lives in the device's page-list entry q // page,
    slot q % page; a device owns exactly ceil(kv_len / page) pages;
  * a step that fails validation or does not fit changes nothing;
  * keeping one path of a tree step (compact) shortens the device to
    base + kept nodes at once and frees, at once, the pages wholly beyond.

Written with plain Python sets/lists; shares nothing with the library's planner.
"""
from __future__ import annotations


class PageModelError(Exception):
    def __init__(self, code, msg):
        super().__init__(msg)
        self.code = code


# status names mirror the C header's enum values (an interface, not code)
EINVAL, ENOMEM, EPOS, EDUP, EDEVICE = -1, -2, -3, -4, -5


class PageModel:
    def __init__(self, n_pages, page_size=16, max_devices=64, max_step_tokens=8192,
                 max_pos=1 << 20, max_verify=8):
        self.n_pages = n_pages
        self.page = page_size
        self.max_devices = max_devices
        self.max_step_tokens = max_step_tokens
        self.max_pos = max_pos
        self.max_verify = max_verify
        self.free = set(range(n_pages))
        self.pages = {}      # device -> list of page ids
        self.length = {}     # device -> kv_len

    def _need(self, length):
        return (length + self.page - 1) // self.page

    def step(self, segments):
        """segments: list of (device, kind, start, n); kind 0 = chunk, 1 = verify.

        Returns per-segment list of (page_id, slot) write targets for its rows.
        """
        seen = set()
        total = 0
        for dev, kind, start, n in segments:
            if not (0 <= dev < self.max_devices):
                raise PageModelError(EDEVICE, "device id out of range")
            if kind not in (0, 1) or n <= 0 or start < 0:
                raise PageModelError(EINVAL, "bad segment")
            if kind == 1 and n > self.max_verify:
                raise PageModelError(EINVAL, "verify segment too long")
            if start + n > self.max_pos:
                raise PageModelError(EINVAL, "position beyond max_pos")
            if dev in seen:
                raise PageModelError(EDUP, "device twice in one step")
            seen.add(dev)
            if start > self.length.get(dev, 0):
                raise PageModelError(EPOS, "gap between cache and start")
            total += n
        if total > self.max_step_tokens:
            raise PageModelError(EINVAL, "too many tokens in step")
        # capacity check on a copy of the counts: frees first, then needs
        free_after = len(self.free)
        need = 0
        for dev, kind, start, n in segments:
            have = len(self.pages.get(dev, []))
            keep = self._need(start)
            free_after += have - keep
            need += self._need(start + n) - keep
        if need > free_after:
            raise PageModelError(ENOMEM, "KV pool exhausted")
        # commit: all rollbacks, then all allocations
        for dev, kind, start, n in segments:
            lst = self.pages.setdefault(dev, [])
            keep = self._need(start)
            while len(lst) > keep:
                self.free.add(lst.pop())
            self.length[dev] = start
        targets = []
        for dev, kind, start, n in segments:
            lst = self.pages[dev]
            tgt = []
            for q in range(start, start + n):
                if q // self.page == len(lst):
                    pid = min(self.free)
                    self.free.remove(pid)
                    lst.append(pid)
                tgt.append((lst[q // self.page], q % self.page))
            self.length[dev] = start + n
            targets.append(tgt)
        return targets

    def compact(self, dev, base, keep):
        """Keep tree nodes `keep` (ascending indices) of the step that started at
        `base`.  Returns the (page, slot) moves as (source, destination) pairs."""
        if not (0 <= dev < self.max_devices):
            raise PageModelError(EDEVICE, "device id out of range")
        keep = list(keep)
        if base < 0 or len(keep) > self.max_verify or any(k < 0 or k >= self.max_verify for k in keep) \
                or any(b <= a for a, b in zip(keep, keep[1:])):
            raise PageModelError(EINVAL, "bad kept-node list")
        length = self.length.get(dev, 0)
        if base > length or (keep and base + keep[-1] >= length):
            raise PageModelError(EPOS, "kept node beyond the cache")
        lst = self.pages.get(dev, [])
        moves = [((lst[(base + k) // self.page], (base + k) % self.page),
                  (lst[(base + i) // self.page], (base + i) % self.page)) for i, k in enumerate(keep)]
        new_len = base + len(keep)
        while len(lst) > self._need(new_len):
            self.free.add(lst.pop())
        if dev in self.length or new_len:
            self.length[dev] = new_len
        return moves

    def release(self, dev):
        if not (0 <= dev < self.max_devices):
            raise PageModelError(EDEVICE, "device id out of range")
        for pid in self.pages.pop(dev, []):
            self.free.add(pid)
        self.length.pop(dev, None)

    def query(self, dev):
        return self.length.get(dev, 0), list(self.pages.get(dev, []))
