"""Per-timestep activation caches of one editing session (section "Cache-based
editing pipeline": the feature maps of every denoising step of the previous
generation are kept and reused by the next edit; the paper moves them between
GPU, CPU memory and disk with asynchronous transfers overlapped with compute).

Two residency modes for the same interface:

* resident (default): every step's cache stays in HBM.  On a 288 GB device the
  50 x 260 MB of an SD-1.5-shaped session (13 GB) fit many times over, so this
  is the normal mode and the one the benchmark's headline figure uses.
* host spill: the caches live in pinned host memory and pass through a small
  window of device slots.  Step t+1's cache is copied in on one copy stream
  while step t computes, and step t's updated cache is copied back on a second
  copy stream afterwards (both directions of the link at once).  Events order
  the three streams; nothing blocks the host.

This is memory and stream plumbing around the library (torch tensors, streams
and events only); it launches no kernels of its own.
"""
from __future__ import annotations

import torch


class CacheRing:
    def __init__(self, n_steps: int, cache_bytes: int, device="cuda:0", host_spill: bool = False, slots: int = 3):
        if n_steps < 1 or cache_bytes < 1:
            raise ValueError("n_steps and cache_bytes must be positive")
        if host_spill and slots < 2:
            raise ValueError("host spill needs at least two device slots (one computing, one in flight)")
        self.n_steps, self.cache_bytes, self.device, self.host_spill = n_steps, cache_bytes, device, host_spill
        if not host_spill:
            self.dev = [torch.zeros(cache_bytes, dtype=torch.uint8, device=device) for _ in range(n_steps)]
            return
        self.slots = min(slots, n_steps)
        self.dev = [torch.zeros(cache_bytes, dtype=torch.uint8, device=device) for _ in range(self.slots)]
        # pinned memory is allocated as such (registering existing memory is not supported everywhere)
        self.host = [torch.zeros(cache_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(n_steps)]
        self.h2d, self.d2h = torch.cuda.Stream(device=device), torch.cuda.Stream(device=device)     # default priority
        self.loaded = [None] * self.slots        # which step each slot holds (or is being filled with)
        self.h2d_done = [None] * self.slots      # event: the slot's contents have arrived
        self.d2h_done = [None] * self.slots      # event: the slot's previous contents are back in host memory
        self.compute_done = [None] * self.slots  # event: the last kernels using the slot have finished

    # -- internals (host spill) ------------------------------------------------------------
    def _slot(self, t):
        return t % self.slots

    def _prefetch(self, t):
        s = self._slot(t)
        if self.loaded[s] == t:
            return
        with torch.cuda.stream(self.h2d):
            if self.d2h_done[s] is not None:
                self.h2d.wait_event(self.d2h_done[s])        # the slot's previous owner has been written back
            elif self.compute_done[s] is not None:
                self.h2d.wait_event(self.compute_done[s])
            self.dev[s].copy_(self.host[t], non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(self.h2d)
        self.h2d_done[s], self.loaded[s] = ev, t
        self.d2h_done[s] = None
        self.compute_done[s] = None

    # -- interface -------------------------------------------------------------------------
    def acquire(self, t: int, prefetch_next: bool = True):
        """Device tensor holding step t's cache, valid for work queued on the CURRENT stream after this call.
        With host spill it also starts moving step t+1's cache in."""
        t %= self.n_steps
        if not self.host_spill:
            return self.dev[t]
        self._prefetch(t)
        s = self._slot(t)
        torch.cuda.current_stream().wait_event(self.h2d_done[s])
        nxt = (t + 1) % self.n_steps
        if prefetch_next and self.slots >= 3 and self._slot(nxt) != s:
            # with three slots or more the next step's slot is normally neither this one nor one still waiting for
            # its write-back to start.  With two slots, and when the step count wraps onto this very slot
            # (n_steps % slots == 1 at the last step), the next copy-in is issued by release() instead, after the
            # work on this slot and its write-back have been ordered in front of it.
            self._prefetch(nxt)
        return self.dev[s]

    def release(self, t: int, write_back: bool = True):
        """Work on step t's cache has been queued on the current stream: (host spill) copy the updated cache
        back once that work ends, and let the slot be reused after that."""
        t %= self.n_steps
        if not self.host_spill:
            return
        s = self._slot(t)
        assert self.loaded[s] == t, "release() of a step that is not in its slot"
        ev = torch.cuda.Event()
        ev.record(torch.cuda.current_stream())
        self.compute_done[s] = ev
        if write_back:
            with torch.cuda.stream(self.d2h):
                self.d2h.wait_event(ev)
                self.host[t].copy_(self.dev[s], non_blocking=True)
                done = torch.cuda.Event()
                done.record(self.d2h)
            self.d2h_done[s] = done
        nxt = (t + 1) % self.n_steps
        if self.slots == 2 or self._slot(nxt) == s:
            self._prefetch(nxt)

    def store(self, t: int, src: torch.Tensor):
        """Set step t's cache from a device tensor (cache building).  Synchronous for host spill."""
        t %= self.n_steps
        if not self.host_spill:
            self.dev[t].copy_(src)
            return
        self.host[t].copy_(src)                   # device -> pinned host, blocking
        s = self._slot(t)
        if self.loaded[s] == t:
            self.loaded[s] = None

    def fetch(self, t: int) -> torch.Tensor:
        """A host copy of step t's cache after all queued work (for checks)."""
        t %= self.n_steps
        torch.cuda.synchronize()
        if not self.host_spill:
            return self.dev[t].cpu()
        return self.host[t].clone()
