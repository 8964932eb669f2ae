"""Per-timestep activation caches of one editing session (section "Cache-based
editing pipeline": the feature maps of every denoising step of the previous
generation are kept and reused by the next edit; the paper moves them between
GPU, CPU memory and disk with asynchronous transfers overlapped with compute).

Residency modes behind one interface:

* resident (default): every step's cache stays in HBM.  On a 288 GB device the
  50 x 436 MB of an SD-1.5-shaped session (22 GB) fit many times over, so this
  is the normal mode and the one the benchmark's headline figure uses.
* host spill, whole buffers (`host_spill=True`): the caches live in pinned host
  memory and pass through a small window of device slots.  Step t+1's cache is
  copied in on one copy stream while step t computes, and step t's updated cache
  is copied back on a second copy stream afterwards.  Events order the three
  streams; nothing blocks the host.
* host spill, active part only (`host_spill=True, unet=<handle>`): the same
  window, but only what a masked step reads is copied in (stored maps at the
  active tiles and their one-pixel ring, K / V^T in full, statistics and
  scale / shift tables) and only what it writes is copied back (maps at the
  active tiles, K rows and V^T columns at the active tokens), by the library's
  fise_unet_cache_move_active kernels reading / writing the pinned host buffers
  directly.  Derived maps are not moved: run the step on such a slot with
  fise_masked_unet_modules over all modules (`ring.trust_derived` is False).
  `kv_home="device"` keeps every step's K / V^T block in HBM (21 % of a cache)
  and moves it slot <-> home with device copies, so the link carries maps only.
  `transfer="kernel"` moves exactly the active tiles (+ ring) with kernels:
  least data, but while their accesses to host memory are in flight every
  concurrent launch of the step runs 2-3x longer.  `transfer="dma"` moves whole
  pixel rows of the tile rows that hold active tiles with the copy engines
  (fise_unet_cache_move_tile_rows: no kernel, the step's launches are not
  disturbed), about twice the data in ~150 copies per direction, and the K / V^T
  block whole.  Default: "dma" with kv_home="device", "kernel" otherwise (the
  faster of the two in each case, measured on SD-1.5 shapes).

Memory and stream plumbing around the library (torch tensors, streams, events);
the only kernels are the library's own cache-moving ones.
"""
from __future__ import annotations

import torch


class CacheRing:
    def __init__(self, n_steps: int, cache_bytes: int, device="cuda:0", host_spill: bool = False, slots: int = 3,
                 unet=None, kv_home: str = "host", transfer: str | None = None):
        if n_steps < 1 or cache_bytes < 1:
            raise ValueError("n_steps and cache_bytes must be positive")
        if host_spill and slots < 2:
            raise ValueError("host spill needs at least two device slots (one computing, one in flight)")
        if kv_home not in ("host", "device"):
            raise ValueError("kv_home is 'host' or 'device'")
        if transfer not in (None, "dma", "kernel"):
            raise ValueError("transfer is 'dma', 'kernel' or None (pick by kv_home)")
        self.transfer = transfer or ("dma" if kv_home == "device" else "kernel")
        self.n_steps, self.cache_bytes, self.device, self.host_spill = n_steps, cache_bytes, device, host_spill
        self.sparse = bool(host_spill and unet is not None)
        self.trust_derived = not self.sparse
        if not host_spill:
            self.dev = [torch.zeros(cache_bytes, dtype=torch.uint8, device=device) for _ in range(n_steps)]
            return
        self.slots = min(slots, n_steps)
        self.dev = [torch.zeros(cache_bytes, dtype=torch.uint8, device=device) for _ in range(self.slots)]
        host_bytes = cache_bytes
        if self.sparse:
            from . import binding as fb
            self.fb, self.u, self.kv_home = fb, unet, kv_home
            self.layout = L = fb.fise_unet_cache_layout(unet)
            if fb.fise_unet_cache_bytes(unet) != cache_bytes:
                raise ValueError("cache_bytes does not match the UNet plan")
            host_bytes = L["derived_maps_off"]                     # derived maps never leave the device
            self.kv_rng = slice(L["kv_off"], L["kv_off"] + L["kv_bytes"])
            self.small_rng = slice(L["small_off"], L["small_off"] + L["small_bytes"])
            wsb = fb.fise_unet_cache_move_workspace_bytes(unet)
            self.ws_in = torch.zeros(wsb, dtype=torch.uint8, device=device)
            self.ws_out = torch.zeros(wsb, dtype=torch.uint8, device=device)
            self.kv = ([torch.zeros(L["kv_bytes"], dtype=torch.uint8, device=device) for _ in range(n_steps)]
                       if kv_home == "device" else None)
            self.mask = None
        # pinned memory is allocated as such (registering existing memory is not supported everywhere)
        self.host = [torch.zeros(host_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(n_steps)]
        self.h2d, self.d2h = torch.cuda.Stream(device=device), torch.cuda.Stream(device=device)     # default priority
        self.loaded = [None] * self.slots        # which step each slot holds (or is being filled with)
        self.h2d_done = [None] * self.slots      # event: the slot's contents have arrived
        self.d2h_done = [None] * self.slots      # event: the slot's previous contents are back in host memory
        self.compute_done = [None] * self.slots  # event: the last kernels using the slot have finished

    def begin_edit(self, tile_idx: torch.Tensor, n_active: int, base_tile: int):
        """(active-part spill) the tile list every step of the coming edit runs on; slots filled for another list
        are not reused."""
        if self.sparse:
            self.mask = (tile_idx, int(n_active), int(base_tile))
            self.loaded = [None] * self.slots
            if self.transfer == "dma":       # the copy engines are driven from the host: the tile rows in use, read back once
                tiles_w = self.fb.fise_unet_desc_of(self.u)["W"] // int(base_tile)
                rows = sorted(set((tile_idx[:int(n_active)].cpu().numpy() // tiles_w).tolist()))
                self.tile_rows = []
                for r in rows:
                    if self.tile_rows and self.tile_rows[-1][1] == r:
                        self.tile_rows[-1][1] = r + 1
                    else:
                        self.tile_rows.append([r, r + 1])

    # -- internals (host spill) ------------------------------------------------------------
    def _slot(self, t):
        return t % self.slots

    def _copy_in(self, t, s):
        if not self.sparse:
            self.dev[s].copy_(self.host[t], non_blocking=True)
            return
        if self.mask is None:
            raise RuntimeError("begin_edit() has not been called")
        idx, na, bt = self.mask
        self.dev[s][self.small_rng].copy_(self.host[t][self.small_rng], non_blocking=True)
        kv_src = self.kv[t] if self.kv is not None else self.host[t][self.kv_rng]
        self.dev[s][self.kv_rng].copy_(kv_src, non_blocking=True)
        if self.transfer == "dma":
            self.fb.fise_unet_cache_move_tile_rows(self.u, self.host[t], self.dev[s], self.tile_rows, bt, 1, self.fb.FISE_MOVE_MAPS,
                                                   stream=self.h2d)
        else:
            self.fb.fise_unet_cache_move_active(self.u, self.host[t], self.dev[s], idx, na, bt, 1, self.fb.FISE_MOVE_MAPS,
                                                self.ws_in, stream=self.h2d)

    def _copy_out(self, t, s):
        if not self.sparse:
            self.host[t].copy_(self.dev[s], non_blocking=True)
            return
        idx, na, bt = self.mask
        what = self.fb.FISE_MOVE_MAPS
        if self.kv is not None:
            self.kv[t].copy_(self.dev[s][self.kv_rng], non_blocking=True)
        elif self.transfer == "dma":             # V^T columns are not row-addressed: the K / V^T block goes back whole
            self.host[t][self.kv_rng].copy_(self.dev[s][self.kv_rng], non_blocking=True)
        else:
            what |= self.fb.FISE_MOVE_K | self.fb.FISE_MOVE_VT
        if self.transfer == "dma":
            self.fb.fise_unet_cache_move_tile_rows(self.u, self.dev[s], self.host[t], self.tile_rows, bt, 0, what, stream=self.d2h)
        else:
            self.fb.fise_unet_cache_move_active(self.u, self.dev[s], self.host[t], idx, na, bt, 0, what, self.ws_out, stream=self.d2h)

    def _prefetch(self, t):
        s = self._slot(t)
        if self.loaded[s] == t:
            return
        with torch.cuda.stream(self.h2d):
            if self.d2h_done[s] is not None:
                self.h2d.wait_event(self.d2h_done[s])        # the slot's previous owner has been written back
            elif self.compute_done[s] is not None:
                self.h2d.wait_event(self.compute_done[s])
            self._copy_in(t, s)
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
                self._copy_out(t, s)
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
        self.host[t].copy_(src[:self.host[t].numel()])          # device -> pinned host, blocking
        if self.sparse and self.kv is not None:
            self.kv[t].copy_(src[self.kv_rng])
        s = self._slot(t)
        if self.loaded[s] == t:
            self.loaded[s] = None

    def fetch(self, t: int) -> torch.Tensor:
        """A host copy of step t's cache after all queued work (for checks); with the active-part spill, of its
        stored tensors and tables (derived maps do not exist off the device)."""
        t %= self.n_steps
        torch.cuda.synchronize()
        if not self.host_spill:
            return self.dev[t].cpu()
        out = self.host[t].clone()
        if self.sparse and self.kv is not None:
            out[self.kv_rng] = self.kv[t].cpu()
        return out
