"""Host-side plumbing around the C-ABI engine: pinned host arrays, packing named
tensors into the flat layout, and one call per training iteration.

Nothing of the method is computed here.  The host arrays are pinned memory from the
library's own allocator (`hmy_host_alloc`), seen from Python as numpy arrays, so this
module needs no PyTorch: a process that imports only it and the binding runs on the
HIP runtime the library was linked against.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import binding as B

# Pack counts beyond the first feasible one that the benchmark lets the planner
# try; the full-size parity tests use the same value so they check the launch
# configuration that is timed.
BENCH_PACK_SEARCH = 4


class Pinned:
    """A pinned host buffer from the library, viewed as a 1-D numpy array."""

    def __init__(self, count: int, dtype):
        self.dtype = np.dtype(dtype)
        self.count = int(count)
        self.nbytes = max(self.count * self.dtype.itemsize, 16)
        self.ptr = B.hmy_host_alloc(self.nbytes)
        buf = (C.c_char * self.nbytes).from_address(self.ptr)
        self.a = np.frombuffer(buf, dtype=self.dtype, count=self.count)

    def free(self) -> None:
        if self.ptr:
            self.a = None
            B.hmy_host_free(self.ptr)
            self.ptr = 0


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even bf16 of fp32 values, as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


class Pageable:
    """An ordinary (not page-locked) host buffer with the interface of Pinned."""

    def __init__(self, count: int, dtype):
        self.a = np.zeros(int(count), dtype=dtype)
        self.ptr = self.a.ctypes.data

    def free(self) -> None:
        self.a = None
        self.ptr = 0


class TrainingState:
    """Caller-owned pinned host state in the library's tensor layout."""

    def __init__(self, cfg, with_grads: bool = True, pageable_optimizer_state: bool = False):
        """with_grads=False: no gradient array (only for schedules with HMY_GRADIENTS_ON_DEVICE, layer-pack-major
        order and the update on the device, which never write it).
        pageable_optimizer_state=True: master, m and v in ordinary memory -- only for schedules with
        HMY_UPDATE_ON_HOST, where nothing but the library's CPU threads touches them (page-locked memory is
        scarce: the weights and gradients, which do cross the link, still get it)."""
        self.cfg = cfg
        self.spec = B.make_spec(cfg)
        self.layout = B.hmy_layout(self.spec)
        self.n_params = B.hmy_model_size(self.spec)[1]
        self.mixed = cfg["precision"] == "bf16"
        n = self.n_params
        self._bufs = []

        def pinned(dtype, pageable=False):
            p = Pageable(n, dtype) if pageable else Pinned(n, dtype)
            self._bufs.append(p)
            return p

        try:
            self.weights = pinned(np.uint16 if self.mixed else np.float32)   # bf16 bit patterns in mixed mode
            self.master = pinned(np.float32, pageable_optimizer_state) if self.mixed else None
            self.adam_m = pinned(np.float32, pageable_optimizer_state)
            self.adam_v = pinned(np.float32, pageable_optimizer_state)
            self.grads = pinned(np.float32) if with_grads else None
        except B.HmyError:
            self.close()      # page-locked memory ran out half way: give back what was taken
            raise
        for p in (self.adam_m, self.adam_v, self.grads):
            if p is not None:
                p.a[:] = 0

    def close(self) -> None:
        for p in getattr(self, "_bufs", []):
            p.free()
        self._bufs = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- named <-> flat -----------------------------------------------------------
    def _flat_set(self, flat: Pinned, named) -> None:
        for t in self.layout:
            src = np.ascontiguousarray(named[t["name"]], dtype=np.float32).reshape(-1)
            flat.a[t["offset"]:t["offset"] + t["count"]] = src

    def _flat_get(self, flat: Pinned, bf16: bool = False):
        out = {}
        for t in self.layout:
            a = flat.a[t["offset"]:t["offset"] + t["count"]]
            a = bf16_bits_to_f32(a) if bf16 else a.astype(np.float32)
            out[t["name"]] = a.reshape(t["rows"], t["cols"]).copy() if t["cols"] > 1 else a.copy()
        return out

    def _round_weights(self) -> None:
        step = 1 << 24
        for lo in range(0, self.n_params, step):
            self.weights.a[lo:lo + step] = f32_to_bf16_bits(self.master.a[lo:lo + step])

    def load(self, params, m=None, v=None) -> None:
        """params: name -> fp32 array.  In bf16 mode they become the fp32 master and
        the compute weights are their round-to-nearest-even bf16 copy."""
        if self.mixed:
            self._flat_set(self.master, params)
            self._round_weights()
        else:
            self._flat_set(self.weights, params)
        if m is not None:
            self._flat_set(self.adam_m, m)
        if v is not None:
            self._flat_set(self.adam_v, v)

    def fill_random(self, seed: int = 0, std: float = 0.02, tile: int = 0) -> None:
        """Benchmark init without the named round trip: matrices N(0, std^2),
        LayerNorm gains 1, everything else 0.  tile > 0: draw that many values once and
        fill every matrix with runs of them (for models of billions of parameters, whose
        drawing would take minutes; a matrix no larger than the tile has no repeats)."""
        rng = np.random.default_rng(seed)
        tgt = (self.master if self.mixed else self.weights).a
        pool = rng.standard_normal(tile, dtype=np.float32) * np.float32(std) if tile else None
        pool16 = f32_to_bf16_bits(pool) if tile and self.mixed else None
        start = 0
        for t in self.layout:
            sl = tgt[t["offset"]:t["offset"] + t["count"]]
            base = t["name"].split(".")[-1]
            if t["cols"] > 1 and tile:
                wsl = self.weights.a[t["offset"]:t["offset"] + t["count"]]
                for lo in range(0, t["count"], tile):      # each matrix starts somewhere else in the pool
                    n = min(tile, t["count"] - lo)
                    k = min(n, tile - start)
                    sl[lo:lo + k] = pool[start:start + k]
                    sl[lo + k:lo + n] = pool[:n - k]
                    if self.mixed:
                        wsl[lo:lo + k] = pool16[start:start + k]
                        wsl[lo + k:lo + n] = pool16[:n - k]
                start = (start + 7919 * 1024) % tile
            elif t["cols"] > 1:
                sl[:] = rng.standard_normal(t["count"], dtype=np.float32) * np.float32(std)
            elif base.endswith("_g"):
                sl[:] = 1.0
            else:
                sl[:] = 0.0
            if tile and self.mixed and t["cols"] == 1:
                self.weights.a[t["offset"]:t["offset"] + t["count"]] = f32_to_bf16_bits(sl)
        if self.mixed and not tile:
            self._round_weights()
        self.adam_m.a[:] = 0
        self.adam_v.a[:] = 0

    def named(self, what: str):
        """what in weights | master | m | v | grads -> name -> fp32 array."""
        flat = {"weights": self.weights, "master": self.master, "m": self.adam_m, "v": self.adam_v,
                "grads": self.grads}[what]
        return self._flat_get(flat, bf16=(what == "weights" and self.mixed))


class Engine:
    """One hmy handle bound to a TrainingState."""

    def __init__(self, state: TrainingState, budget_bytes: int, n_micro: int, micro_batch: int, sched=None,
                 device: int = 0, search: int = 0, arena_ptr: int = 0, arena_bytes: int = 0, **budget_kw):
        """arena_ptr / arena_bytes: device memory of the caller's (256-byte aligned, at least the arena's size) for the
        engine to live in, instead of an allocation of its own; the caller keeps it alive until close().
        budget_kw: what the planner may sweep when sched is None (binding.make_budget)."""
        self.state = state
        self.M, self.b = n_micro, micro_batch
        # fails with HMY_E_NO_DEVICE when there is no GPU: there is no CPU fallback
        self.handle = B.hmy_create(state.spec, budget_bytes, n_micro, micro_batch, sched, device, arena_ptr=arena_ptr,
                                   arena_bytes=arena_bytes, search=search, **budget_kw)
        self._ids = None
        self._tgt = None
        try:
            self.sched = B.hmy_get_schedule(self.handle)
            self.packs = B.schedule_packs(self.sched)
            self.arena = B.hmy_arena(state.spec, self.sched, n_micro, micro_batch)
            B.hmy_bind_state(self.handle, state.weights.ptr, state.master.ptr if state.mixed else None,
                             state.adam_m.ptr, state.adam_v.ptr,
                             state.grads.ptr if state.grads is not None else None, state.n_params)
        except B.HmyError:
            self.close()      # the handle holds the whole device arena
            raise

    def set_batch(self, ids: np.ndarray, targets: np.ndarray) -> None:
        s = self.state.cfg["seq_len"]
        assert ids.shape == (self.M, self.b, s) and targets.shape == ids.shape
        for old in (self._ids, self._tgt):
            if old is not None:
                old.free()
        self._ids, self._tgt = Pinned(ids.size, np.int32), Pinned(ids.size, np.int32)
        self._ids.a[:] = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
        self._tgt.a[:] = np.ascontiguousarray(targets, dtype=np.int32).reshape(-1)

    def resident_params(self) -> int:
        """Parameters whose optimizer state the schedule keeps on the device."""
        return B.hmy_resident_params(self.handle)

    def sync_state(self) -> None:
        """Write optimizer state that is resident on the device back to the TrainingState's arrays."""
        B.hmy_sync_state(self.handle)

    def rebind(self) -> None:
        """After the TrainingState's arrays were rewritten by the caller: resident state is read from them again."""
        st = self.state
        B.hmy_bind_state(self.handle, st.weights.ptr, st.master.ptr if st.mixed else None, st.adam_m.ptr, st.adam_v.ptr,
                         st.grads.ptr if st.grads is not None else None, st.n_params)

    def step(self, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, step=1, want_stats=True):
        return B.hmy_iteration(self.handle, self.M, self.b, self._ids.ptr, self._tgt.ptr, lr, beta1, beta2, eps, step,
                               want_stats)

    def close(self) -> None:
        if self.handle is not None:
            B.hmy_destroy(self.handle)
            self.handle = None
        for old in (self._ids, self._tgt):
            if old is not None:
                old.free()
        self._ids = self._tgt = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
