"""Host-side plumbing around the C-ABI engine: pinned host arrays, packing named
tensors into the flat layout, and one call per training iteration.

Nothing of the method is computed here: PyTorch only owns pinned host memory
(and optionally the device arena); every step runs inside libhmy.so.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

# Pack counts beyond the first feasible one that the benchmark lets the planner
# try; the full-size parity tests use the same value so they check the launch
# configuration that is timed.
BENCH_PACK_SEARCH = 4


class TrainingState:
    """Caller-owned pinned host state in the library's tensor layout."""

    def __init__(self, cfg):
        self.cfg = cfg
        self.spec = B.make_spec(cfg)
        self.layout = B.hmy_layout(self.spec)
        self.n_params = B.hmy_model_size(self.spec)[1]
        self.mixed = cfg["precision"] == "bf16"
        wdtype = torch.bfloat16 if self.mixed else torch.float32
        n = self.n_params
        self.weights = torch.empty(n, dtype=wdtype, pin_memory=True)
        self.master = torch.empty(n, dtype=torch.float32, pin_memory=True) if self.mixed else None
        self.adam_m = torch.zeros(n, dtype=torch.float32, pin_memory=True)
        self.adam_v = torch.zeros(n, dtype=torch.float32, pin_memory=True)
        self.grads = torch.zeros(n, dtype=torch.float32, pin_memory=True)

    # -- named <-> flat -----------------------------------------------------------
    def _flat_set(self, flat: torch.Tensor, named) -> None:
        for t in self.layout:
            src = torch.from_numpy(np.ascontiguousarray(named[t["name"]], dtype=np.float32)).reshape(-1)
            flat[t["offset"]:t["offset"] + t["count"]].copy_(src.to(flat.dtype))

    def _flat_get(self, flat: torch.Tensor):
        out = {}
        for t in self.layout:
            a = flat[t["offset"]:t["offset"] + t["count"]].to(torch.float32).numpy().copy()
            out[t["name"]] = a.reshape(t["rows"], t["cols"]) if t["cols"] > 1 else a
        return out

    def load(self, params, m=None, v=None) -> None:
        """params: name -> fp32 array.  In bf16 mode they become the fp32 master and
        the compute weights are their round-to-nearest-even bf16 copy."""
        if self.mixed:
            self._flat_set(self.master, params)
            self.weights.copy_(self.master.to(torch.bfloat16))
        else:
            self._flat_set(self.weights, params)
        if m is not None:
            self._flat_set(self.adam_m, m)
        if v is not None:
            self._flat_set(self.adam_v, v)

    def fill_random(self, seed: int = 0, std: float = 0.02) -> None:
        """Benchmark init without the named round trip: matrices N(0, std^2),
        LayerNorm gains 1, everything else 0."""
        g = torch.Generator().manual_seed(seed)
        tgt = self.master if self.mixed else self.weights
        for t in self.layout:
            sl = tgt[t["offset"]:t["offset"] + t["count"]]
            base = t["name"].split(".")[-1]
            if t["cols"] > 1:
                sl.normal_(0.0, std, generator=g)
            elif base.endswith("_g"):
                sl.fill_(1.0)
            else:
                sl.zero_()
        if self.mixed:
            self.weights.copy_(self.master.to(torch.bfloat16))
        self.adam_m.zero_()
        self.adam_v.zero_()

    def named(self, what: str):
        """what in weights | master | m | v | grads -> name -> fp32 array."""
        flat = {"weights": self.weights, "master": self.master, "m": self.adam_m, "v": self.adam_v,
                "grads": self.grads}[what]
        return self._flat_get(flat)


class Engine:
    """One hmy handle bound to a TrainingState."""

    def __init__(self, state: TrainingState, budget_bytes: int, n_micro: int, micro_batch: int, sched=None,
                 device: int = 0, search: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("the engine needs a GPU (there is no CPU fallback)")
        self.state = state
        self.M, self.b = n_micro, micro_batch
        self.handle = B.hmy_create(state.spec, budget_bytes, n_micro, micro_batch, sched, device, search=search)
        self.sched = B.hmy_get_schedule(self.handle)
        self.packs = B.schedule_packs(self.sched)
        self.arena = B.hmy_arena(state.spec, self.sched, n_micro, micro_batch)
        B.hmy_bind_state(self.handle, state.weights.data_ptr(),
                         state.master.data_ptr() if state.mixed else None, state.adam_m.data_ptr(),
                         state.adam_v.data_ptr(), state.grads.data_ptr(), state.n_params)
        self._ids = None
        self._tgt = None

    def set_batch(self, ids: np.ndarray, targets: np.ndarray) -> None:
        s = self.state.cfg["seq_len"]
        assert ids.shape == (self.M, self.b, s) and targets.shape == ids.shape
        self._ids = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).pin_memory()
        self._tgt = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).pin_memory()

    def step(self, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, step=1, want_stats=True):
        return B.hmy_iteration(self.handle, self.M, self.b, self._ids.data_ptr(), self._tgt.data_ptr(), lr, beta1,
                               beta2, eps, step, want_stats)

    def close(self) -> None:
        if self.handle is not None:
            B.hmy_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
