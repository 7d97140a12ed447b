"""ctypes binding of libhmy.so: same names as include/hmy.h, argument marshalling only.

Every step of the training iteration runs inside the library's HIP kernels; this
module converts Python values to the C structs and raises HmyError on a
negative return code.  The library must have been built
(`python paper_2202_01306_amd/build.py`); importing this module without it fails.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhmy.so")

HMY_MAX_LAYERS = 512
HMY_NAME_LEN = 32
HMY_NKINDS = 7
KIND_NAMES = ("W", "dW", "K", "sX", "XY", "dXdY", "ids")
HMY_PREC_FP32, HMY_PREC_BF16 = 0, 1
HMY_ORDER_LAYER_PACK_MAJOR, HMY_ORDER_MICROBATCH_MAJOR = 0, 1
HMY_UPDATE_ON_DEVICE, HMY_UPDATE_ON_HOST = 0, 1
HMY_GRADIENTS_EXPORTED, HMY_GRADIENTS_ON_DEVICE = 0, 1
HMY_STATE_SWAPPED, HMY_STATE_RESIDENT_IN_SPARE_BUDGET = 0, 1
HMY_SWAP_OUT_KERNEL, HMY_SWAP_OUT_MEMCPY = 0, 1
HMY_MAX_WEIGHT_SLOTS = 4
(HMY_OK, HMY_E_INVALID, HMY_E_BUDGET_TOO_SMALL, HMY_E_BAD_SCHEDULE, HMY_E_HIP,
 HMY_E_NOT_BOUND, HMY_E_NO_DEVICE) = (0, -1, -2, -3, -4, -5, -6)


class HmyError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__(f"hmy error {code}: {detail}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2202_01306_amd/build.py` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)


class hmy_model_spec(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_blocks", "d_model", "n_heads", "d_ffn", "seq_len", "vocab",
                                         "causal", "precision")] + [("ln_eps", C.c_float)]


class hmy_measured_profile(C.Structure):
    _fields_ = [("micro_batch", C.c_int32), ("reserved_", C.c_int32), ("embed_fwd_ns", C.c_uint64),
                ("embed_bwd_ns", C.c_uint64), ("block_fwd_ns", C.c_uint64), ("block_bwd_ns", C.c_uint64),
                ("head_ns", C.c_uint64), ("embed_fwd_beside_ns", C.c_uint64), ("embed_bwd_beside_ns", C.c_uint64),
                ("block_fwd_beside_ns", C.c_uint64), ("block_bwd_beside_ns", C.c_uint64), ("head_beside_ns", C.c_uint64)]


MEASURED_FIELDS = ("micro_batch", "embed_fwd_ns", "embed_bwd_ns", "block_fwd_ns", "block_bwd_ns", "head_ns")
MEASURED_BESIDE_FIELDS = ("embed_fwd_beside_ns", "embed_bwd_beside_ns", "block_fwd_beside_ns", "block_bwd_beside_ns",
                          "head_beside_ns")


class hmy_budget(C.Structure):
    _fields_ = [("hbm_budget_bytes", C.c_uint64), ("host_link_MBps", C.c_uint32), ("compute_GFLOPs", C.c_uint32),
                ("max_extra_packs", C.c_uint32), ("update_site", C.c_uint32), ("min_weight_slots", C.c_uint32),
                ("max_weight_slots", C.c_uint32), ("max_fwd_micro_batch", C.c_uint32),
                ("max_bwd_micro_batch", C.c_uint32), ("n_measured", C.c_uint32),
                ("measured", C.POINTER(hmy_measured_profile))]


def make_budget(budget_bytes, search=0, link_MBps=0, compute_GFLOPs=0, update_site=0, slots=(0, 0), max_fwd_micro_batch=0,
                max_bwd_micro_batch=0, measured=None) -> hmy_budget:
    """slots: (min, max) weight slots to sweep (0 = 3); measured: list of dicts with MEASURED_FIELDS (what
    hmy_measure_profile returns), one per microbatch size."""
    b = hmy_budget(int(budget_bytes), int(link_MBps), int(compute_GFLOPs), int(search), int(update_site),
                   int(slots[0]), int(slots[1]), int(max_fwd_micro_batch), int(max_bwd_micro_batch), 0, None)
    if measured:
        arr = (hmy_measured_profile * len(measured))()
        for i, mp in enumerate(measured):
            for f in MEASURED_FIELDS:
                setattr(arr[i], f, int(mp[f]))
            for f in MEASURED_BESIDE_FIELDS:      # optional: 0 = as alone
                setattr(arr[i], f, int(mp.get(f, 0)))
        b.n_measured = len(measured)
        b.measured = C.cast(arr, C.POINTER(hmy_measured_profile))
        b._keep = arr      # the struct only holds the address
    return b


class hmy_schedule(C.Structure):
    _fields_ = [("n_fwd_packs", C.c_int32), ("n_bwd_packs", C.c_int32),
                ("fwd_pack_end", C.c_int32 * HMY_MAX_LAYERS), ("bwd_pack_end", C.c_int32 * HMY_MAX_LAYERS),
                ("order", C.c_int32), ("update_site", C.c_int32), ("gradients", C.c_int32), ("resident_state", C.c_int32),
                ("swap_out", C.c_int32), ("weight_slots", C.c_int32), ("prefetch_distance", C.c_int32),
                ("fwd_micro_batch", C.c_int32), ("bwd_micro_batch", C.c_int32)]


class hmy_minibatch(C.Structure):
    _fields_ = [("n_micro", C.c_int32), ("micro_batch", C.c_int32),
                ("token_ids", C.c_void_p), ("targets", C.c_void_p)]


class hmy_adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("step", C.c_int64)]


class hmy_host_state(C.Structure):
    _fields_ = [("weights", C.c_void_p), ("master", C.c_void_p), ("adam_m", C.c_void_p),
                ("adam_v", C.c_void_p), ("grads", C.c_void_p), ("n_params", C.c_uint64)]


class hmy_stats(C.Structure):
    _fields_ = [("h2d", C.c_uint64 * HMY_NKINDS), ("d2h", C.c_uint64 * HMY_NKINDS), ("loss", C.c_double),
                ("t_iter_s", C.c_double), ("t_compute_s", C.c_double), ("t_h2d_busy_s", C.c_double),
                ("t_d2h_busy_s", C.c_double), ("t_stall_s", C.c_double), ("n_targets", C.c_uint64),
                ("gemm_calls", C.c_uint64 * 4), ("gemm_flops", C.c_double * 4), ("gemm_s", C.c_double * 4),
                ("t_event_pair_s", C.c_double)]


class hmy_tensor_desc(C.Structure):
    _fields_ = [("name", C.c_char * HMY_NAME_LEN), ("layer", C.c_int32), ("rows", C.c_int32),
                ("cols", C.c_int32), ("offset", C.c_uint64), ("count", C.c_uint64)]


class hmy_layer_profile(C.Structure):
    _fields_ = [("ns_fwd", C.c_int64), ("ns_bwd", C.c_int64), ("ns_fwd_beside", C.c_int64), ("ns_bwd_beside", C.c_int64),
                ("flops_fwd", C.c_int64), ("params", C.c_uint64),
                ("mem_fwd", C.c_uint64), ("mem_bwd", C.c_uint64), ("act_bwd", C.c_uint64)]


class hmy_arena_plan(C.Structure):
    _fields_ = [("total", C.c_uint64), ("reserved", C.c_uint64), ("slot_bytes", C.c_uint64),
                ("act_bytes", C.c_uint64), ("k_chunk_params", C.c_uint64), ("weight_slots", C.c_int32),
                ("prefetch_distance", C.c_int32), ("fwd_micro_batch", C.c_int32), ("bwd_micro_batch", C.c_int32)]


class hmy_region(C.Structure):
    _fields_ = [("name", C.c_char * HMY_NAME_LEN), ("offset", C.c_uint64), ("bytes", C.c_uint64)]


class hmy_gemm_desc(C.Structure):
    _fields_ = [("prec", C.c_int32), ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("ta", C.c_int32), ("tb", C.c_int32), ("c_fp32", C.c_int32), ("accumulate", C.c_int32),
                ("A", C.c_void_p), ("lda", C.c_int64), ("B", C.c_void_p), ("ldb", C.c_int64),
                ("C", C.c_void_p), ("ldc", C.c_int64), ("bias", C.c_void_p),
                ("res", C.c_void_p), ("ldr", C.c_int64), ("gelu_out", C.c_void_p), ("res_fp32", C.c_int32)]


EXPORTS = [
    "hmy_strerror", "hmy_last_error", "hmy_model_size", "hmy_layout", "hmy_profile", "hmy_plan", "hmy_estimate", "hmy_arena",
    "hmy_arena_regions", "hmy_measure_profile",
    "hmy_count_swaps", "hmy_host_alloc", "hmy_host_free", "hmy_create", "hmy_get_schedule", "hmy_bind_state", "hmy_resident_params", "hmy_sync_state",
    "hmy_iteration", "hmy_destroy", "hmy_set_profiling", "hmy_set_progress", "hmy_set_kernel_path", "hmy_k_embed_fwd", "hmy_k_embed_bwd",
    "hmy_k_layernorm_fwd", "hmy_k_layernorm_bwd", "hmy_k_layernorm_bwd_static", "hmy_k_gelu_fwd", "hmy_k_gelu_bwd", "hmy_k_gelu_bwd_colsum", "hmy_k_colsum",
    "hmy_k_gemm", "hmy_k_attn_fwd", "hmy_k_attn_bwd", "hmy_k_xent", "hmy_k_adam", "hmy_host_adam",
]

lib.hmy_strerror.restype = C.c_char_p
lib.hmy_last_error.restype = C.c_char_p
for _n in EXPORTS[2:]:
    getattr(lib, _n).restype = C.c_int


def _check(rc: int) -> None:
    if rc != 0:
        raise HmyError(rc, (lib.hmy_last_error() or b"").decode() or lib.hmy_strerror(rc).decode())


def make_spec(cfg) -> hmy_model_spec:
    """cfg: mapping with n_blocks, d_model, n_heads, d_ffn, seq_len, vocab, causal, precision('fp32'|'bf16')."""
    prec = {"fp32": HMY_PREC_FP32, "bf16": HMY_PREC_BF16}[cfg["precision"]]
    return hmy_model_spec(cfg["n_blocks"], cfg["d_model"], cfg["n_heads"], cfg["d_ffn"], cfg["seq_len"],
                          cfg["vocab"], int(cfg["causal"]), prec, float(cfg.get("ln_eps", 1e-5)))


def make_schedule(fwd_ends, bwd_ends, order=0, update_site=0, gradients=0, resident_state=0, swap_out=0, slots=0,
                  distance=0, fwd_micro_batch=0, bwd_micro_batch=0) -> hmy_schedule:
    s = hmy_schedule()
    s.order = order
    s.update_site = update_site
    s.gradients = gradients
    s.resident_state = resident_state
    s.swap_out = swap_out
    s.weight_slots = slots
    s.prefetch_distance = distance
    s.fwd_micro_batch = fwd_micro_batch
    s.bwd_micro_batch = bwd_micro_batch
    s.n_fwd_packs, s.n_bwd_packs = len(fwd_ends), len(bwd_ends)
    for i, e in enumerate(fwd_ends):
        s.fwd_pack_end[i] = e
    for i, e in enumerate(bwd_ends):
        s.bwd_pack_end[i] = e
    return s


def schedule_packs(s: hmy_schedule):
    """-> (P_F, P_B) as lists of (start, end)."""
    def ranges(ends):
        out, pos = [], 0
        for e in ends:
            out.append((pos, e))
            pos = e
        return out
    return (ranges(list(s.fwd_pack_end[:s.n_fwd_packs])), ranges(list(s.bwd_pack_end[:s.n_bwd_packs])))


# ---- host-only ------------------------------------------------------------------

def hmy_model_size(spec):
    nl, npar = C.c_int32(), C.c_uint64()
    _check(lib.hmy_model_size(C.byref(spec), C.byref(nl), C.byref(npar)))
    return nl.value, npar.value


def hmy_layout(spec):
    n = C.c_int32()
    _check(lib.hmy_layout(C.byref(spec), None, 0, C.byref(n)))
    arr = (hmy_tensor_desc * n.value)()
    _check(lib.hmy_layout(C.byref(spec), arr, n.value, C.byref(n)))
    return [dict(name=t.name.decode(), layer=t.layer, rows=t.rows, cols=t.cols, offset=t.offset, count=t.count)
            for t in arr]


def hmy_profile(spec, n_micro, micro_batch, sched=None, budget=None):
    """-> (per-layer profile, pack-independent reserve in bytes) for the microbatch sizes and slot count of
    `sched` (None: the caller's micro_batch, three slots) and the rates / measurements of `budget` (a make_budget)."""
    R, _ = hmy_model_size(spec)
    arr = (hmy_layer_profile * R)()
    res = C.c_uint64()
    _check(lib.hmy_profile(C.byref(spec), C.byref(budget) if budget is not None else None,
                           C.byref(sched) if sched is not None else None, n_micro, micro_batch, arr, C.byref(res)))
    prof = [dict(ns_fwd=p.ns_fwd, ns_bwd=p.ns_bwd, ns_fwd_beside=p.ns_fwd_beside, ns_bwd_beside=p.ns_bwd_beside,
                 flops_fwd=p.flops_fwd, params=p.params, mem_fwd=p.mem_fwd,
                 mem_bwd=p.mem_bwd, act_bwd=p.act_bwd) for p in arr]
    return prof, res.value


def hmy_plan(spec, budget_bytes, n_micro, micro_batch, search=0, link_MBps=0, compute_GFLOPs=0,
             update_site=0, **budget_kw) -> hmy_schedule:
    """budget_kw: slots=(min, max), max_fwd_micro_batch, max_bwd_micro_batch, measured (see make_budget)."""
    s = hmy_schedule()
    b = make_budget(budget_bytes, search, link_MBps, compute_GFLOPs, update_site, **budget_kw)
    _check(lib.hmy_plan(C.byref(spec), C.byref(b), n_micro, micro_batch, C.byref(s)))
    return s


def hmy_estimate(spec, sched, n_micro, micro_batch, link_MBps=0, compute_GFLOPs=0, measured=None) -> int:
    ns = C.c_uint64()
    b = make_budget(0, 0, link_MBps, compute_GFLOPs, measured=measured)
    _check(lib.hmy_estimate(C.byref(spec), C.byref(sched), C.byref(b), n_micro, micro_batch, C.byref(ns)))
    return ns.value


def hmy_arena(spec, sched, n_micro, micro_batch):
    a = hmy_arena_plan()
    _check(lib.hmy_arena(C.byref(spec), C.byref(sched), n_micro, micro_batch, C.byref(a)))
    return dict(total=a.total, reserved=a.reserved, slot_bytes=a.slot_bytes, act_bytes=a.act_bytes,
                k_chunk_params=a.k_chunk_params, weight_slots=a.weight_slots, prefetch_distance=a.prefetch_distance,
                fwd_micro_batch=a.fwd_micro_batch, bwd_micro_batch=a.bwd_micro_batch)


def hmy_arena_regions(spec, sched, n_micro, micro_batch):
    """-> [(name, offset, bytes)] of every buffer the engine addresses inside its arena."""
    n = C.c_int32()
    _check(lib.hmy_arena_regions(C.byref(spec), C.byref(sched), n_micro, micro_batch, None, 0, C.byref(n)))
    arr = (hmy_region * n.value)()
    _check(lib.hmy_arena_regions(C.byref(spec), C.byref(sched), n_micro, micro_batch, arr, n.value, C.byref(n)))
    return [(r.name.decode(), r.offset, r.bytes) for r in arr]


def hmy_measure_profile(spec, micro_batch, device=0, reps=3):
    """Per-layer times of this library's kernels on the device for one microbatch size, alone and beside
    host-link traffic (needs a GPU)."""
    mp = hmy_measured_profile()
    _check(lib.hmy_measure_profile(C.byref(spec), micro_batch, device, reps, C.byref(mp)))
    return {f: getattr(mp, f) for f in MEASURED_FIELDS + MEASURED_BESIDE_FIELDS}


def _stats_dict(st: hmy_stats):
    return dict(h2d={k: st.h2d[i] for i, k in enumerate(KIND_NAMES)},
                d2h={k: st.d2h[i] for i, k in enumerate(KIND_NAMES)},
                loss=st.loss, t_iter_s=st.t_iter_s, t_compute_s=st.t_compute_s, t_h2d_busy_s=st.t_h2d_busy_s,
                t_d2h_busy_s=st.t_d2h_busy_s, t_stall_s=st.t_stall_s, n_targets=st.n_targets,
                gemm_calls=list(st.gemm_calls), gemm_flops=list(st.gemm_flops), gemm_s=list(st.gemm_s),
                t_event_pair_s=st.t_event_pair_s)


def hmy_count_swaps(spec, sched, n_micro, micro_batch):
    st = hmy_stats()
    _check(lib.hmy_count_swaps(C.byref(spec), C.byref(sched), n_micro, micro_batch, C.byref(st)))
    return _stats_dict(st)


def hmy_set_kernel_path(use_mfma) -> None:
    """False/0: reference kernels; True/1: MFMA kernels; 2: MFMA without the large-tile GEMM."""
    _check(lib.hmy_set_kernel_path(int(use_mfma)))


# ---- device ---------------------------------------------------------------------

def hmy_host_alloc(nbytes: int) -> int:
    p = C.c_void_p()
    _check(lib.hmy_host_alloc(C.c_uint64(nbytes), C.byref(p)))
    return p.value


def hmy_host_free(ptr: int) -> None:
    _check(lib.hmy_host_free(C.c_void_p(ptr)))


def hmy_create(spec, budget_bytes, n_micro, micro_batch, sched=None, device=0, arena_ptr=None, arena_bytes=0,
               search=0, link_MBps=0, compute_GFLOPs=0, **budget_kw):
    h = C.c_void_p()
    budget = make_budget(budget_bytes, search, link_MBps, compute_GFLOPs, **budget_kw)
    _check(lib.hmy_create(C.byref(spec), C.byref(budget),
                          n_micro, micro_batch,
                          C.byref(sched) if sched is not None else None, device,
                          C.c_void_p(arena_ptr) if arena_ptr else None, C.c_uint64(arena_bytes), C.byref(h)))
    return h


def hmy_get_schedule(h) -> hmy_schedule:
    s = hmy_schedule()
    _check(lib.hmy_get_schedule(h, C.byref(s)))
    return s


def hmy_bind_state(h, weights_ptr, master_ptr, m_ptr, v_ptr, grads_ptr, n_params):
    st = hmy_host_state(weights_ptr, master_ptr, m_ptr, v_ptr, grads_ptr, n_params)
    _check(lib.hmy_bind_state(h, C.byref(st)))


def hmy_resident_params(h) -> int:
    n = C.c_uint64()
    _check(lib.hmy_resident_params(h, C.byref(n)))
    return n.value


def hmy_sync_state(h):
    _check(lib.hmy_sync_state(h))


def hmy_iteration(h, n_micro, micro_batch, ids_ptr, targets_ptr, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8,
                  step=1, want_stats=True):
    mb = hmy_minibatch(n_micro, micro_batch, ids_ptr, targets_ptr)
    hp = hmy_adam(lr, beta1, beta2, eps, step)
    st = hmy_stats()
    _check(lib.hmy_iteration(h, C.byref(mb), C.byref(hp), C.byref(st) if want_stats else None))
    return _stats_dict(st) if want_stats else None


def hmy_destroy(h) -> None:
    _check(lib.hmy_destroy(h))


def hmy_set_profiling(h, level: int) -> None:
    """0: counters, loss, host-clock time; 1: + copy / stall / compute spans; 2: + every GEMM launch."""
    _check(lib.hmy_set_profiling(h, int(level)))


def hmy_set_progress(h, on: bool) -> None:
    """A line on stderr after every visit (the iteration then waits for each visit's kernels)."""
    _check(lib.hmy_set_progress(h, int(bool(on))))


def _p(x):
    """Device/host address of a torch tensor, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    return C.c_void_p(x.data_ptr())


def hmy_k_embed_fwd(prec, ids, wte, wpe, x, T, d, s, vocab, stream=None):
    _check(lib.hmy_k_embed_fwd(prec, _p(ids), _p(wte), _p(wpe), _p(x), T, d, s, vocab, _p(stream)))


def hmy_k_embed_bwd(prec, ids, dx, dwte, dwpe, T, d, s, vocab, stream=None):
    _check(lib.hmy_k_embed_bwd(prec, _p(ids), _p(dx), _p(dwte), _p(dwpe), T, d, s, vocab, _p(stream)))


def hmy_k_layernorm_fwd(prec, x, gamma, beta, y, mean, rstd, T, d, eps, stream=None):
    _check(lib.hmy_k_layernorm_fwd(prec, _p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(rstd), T, d,
                                   C.c_float(eps), _p(stream)))


def hmy_k_layernorm_bwd(prec, dy, x, mean, rstd, gamma, res, dx, dgamma, dbeta, T, d, stream=None, workspace=None,
                        dx_e=None, dres_sum=None):
    """x, res, dx: fp32 (the residual stream); dy, gamma: element type; dx_e: optional element-typed copy of dx;
    dres_sum: optional fp32 [d], += column sums of res."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hmy_k_layernorm_bwd(prec, _p(dy), _p(x), _p(mean), _p(rstd), _p(gamma), _p(res), _p(dx), _p(dx_e),
                                   _p(dgamma), _p(dbeta), _p(dres_sum), T, d, _p(stream), _p(workspace),
                                   C.c_uint64(ws_bytes)))


def hmy_k_layernorm_bwd_static(prec, dy, x, mean, rstd, gamma, res, dx, dgamma, dbeta, T, d, stream=None, dx_e=None):
    _check(lib.hmy_k_layernorm_bwd_static(prec, _p(dy), _p(x), _p(mean), _p(rstd), _p(gamma), _p(res), _p(dx), _p(dx_e),
                                          _p(dgamma), _p(dbeta), T, d, _p(stream)))


def hmy_k_gelu_fwd(prec, u, g, n, stream=None):
    _check(lib.hmy_k_gelu_fwd(prec, _p(u), _p(g), C.c_uint64(n), _p(stream)))


def hmy_k_gelu_bwd(prec, dg, u, du, n, stream=None):
    _check(lib.hmy_k_gelu_bwd(prec, _p(dg), _p(u), _p(du), C.c_uint64(n), _p(stream)))


def hmy_k_gelu_bwd_colsum(prec, dg, u, du, db, T, N, stream=None):
    _check(lib.hmy_k_gelu_bwd_colsum(prec, _p(dg), _p(u), _p(du), _p(db), T, N, _p(stream)))


def hmy_k_colsum(prec, a, out, T, N, stream=None):
    _check(lib.hmy_k_colsum(prec, _p(a), _p(out), T, N, _p(stream)))


def hmy_k_gemm(prec, M, N, K, A, lda, B, ldb, Cc, ldc, ta=0, tb=0, c_fp32=0, accumulate=0, bias=None, res=None,
               ldr=0, gelu_out=None, stream=None, res_fp32=0):
    g = hmy_gemm_desc(prec, M, N, K, ta, tb, c_fp32, accumulate, _p(A), lda, _p(B), ldb, _p(Cc), ldc,
                      _p(bias), _p(res), ldr, _p(gelu_out), res_fp32)
    _check(lib.hmy_k_gemm(C.byref(g), _p(stream)))


def hmy_k_attn_fwd(prec, qkv, o, lse, b, s, H, dh, causal, stream=None):
    _check(lib.hmy_k_attn_fwd(prec, _p(qkv), _p(o), _p(lse), b, s, H, dh, int(causal), _p(stream)))


def hmy_k_attn_bwd(prec, qkv, o, d_o, lse, delta, dqkv, b, s, H, dh, causal, stream=None, dbias=None):
    _check(lib.hmy_k_attn_bwd(prec, _p(qkv), _p(o), _p(d_o), _p(lse), _p(delta), _p(dqkv), _p(dbias), b, s, H, dh,
                              int(causal), _p(stream)))


def hmy_k_xent(prec, logits, targets, loss_acc, dlogits, T, V, ldl, inv_ntgt, stream=None):
    _check(lib.hmy_k_xent(prec, _p(logits), _p(targets), _p(loss_acc), _p(dlogits), T, V, C.c_int64(ldl),
                          C.c_float(inv_ntgt), _p(stream)))


def hmy_host_adam(prec, grad_ptr, master_ptr, m_ptr, v_ptr, weights_ptr, n, lr, beta1, beta2, eps, step, threads=0):
    """Host pointers (ints); in place."""
    hp = hmy_adam(lr, beta1, beta2, eps, step)
    vp = lambda x: C.c_void_p(x) if x else None
    _check(lib.hmy_host_adam(prec, vp(grad_ptr), vp(master_ptr), vp(m_ptr), vp(v_ptr), vp(weights_ptr), C.c_uint64(n),
                             C.byref(hp), int(threads)))


def hmy_k_adam(prec, grad, master, m, v, w_out, n, lr, beta1, beta2, eps, step, stream=None):
    hp = hmy_adam(lr, beta1, beta2, eps, step)
    _check(lib.hmy_k_adam(prec, _p(grad), _p(master), _p(m), _p(v), _p(w_out), C.c_uint64(n), C.byref(hp),
                          _p(stream)))
