"""Thin ctypes binding of libadaptra.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch supplies device
memory (tensors) and the current stream; nothing here computes.  If the library is
missing this module raises -- there is no CPU fallback.

Names and arguments mirror include/adaptra.h.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadaptra.so")

OK, EINVAL, EWORKSPACE, EHIP, ERANGE, EOVERFLOW, ELIMIT = 0, 1, 2, 3, 4, 5, 6
ERROR_NAMES = {0: "ADAPTRA_OK", 1: "ADAPTRA_EINVAL", 2: "ADAPTRA_EWORKSPACE", 3: "ADAPTRA_EHIP",
               4: "ADAPTRA_ERANGE", 5: "ADAPTRA_EOVERFLOW", 6: "ADAPTRA_ELIMIT"}
STATIC_MAX_CANDIDATES, STATIC_MAX_SCENARIOS, STATIC_MAX_MICROBATCHES = 65536, 4096, 1024
FLAG_FEASIBLE, FLAG_DEADLOCK, FLAG_MEMCAP = 1, 2, 4
INT32_MAX = 2 ** 31 - 1

# include/adaptra.h
EXPORTS = ("adaptra_workspace_bytes", "adaptra_best_workspace_bytes", "adaptra_search_workspace_bytes", "adaptra_search",
           "adaptra_check_inputs", "adaptra_eval", "adaptra_best", "adaptra_best_static", "adaptra_eval_best",
           "adaptra_seed", "adaptra_sensitivity_workspace_bytes", "adaptra_sensitivity",
           "adaptra_zb_workspace_bytes", "adaptra_zb_check_inputs", "adaptra_zb_eval",
           "adaptra_last_hip_error", "adaptra_version")
# include/adaptra_testing.h
TESTING_EXPORTS = ("adaptra_set_kernel_mode", "adaptra_set_resolve_events", "adaptra_valu_probe")
PROBE_MIXES = ("add_max", "add_vgpr", "add_sgpr", "add_inline", "add_literal", "add_e64", "sub", "add_co", "add3", "max", "max_sgpr", "max_e64", "max_u32", "min", "max3", "med3", "and", "or", "xor", "lshl", "mov", "cndmask", "cndmask_sgpr", "cndmask_bfe", "cmp_cndmask", "add_max_alt", "add_max_batch", "add_max_batch_nop", "add_max_alt_dense", "readlane", "forward_step")


class AdaptraError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        self.hip_error = hip
        extra = f" (hipError_t {hip})" if code == EHIP else ""
        super().__init__(f"{where}: {ERROR_NAMES.get(code, code)}{extra}")


class Params(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("M", ctypes.c_int32),
                ("t_f", ctypes.c_void_p), ("t_b", ctypes.c_void_p), ("mem_cap", ctypes.c_void_p),
                ("hist_bins", ctypes.c_int32), ("hist_shift", ctypes.c_int32)]


class Candidates(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("w", ctypes.c_void_p), ("w_bound", ctypes.c_int32)]


class Scenarios(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("c_fwd", ctypes.c_void_p), ("c_bwd", ctypes.c_void_p),
                ("t_f", ctypes.c_void_p), ("t_b", ctypes.c_void_p)]


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library built in-tree; fail loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_19232_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        P, C, Sc = ctypes.POINTER(Params), ctypes.POINTER(Candidates), ctypes.POINTER(Scenarios)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        lib.adaptra_workspace_bytes.restype = sz
        lib.adaptra_workspace_bytes.argtypes = [P, ctypes.c_int64, ctypes.c_int64]
        lib.adaptra_best_workspace_bytes.restype = sz
        lib.adaptra_best_workspace_bytes.argtypes = [P, ctypes.c_int64, ctypes.c_int64]
        lib.adaptra_search_workspace_bytes.restype = sz
        lib.adaptra_search_workspace_bytes.argtypes = [P, ctypes.c_int64, ctypes.c_int32]
        lib.adaptra_search.restype = ctypes.c_int
        lib.adaptra_search.argtypes = [P, Sc, vp, ctypes.c_int32, ctypes.c_int32, vp, vp,
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64), vp, sz, vp]
        lib.adaptra_check_inputs.restype = ctypes.c_int
        lib.adaptra_check_inputs.argtypes = [P, C, Sc, vp, sz, vp]
        lib.adaptra_eval.restype = ctypes.c_int
        lib.adaptra_eval.argtypes = [P, C, Sc, vp, vp, vp, vp, sz, vp]
        lib.adaptra_best.restype = ctypes.c_int
        lib.adaptra_best.argtypes = [P, C, Sc, vp, vp, vp, vp, vp, sz, vp]
        lib.adaptra_eval_best.restype = ctypes.c_int
        lib.adaptra_eval_best.argtypes = [P, C, Sc, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.adaptra_seed.restype = ctypes.c_int
        lib.adaptra_seed.argtypes = [P, Sc, ctypes.c_int32, vp, vp, vp, vp, vp]
        lib.adaptra_sensitivity_workspace_bytes.restype = sz
        lib.adaptra_sensitivity_workspace_bytes.argtypes = [P, ctypes.c_int64, ctypes.c_int64]
        lib.adaptra_sensitivity.restype = ctypes.c_int
        lib.adaptra_sensitivity.argtypes = [P, C, Sc, ctypes.c_int32, vp, vp, vp, vp, sz, vp]
        lib.adaptra_zb_workspace_bytes.restype = sz
        lib.adaptra_zb_workspace_bytes.argtypes = [P, ctypes.c_int64, ctypes.c_int64]
        lib.adaptra_zb_eval.restype = ctypes.c_int
        lib.adaptra_zb_eval.argtypes = [P, vp, C, Sc, ctypes.c_int64, vp, vp, vp, sz, vp]
        lib.adaptra_set_kernel_mode.restype = ctypes.c_int
        lib.adaptra_set_kernel_mode.argtypes = [ctypes.c_int]
        lib.adaptra_set_resolve_events.restype = ctypes.c_int
        lib.adaptra_set_resolve_events.argtypes = [vp, vp]
        lib.adaptra_valu_probe.restype = ctypes.c_int
        lib.adaptra_valu_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp,
                                           ctypes.POINTER(ctypes.c_int64)]
        lib.adaptra_best_static.restype = ctypes.c_int
        lib.adaptra_best_static.argtypes = [P, C, Sc, vp, vp, vp, vp, vp]
        lib.adaptra_zb_check_inputs.restype = ctypes.c_int
        lib.adaptra_zb_check_inputs.argtypes = [P, vp, C, Sc, vp, sz, vp]
        lib.adaptra_last_hip_error.restype = ctypes.c_int
        lib.adaptra_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check_i32(t, name, shape=None):
    import torch
    if t is None:
        return
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous int32 CUDA tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


class Problem:
    """Device-resident inputs of one batch, plus the marshalled structs.

    t_f, t_b, mem_cap: int32 [S]; w: int32 [S, C]; c_fwd, c_bwd: int32 [S-1, K] -- all CUDA
    tensors, kept alive by this object."""

    def __init__(self, M: int, t_f, t_b, w, c_fwd, c_bwd, mem_cap=None, hist_bins: int = 0, hist_shift: int = 0,
                 w_bound: int = -1, t_f_scen=None, t_b_scen=None):
        S = int(t_f.shape[0])
        C = int(w.shape[1])
        K = int(c_fwd.shape[1])
        _check_i32(t_f, "t_f", (S,)); _check_i32(t_b, "t_b", (S,)); _check_i32(mem_cap, "mem_cap", (S,))
        _check_i32(w, "w", (S, C)); _check_i32(c_fwd, "c_fwd", (S - 1, K)); _check_i32(c_bwd, "c_bwd", (S - 1, K))
        self.S, self.M, self.C, self.K = S, int(M), C, K
        self.hist_bins, self.hist_shift = int(hist_bins), int(hist_shift)
        _check_i32(t_f_scen, "t_f_scen", (S, K)); _check_i32(t_b_scen, "t_b_scen", (S, K))
        self.tensors = (t_f, t_b, w, c_fwd, c_bwd, mem_cap, t_f_scen, t_b_scen)
        self.device = w.device
        self.params = Params(S, int(M), _ptr(t_f), _ptr(t_b), _ptr(mem_cap), int(hist_bins), int(hist_shift))
        self.cands = Candidates(C, _ptr(w), int(w_bound))
        self.scens = Scenarios(K, _ptr(c_fwd) if S > 1 else None, _ptr(c_bwd) if S > 1 else None,
                               _ptr(t_f_scen), _ptr(t_b_scen))

    @classmethod
    def from_workload(cls, wl, device="cuda:0", w_bound: int = -1, t_f_scen=None, t_b_scen=None):
        import torch
        dev = torch.device(device)

        def up(a):
            return None if a is None else torch.from_numpy(a).to(dev)
        return cls(wl.M, up(wl.t_f), up(wl.t_b), up(wl.w), up(wl.c_fwd), up(wl.c_bwd), up(wl.mem_cap),
                   wl.hist_bins, wl.hist_shift, w_bound, up(t_f_scen), up(t_b_scen))


def adaptra_workspace_bytes(S: int, M: int, n_cand: int, n_scen: int) -> int:
    p = Params(S, M, None, None, None, 0, 0)
    return int(load().adaptra_workspace_bytes(ctypes.byref(p), n_cand, n_scen))


def alloc_workspace(prob: Problem):
    import torch
    n = adaptra_workspace_bytes(prob.S, prob.M, prob.C, prob.K)
    if n == 0:
        raise AdaptraError(EINVAL, "adaptra_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=prob.device)


def _raise(rc: int, where: str):
    if rc != OK:
        raise AdaptraError(rc, where, load().adaptra_last_hip_error())


def adaptra_check_inputs(prob: Problem, workspace=None, stream=None) -> int:
    """Returns the library's code (OK, ERANGE, EOVERFLOW ...) without raising for data findings."""
    ws = alloc_workspace(prob) if workspace is None else workspace
    rc = load().adaptra_check_inputs(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                                     ws.data_ptr(), ws.numel(), _stream(stream))
    if rc in (EINVAL, EWORKSPACE, EHIP):
        _raise(rc, "adaptra_check_inputs")
    return rc


def adaptra_eval(prob: Problem, out_makespan=None, out_bubble=None, out_feasible=None, *,
                 want_bubble: bool = True, workspace=None, stream=None):
    """Enqueue the evaluation of every pair; returns (makespan [K,C], bubble [S,K,C] | None, feasible [K,C])."""
    import torch
    dev = prob.device
    if out_makespan is None:
        out_makespan = torch.empty((prob.K, prob.C), dtype=torch.int32, device=dev)
    if out_feasible is None:
        out_feasible = torch.empty((prob.K, prob.C), dtype=torch.uint8, device=dev)
    if out_bubble is None and want_bubble:
        out_bubble = torch.empty((prob.S, prob.K, prob.C), dtype=torch.int32, device=dev)
    ws = alloc_workspace(prob) if workspace is None else workspace
    rc = load().adaptra_eval(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                             out_makespan.data_ptr(), _ptr(out_bubble), out_feasible.data_ptr(),
                             ws.data_ptr(), ws.numel(), _stream(stream))
    _raise(rc, "adaptra_eval")
    return out_makespan, out_bubble, out_feasible


def adaptra_best(prob: Problem, out_best_idx=None, out_best_makespan=None, out_best_bubble=None, out_hist=None, *,
                 want_bubble: bool = True, workspace=None, stream=None):
    """Enqueue the per-scenario search; returns (best_idx [K], best_makespan [K], best_bubble [K,S] | None,
    hist [S,bins] | None)."""
    import torch
    dev = prob.device
    if out_best_idx is None:
        out_best_idx = torch.empty(prob.K, dtype=torch.int32, device=dev)
    if out_best_makespan is None:
        out_best_makespan = torch.empty(prob.K, dtype=torch.int32, device=dev)
    if out_best_bubble is None and want_bubble:
        out_best_bubble = torch.empty((prob.K, prob.S), dtype=torch.int32, device=dev)
    if out_hist is None and prob.hist_bins > 0:
        out_hist = torch.empty((prob.S, prob.hist_bins), dtype=torch.int64, device=dev)
    ws = alloc_workspace(prob) if workspace is None else workspace
    rc = load().adaptra_best(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                             out_best_idx.data_ptr(), out_best_makespan.data_ptr(), _ptr(out_best_bubble),
                             _ptr(out_hist), ws.data_ptr(), ws.numel(), _stream(stream))
    _raise(rc, "adaptra_best")
    return out_best_idx, out_best_makespan, out_best_bubble, out_hist


def adaptra_best_static(prob: Problem, out_best_idx, out_best_makespan, out_best_bubble=None, out_hist=None, *,
                        stream=None):
    """Enqueue the per-scenario search on the library's own fixed scratch: the caller passes every
    output, nothing is allocated here or in the library."""
    rc = load().adaptra_best_static(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                                    out_best_idx.data_ptr(), out_best_makespan.data_ptr(), _ptr(out_best_bubble),
                                    _ptr(out_hist), _stream(stream))
    _raise(rc, "adaptra_best_static")
    return out_best_idx, out_best_makespan, out_best_bubble, out_hist


def adaptra_eval_best(prob: Problem, out_makespan=None, out_bubble=None, out_feasible=None, out_best_idx=None,
                      out_best_makespan=None, out_best_bubble=None, out_hist=None, *, want_bubble: bool = True,
                      workspace=None, stream=None):
    """Enqueue evaluation and search in one pass; returns the outputs of adaptra_eval followed by
    those of adaptra_best: (makespan, bubble | None, feasible, best_idx, best_makespan,
    best_bubble | None, hist | None)."""
    import torch
    dev = prob.device
    if out_makespan is None:
        out_makespan = torch.empty((prob.K, prob.C), dtype=torch.int32, device=dev)
    if out_feasible is None:
        out_feasible = torch.empty((prob.K, prob.C), dtype=torch.uint8, device=dev)
    if out_bubble is None and want_bubble:
        out_bubble = torch.empty((prob.S, prob.K, prob.C), dtype=torch.int32, device=dev)
    if out_best_idx is None:
        out_best_idx = torch.empty(prob.K, dtype=torch.int32, device=dev)
    if out_best_makespan is None:
        out_best_makespan = torch.empty(prob.K, dtype=torch.int32, device=dev)
    if out_best_bubble is None and want_bubble:
        out_best_bubble = torch.empty((prob.K, prob.S), dtype=torch.int32, device=dev)
    if out_hist is None and prob.hist_bins > 0:
        out_hist = torch.empty((prob.S, prob.hist_bins), dtype=torch.int64, device=dev)
    ws = alloc_workspace(prob) if workspace is None else workspace
    rc = load().adaptra_eval_best(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                                  out_makespan.data_ptr(), _ptr(out_bubble), out_feasible.data_ptr(),
                                  out_best_idx.data_ptr(), out_best_makespan.data_ptr(), _ptr(out_best_bubble),
                                  _ptr(out_hist), ws.data_ptr(), ws.numel(), _stream(stream))
    _raise(rc, "adaptra_eval_best")
    return out_makespan, out_bubble, out_feasible, out_best_idx, out_best_makespan, out_best_bubble, out_hist


def adaptra_seed(prob: Problem, x_max: int = 1, w_current=None, *, want_init: bool = True,
                 want_adapted: bool = True, want_not_absorbed: bool = False, out=None, stream=None):
    """Enqueue the analytic planning; returns (w_init [S] | None, w_adapted [S,K] | None,
    not_absorbed [S-1,K] | None).  out: the three outputs of an earlier call, written again
    instead of allocating new ones."""
    import torch
    dev = prob.device
    if out is not None:
        w_init, w_ad, na = out
    else:
        w_init = torch.empty(prob.S, dtype=torch.int32, device=dev) if want_init else None
        w_ad = torch.empty((prob.S, prob.K), dtype=torch.int32, device=dev) if want_adapted else None
        na = torch.empty((max(prob.S - 1, 0), prob.K), dtype=torch.uint8, device=dev) if want_not_absorbed else None
    _check_i32(w_current, "w_current", (prob.S,))
    rc = load().adaptra_seed(ctypes.byref(prob.params), ctypes.byref(prob.scens), int(x_max), _ptr(w_current),
                             _ptr(w_init), _ptr(w_ad), _ptr(na), _stream(stream))
    _raise(rc, "adaptra_seed")
    return w_init, w_ad, na


def adaptra_sensitivity(prob: Problem, delta: int = 1, *, want_makespan: bool = True, workspace=None, out=None,
                        stream=None):
    """Enqueue the per-link finite differences; returns (makespan [C,K] | None, flag [C,K] | None,
    sens [C,S-1,K]) -- candidate-major, unlike adaptra_eval.  out: the three outputs of an
    earlier call, written again instead of allocating new ones."""
    import torch
    dev = prob.device
    if out is not None:
        mk, fl, sens = out
    else:
        mk = torch.empty((prob.C, prob.K), dtype=torch.int32, device=dev) if want_makespan else None
        fl = torch.empty((prob.C, prob.K), dtype=torch.uint8, device=dev) if want_makespan else None
        sens = torch.empty((prob.C, prob.S - 1, prob.K), dtype=torch.int32, device=dev)
    if workspace is None:
        n = int(load().adaptra_sensitivity_workspace_bytes(ctypes.byref(prob.params), prob.C, prob.K))
        if n == 0:
            raise AdaptraError(EINVAL, "adaptra_sensitivity_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    rc = load().adaptra_sensitivity(ctypes.byref(prob.params), ctypes.byref(prob.cands), ctypes.byref(prob.scens),
                                    int(delta), _ptr(mk), _ptr(fl), _ptr(sens) if prob.S > 1 else None,
                                    workspace.data_ptr(), workspace.numel(), _stream(stream))
    _raise(rc, "adaptra_sensitivity")
    return mk, fl, sens


def adaptra_search(prob: Problem, w_start, neighbourhood: int = 0, max_iters: int = 1000, *, workspace=None,
                   stream=None):
    """Run the guided search (synchronous); prob's candidates are ignored.  Returns
    (w [S,K], makespan [K], rounds, pairs evaluated)."""
    import torch
    dev = prob.device
    _check_i32(w_start, "w_start", (prob.S,))
    w = torch.empty((prob.S, prob.K), dtype=torch.int32, device=dev)
    mk = torch.empty(prob.K, dtype=torch.int32, device=dev)
    if workspace is None:
        n = int(load().adaptra_search_workspace_bytes(ctypes.byref(prob.params), prob.K, int(neighbourhood)))
        if n == 0:
            raise AdaptraError(EINVAL, "adaptra_search_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    rounds, evaluated = ctypes.c_int32(0), ctypes.c_int64(0)
    rc = load().adaptra_search(ctypes.byref(prob.params), ctypes.byref(prob.scens), w_start.data_ptr(),
                               int(neighbourhood), int(max_iters), w.data_ptr(), mk.data_ptr(),
                               ctypes.byref(rounds), ctypes.byref(evaluated),
                               workspace.data_ptr(), workspace.numel(), _stream(stream))
    _raise(rc, "adaptra_search")
    return w, mk, int(rounds.value), int(evaluated.value)


def adaptra_zb_check_inputs(prob: Problem, t_w, workspace=None, stream=None) -> int:
    """Returns the library's code (OK, ERANGE, EOVERFLOW) without raising for data findings."""
    import torch
    _check_i32(t_w, "t_w", (prob.S,))
    if workspace is None:
        n = int(load().adaptra_zb_workspace_bytes(ctypes.byref(prob.params), prob.C, prob.K))
        if n == 0:
            raise AdaptraError(EINVAL, "adaptra_zb_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=prob.device)
    rc = load().adaptra_zb_check_inputs(ctypes.byref(prob.params), t_w.data_ptr(), ctypes.byref(prob.cands),
                                        ctypes.byref(prob.scens), workspace.data_ptr(), workspace.numel(),
                                        _stream(stream))
    if rc in (EINVAL, EWORKSPACE, EHIP):
        _raise(rc, "adaptra_zb_check_inputs")
    return rc


def adaptra_zb_eval(prob: Problem, t_w, plan_scenario: int = -1, *, want_bubble: bool = True,
                    workspace=None, stream=None):
    """Enqueue the ZeroBubble (F / B / W) evaluation; returns (makespan [K,C], bubble [S,K,C] | None)."""
    import torch
    dev = prob.device
    _check_i32(t_w, "t_w", (prob.S,))
    mk = torch.empty((prob.K, prob.C), dtype=torch.int32, device=dev)
    bub = torch.empty((prob.S, prob.K, prob.C), dtype=torch.int32, device=dev) if want_bubble else None
    if workspace is None:
        n = int(load().adaptra_zb_workspace_bytes(ctypes.byref(prob.params), prob.C, prob.K))
        if n == 0:
            raise AdaptraError(EINVAL, "adaptra_zb_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    rc = load().adaptra_zb_eval(ctypes.byref(prob.params), t_w.data_ptr(), ctypes.byref(prob.cands),
                                ctypes.byref(prob.scens), int(plan_scenario), mk.data_ptr(), _ptr(bub),
                                workspace.data_ptr(), workspace.numel(), _stream(stream))
    _raise(rc, "adaptra_zb_eval")
    return mk, bub


def adaptra_set_kernel_mode(mode: int) -> int:
    return int(load().adaptra_set_kernel_mode(int(mode)))


def adaptra_set_resolve_events(before: Optional[int], after: Optional[int]) -> int:
    """before / after: raw hipEvent_t handles (ints) or None."""
    return int(load().adaptra_set_resolve_events(before, after))


def adaptra_valu_probe(mix: int, blocks: int, iters: int, scratch, stream=None) -> int:
    """Enqueue one issue-rate probe (mix: index into PROBE_MIXES); returns the number of vector
    instructions (wavefront instructions) the launch issues."""
    n = ctypes.c_int64(0)
    rc = load().adaptra_valu_probe(int(mix), int(blocks), int(iters), scratch.data_ptr(), _stream(stream),
                                   ctypes.byref(n))
    _raise(rc, "adaptra_valu_probe")
    return int(n.value)


def adaptra_version() -> int:
    return int(load().adaptra_version())
