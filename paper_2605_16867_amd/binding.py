"""ctypes binding of libgoodroute: same names as the C interface, argument
marshalling only.  Tensors are torch tensors on the GPU (device memory and the
current stream come from torch; every step of the path runs in the library's
kernels).  There is no fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libgoodroute.so")

EXPORTS = ("gr_create", "gr_destroy", "gr_build_status", "gr_score_route", "gr_score_route_noalloc", "gr_score_route_cached", "gr_route_feedback",
           "gr_risk_scan", "gr_observe", "gr_set_blend", "gr_set_batch_cap", "gr_set_small_batch_pairs",
           "gr_device_status", "gr_strerror", "gr_profile_enable", "gr_profile_select", "gr_profile_read",
           "gr_profile_read_launches", "gr_profile_kernel_count", "gr_profile_kernel_name")

_lib = None


class GoodRouteError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib() -> C.CDLL:
    """Load libgoodroute.so (built by paper_2605_16867_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2605_16867_amd.build`")
        l = C.CDLL(LIB_PATH)
        p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.gr_create.restype = C.c_int
        l.gr_create.argtypes = [C.POINTER(p), i32, i32, p, p, p, p, p, i32, i32, i64]
        l.gr_destroy.restype = C.c_int
        l.gr_destroy.argtypes = [p]
        l.gr_build_status.restype = C.c_int
        l.gr_build_status.argtypes = [p, p, p, p, p, i64, p, p, p, i64, p, p, p, p, p]
        l.gr_score_route.restype = C.c_int
        l.gr_score_route.argtypes = [p, i64, p, p, p, p, p, p, p, p, p]
        l.gr_score_route_noalloc.restype = C.c_int
        l.gr_score_route_noalloc.argtypes = [p, i64, p, p, p, p, p, p, p, p]
        l.gr_score_route_cached.restype = C.c_int
        l.gr_score_route_cached.argtypes = [p, i64, p, p, p, p, p, p, p, i64, p, p, p, p, p]
        l.gr_route_feedback.restype = C.c_int
        l.gr_route_feedback.argtypes = [p, i64, i64, p, p, p, p, p, p, p, p]
        l.gr_risk_scan.restype = C.c_int
        l.gr_risk_scan.argtypes = [p, p, p, p, p, i64, p, p, p, i64, p, p, p, p, p, p, p]
        l.gr_observe.restype = C.c_int
        l.gr_observe.argtypes = [p, C.c_double, p, p, p, p]
        l.gr_set_blend.restype = C.c_int
        l.gr_set_blend.argtypes = [p, C.c_double]
        l.gr_set_small_batch_pairs.restype = C.c_int
        l.gr_set_small_batch_pairs.argtypes = [p, C.c_int64]
        l.gr_set_batch_cap.restype = C.c_int
        l.gr_set_batch_cap.argtypes = [p, p]
        l.gr_device_status.restype = C.c_int
        l.gr_device_status.argtypes = [p, C.POINTER(i32)]
        l.gr_profile_enable.restype = C.c_int
        l.gr_profile_enable.argtypes = [p, i32]
        l.gr_profile_select.restype = C.c_int
        l.gr_profile_select.argtypes = [p, C.c_uint64]
        l.gr_profile_read.restype = C.c_int
        l.gr_profile_read.argtypes = [p, i32, p, p]
        l.gr_profile_read_launches.restype = C.c_int
        l.gr_profile_read_launches.argtypes = [p, i32, p, p, p]
        l.gr_profile_kernel_count.restype = i32
        l.gr_profile_kernel_count.argtypes = []
        l.gr_profile_kernel_name.restype = C.c_char_p
        l.gr_profile_kernel_name.argtypes = [i32]
        l.gr_strerror.restype = C.c_char_p
        l.gr_strerror.argtypes = [C.c_int]
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().gr_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise GoodRouteError(code, where)


def _dev(t, dtype, name: str, n: Optional[int] = None):
    """Device pointer of a contiguous GPU tensor of the given dtype (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} GPU tensor, got {t.dtype} on {t.device}")
    if n is not None and t.numel() < n:
        raise ValueError(f"{name}: {t.numel()} elements, need {n}")
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Fleet:
    """Owns a gr_fleet handle on the current device."""

    def __init__(self, delta, alpha, beta, gamma, inst_class, max_entries_per_inst: int,
                 max_len: int, max_requests: int):
        import numpy as np
        self._h = C.c_void_p()
        co = [np.ascontiguousarray(x, dtype=np.float64) for x in (delta, alpha, beta, gamma)]
        ic = np.ascontiguousarray(inst_class, dtype=np.int32)
        self.n_inst = int(ic.shape[0])
        _check(lib().gr_create(C.byref(self._h), self.n_inst, int(co[0].shape[0]),
                               *[c.ctypes.data_as(C.c_void_p) for c in co],
                               ic.ctypes.data_as(C.c_void_p), int(max_entries_per_inst),
                               int(max_len), int(max_requests)), "gr_create")

    def close(self) -> None:
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib().gr_destroy(h), "gr_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def gr_build_status(self, act_off, act_prompt, act_gen, act_rem, q_off, q_prompt, q_len,
                        out_act_finish, out_q_finish=None, out_d=None, out_rank=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        na, nq, M = act_prompt.numel(), q_prompt.numel(), self.n_inst
        _check(lib().gr_build_status(
            self._h, _dev(act_off, i32, "act_off", M + 1), _dev(act_prompt, i32, "act_prompt"),
            _dev(act_gen, i32, "act_gen", na), _dev(act_rem, i32, "act_rem", na), na,
            _dev(q_off, i32, "q_off", M + 1), _dev(q_prompt, i32, "q_prompt"),
            _dev(q_len, i32, "q_len", nq), nq,
            _dev(out_act_finish, f32, "out_act_finish", na), _dev(out_q_finish, f32, "out_q_finish", nq),
            _dev(out_d, torch.float64, "out_d", M), _dev(out_rank, i32, "out_rank", M),
            _stream()), "gr_build_status")

    def gr_score_route(self, ctx0, pred_len, budget, out_inst, out_slack, exclude_inst=None,
                       out_fallback=None, out_T=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        n = ctx0.numel()
        _check(lib().gr_score_route(
            self._h, n, _dev(ctx0, i32, "ctx0"), _dev(pred_len, i32, "pred_len", n),
            _dev(budget, f32, "budget", n), _dev(exclude_inst, i32, "exclude_inst", n),
            _dev(out_inst, i32, "out_inst", n), _dev(out_slack, f32, "out_slack", n),
            _dev(out_fallback, torch.uint8, "out_fallback", n),
            _dev(out_T, f32, "out_T", n * self.n_inst), _stream()), "gr_score_route")

    def gr_score_route_noalloc(self, ctx0, pred_len, budget, out_inst, out_slack, exclude_inst=None,
                               out_fallback=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        n = ctx0.numel()
        _check(lib().gr_score_route_noalloc(
            self._h, n, _dev(ctx0, i32, "ctx0"), _dev(pred_len, i32, "pred_len", n),
            _dev(budget, f32, "budget", n), _dev(exclude_inst, i32, "exclude_inst", n),
            _dev(out_inst, i32, "out_inst", n), _dev(out_slack, f32, "out_slack", n),
            _dev(out_fallback, torch.uint8, "out_fallback", n), _stream()), "gr_score_route_noalloc")

    def gr_score_route_cached(self, ctx0, pred_len, budget, hit_off, hit_inst, hit_len, out_inst, out_slack,
                              exclude_inst=None, out_fallback=None, out_T=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        n, nh = ctx0.numel(), hit_inst.numel()
        _check(lib().gr_score_route_cached(
            self._h, n, _dev(ctx0, i32, "ctx0"), _dev(pred_len, i32, "pred_len", n),
            _dev(budget, f32, "budget", n), _dev(exclude_inst, i32, "exclude_inst", n),
            _dev(hit_off, i32, "hit_off", n + 1), _dev(hit_inst, i32, "hit_inst"),
            _dev(hit_len, i32, "hit_len", nh), nh,
            _dev(out_inst, i32, "out_inst", n), _dev(out_slack, f32, "out_slack", n),
            _dev(out_fallback, torch.uint8, "out_fallback", n),
            _dev(out_T, f32, "out_T", n * self.n_inst), _stream()), "gr_score_route_cached")

    def gr_route_feedback(self, chunk: int, ctx0, pred_len, budget, out_inst, out_slack, exclude_inst=None,
                          out_fallback=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        n = ctx0.numel()
        _check(lib().gr_route_feedback(
            self._h, n, int(chunk), _dev(ctx0, i32, "ctx0"), _dev(pred_len, i32, "pred_len", n),
            _dev(budget, f32, "budget", n), _dev(exclude_inst, i32, "exclude_inst", n),
            _dev(out_inst, i32, "out_inst", n), _dev(out_slack, f32, "out_slack", n),
            _dev(out_fallback, torch.uint8, "out_fallback", n), _stream()), "gr_route_feedback")

    def gr_risk_scan(self, act_off, act_prompt, act_gen, act_rem_refreshed, q_off, q_prompt, q_len,
                     act_budget, out_flag, out_finish, out_target, out_target_slack,
                     out_n_flagged=None) -> None:
        import torch
        i32, f32 = torch.int32, torch.float32
        na, nq, M = act_prompt.numel(), q_prompt.numel(), self.n_inst
        _check(lib().gr_risk_scan(
            self._h, _dev(act_off, i32, "act_off", M + 1), _dev(act_prompt, i32, "act_prompt"),
            _dev(act_gen, i32, "act_gen", na), _dev(act_rem_refreshed, i32, "act_rem_refreshed", na), na,
            _dev(q_off, i32, "q_off", M + 1), _dev(q_prompt, i32, "q_prompt"),
            _dev(q_len, i32, "q_len", nq), nq,
            _dev(act_budget, f32, "act_budget", na), _dev(out_flag, torch.uint8, "out_flag", na),
            _dev(out_finish, f32, "out_finish", na), _dev(out_target, i32, "out_target", na),
            _dev(out_target_slack, f32, "out_target_slack", na),
            _dev(out_n_flagged, i32, "out_n_flagged", 1), _stream()), "gr_risk_scan")

    def gr_observe(self, weight: float, obs_wait=None, obs_prefill=None, obs_decode=None) -> None:
        import torch
        f32, M = torch.float32, self.n_inst
        _check(lib().gr_observe(self._h, float(weight), _dev(obs_wait, f32, "obs_wait", M),
                                _dev(obs_prefill, f32, "obs_prefill", M),
                                _dev(obs_decode, f32, "obs_decode", M), _stream()), "gr_observe")

    def gr_set_blend(self, black_box_weight: float) -> None:
        _check(lib().gr_set_blend(self._h, float(black_box_weight)), "gr_set_blend")

    def gr_set_small_batch_pairs(self, max_pairs: int) -> None:
        _check(lib().gr_set_small_batch_pairs(self._h, int(max_pairs)), "gr_set_small_batch_pairs")

    def gr_set_batch_cap(self, cap) -> None:
        """cap: host int array of n_inst entries, or None to remove the caps."""
        import numpy as np
        if cap is None:
            _check(lib().gr_set_batch_cap(self._h, None), "gr_set_batch_cap")
            return
        c = np.ascontiguousarray(cap, dtype=np.int32)
        if c.shape != (self.n_inst,):
            raise ValueError(f"cap: need {self.n_inst} entries")
        _check(lib().gr_set_batch_cap(self._h, c.ctypes.data_as(C.c_void_p)), "gr_set_batch_cap")

    def gr_profile_enable(self, max_launches: int) -> None:
        _check(lib().gr_profile_enable(self._h, int(max_launches)), "gr_profile_enable")

    def gr_profile_select(self, names=None) -> None:
        """Time only the kernels whose name starts with one of `names` (None: all)."""
        n = int(lib().gr_profile_kernel_count())
        mask = 0
        for k in range(n):
            nm = lib().gr_profile_kernel_name(k).decode()
            if names is None or any(nm.startswith(x) for x in names):
                mask |= 1 << k
        _check(lib().gr_profile_select(self._h, mask), "gr_profile_select")

    def gr_profile_read(self) -> dict:
        """{kernel name: (total milliseconds, launches)} since the last read."""
        n = int(lib().gr_profile_kernel_count())
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        _check(lib().gr_profile_read(self._h, n, ms, cnt), "gr_profile_read")
        return {lib().gr_profile_kernel_name(k).decode(): (float(ms[k]), int(cnt[k])) for k in range(n)}

    def gr_profile_read_launches(self, max_launches: int) -> dict:
        """{kernel name: [milliseconds of each recorded launch, in launch order]} since the last read."""
        ids = (C.c_int32 * max(max_launches, 1))()
        ms = (C.c_float * max(max_launches, 1))()
        n = C.c_int32(0)
        _check(lib().gr_profile_read_launches(self._h, int(max_launches), ids, ms, C.byref(n)), "gr_profile_read_launches")
        out = {}
        for i in range(int(n.value)):
            out.setdefault(lib().gr_profile_kernel_name(ids[i]).decode(), []).append(float(ms[i]))
        return out

    def gr_device_status(self) -> int:
        bits = C.c_int32(0)
        _check(lib().gr_device_status(self._h, C.byref(bits)), "gr_device_status")
        return int(bits.value)
