"""Thin ctypes binding of libddef.so: same names as include/ddef.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels; nothing here computes.  There is no
fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

from . import build as _build

OK, EINVAL, ESTATE, ENOMEM, EHIP, ENONFINITE, EINTERNAL = 0, -1, -2, -3, -4, -5, -6
COMPRESSOR_TOPK, COMPRESSOR_RANDK, COMPRESSOR_COMPOSED = 0, 1, 2
NOISE_NONE, NOISE_GAUSS, NOISE_STUDENT_T3 = 0, 1, 2
OPT_FORCE_FULL_SELECT, OPT_CANDIDATE_SLACK_X16, OPT_PREFETCH_GRAD, OPT_FUSE_GRAD, OPT_GRAPH = 1, 2, 3, 4, 5
OPT_RANDK_BUCKET_PERCENT = 6
OPT_COMPOSED_BOUND = 7
OPT_DENSE_SPLIT = 8

_u32p, _f32p, _u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_float), C.POINTER(C.c_uint64)
_ctx = C.c_void_p

SIGNATURES = {
    "ddef_init": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.POINTER(_ctx)]),
    "ddef_init_queue": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.POINTER(_ctx)]),
    "ddef_destroy": (C.c_int, [_ctx]),
    "ddef_set_stream": (C.c_int, [_ctx, C.c_void_p]),
    "ddef_set_problem": (C.c_int, [_ctx, _f32p, _f32p, _f32p, C.c_uint64, C.c_int, C.c_float]),
    "ddef_set_tau": (C.c_int, [_ctx, C.c_uint32]),
    "ddef_set_compressor": (C.c_int, [_ctx, C.c_int]),
    "ddef_set_composed": (C.c_int, [_ctx, C.c_double]),
    "ddef_objective": (C.c_int, [_ctx, C.POINTER(C.c_double)]),
    "ddef_get_message_codes": (C.c_int, [_ctx, C.c_uint32, C.POINTER(C.c_uint8), _f32p, _u64p]),
    "ddef_set_heterogeneity": (C.c_int, [_ctx, C.c_float]),
    "ddef_deco_noniid": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_double, _u32p, C.POINTER(C.c_double)]),
    "ddef_phi_prime": (C.c_double, [C.c_double, C.c_double]),
    "ddef_corner_compression_only": (C.c_int, [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]),
    "ddef_corner_delay_only": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint32, _u32p]),
    "ddef_grad": (C.c_int, [_ctx]),
    "ddef_load_grad": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_ef_compress": (C.c_int, [_ctx, C.c_double, C.c_float]),
    "ddef_aggregate": (C.c_int, [_ctx]),
    "ddef_step": (C.c_int, [_ctx, C.c_double, C.c_float]),
    "ddef_get_snapshot": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_set_snapshot": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_set_step_index": (C.c_int, [_ctx, C.c_uint64]),
    "ddef_device_info": (C.c_int, [_ctx, _u32p, _u32p, _u64p, _u64p, _u32p, _u32p, _u32p, C.c_char_p, C.c_uint32]),
    "ddef_graph_replays": (C.c_int, [_ctx, _u64p]),
    "ddef_apply_delayed": (C.c_int, [_ctx, C.c_float]),
    "ddef_sync": (C.c_int, [_ctx]),
    "ddef_step_index": (C.c_int, [_ctx, _u64p]),
    "ddef_get_model": (C.c_int, [_ctx, _f32p]),
    "ddef_set_model": (C.c_int, [_ctx, _f32p]),
    "ddef_get_error": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_set_error": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_get_grad": (C.c_int, [_ctx, C.c_uint32, _f32p]),
    "ddef_get_update": (C.c_int, [_ctx, _f32p]),
    "ddef_get_message": (C.c_int, [_ctx, C.c_uint32, _u32p, _f32p, _u64p]),
    "ddef_get_threshold": (C.c_int, [_ctx, C.c_uint32, _u32p, _u64p]),
    "ddef_k_from_delta": (C.c_uint64, [C.c_double, C.c_uint64]),
    "ddef_deco": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_double, _u32p, C.POINTER(C.c_double)]),
    "ddef_phi": (C.c_double, [C.c_double, C.c_double]),
    "ddef_t_avg_model": (C.c_double, [C.c_uint32, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double]),
    "ddef_t_avg_simulate": (C.c_double, [C.c_uint32, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double,
                                         C.c_uint64]),
    "ddef_lut_build": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_uint32, C.c_double, C.c_double,
                                 C.POINTER(C.c_void_p)]),
    "ddef_lut_query": (C.c_int, [C.c_void_p, C.c_double, _u32p, C.POINTER(C.c_double), C.POINTER(C.c_int)]),
    "ddef_lut_destroy": (C.c_int, [C.c_void_p]),
    "ddef_profile_enable": (C.c_int, [_ctx, C.c_int]),
    "ddef_profile_slots": (C.c_int, []),
    "ddef_profile_read": (C.c_int, [_ctx, C.c_int, C.POINTER(C.c_char_p), _u64p, C.POINTER(C.c_double)]),
    "ddef_copy_probe": (C.c_int, [_ctx, _u64p]),
    "ddef_full_select_count":  (C.c_int, [_ctx, _u64p]),
    "ddef_set_option": (C.c_int, [_ctx, C.c_int, C.c_int64]),
    "ddef_get_filter_state": (C.c_int, [_ctx, C.c_uint32, _u32p, _u32p, _u32p]),
    "ddef_ef_compress_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32, C.c_double,
                                          C.c_float, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "ddef_strerror": (C.c_char_p, [C.c_int]),
}

_lib = None


class DdefError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


def library_path() -> str:
    return _build.LIB


def load():
    """Load libddef.so (building it first only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library()
    lib = C.CDLL(_build.LIB)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the library lacks a declared symbol
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().ddef_strerror(int(code)).decode()


def k_from_delta(delta: float, d: int) -> int:
    return int(load().ddef_k_from_delta(float(delta), int(d)))


def deco(v_g_bits: float, a_bps: float, b_s: float, t_comp_s: float) -> Optional[Tuple[int, float]]:
    tau, delta = C.c_uint32(), C.c_double()
    rc = load().ddef_deco(float(v_g_bits), float(a_bps), float(b_s), float(t_comp_s),
                          C.byref(tau), C.byref(delta))
    if rc == EINVAL:
        return None
    if rc != OK:
        raise DdefError(rc, "ddef_deco")
    return int(tau.value), float(delta.value)


def deco_noniid(v_g_bits: float, a_bps: float, b_s: float, t_comp_s: float) -> Optional[Tuple[int, float]]:
    tau, delta = C.c_uint32(), C.c_double()
    rc = load().ddef_deco_noniid(float(v_g_bits), float(a_bps), float(b_s), float(t_comp_s),
                                 C.byref(tau), C.byref(delta))
    if rc == EINVAL:
        return None
    if rc != OK:
        raise DdefError(rc, "ddef_deco_noniid")
    return int(tau.value), float(delta.value)


def ef_compress_static(dev_e: int, dev_g: int, ld: int, d: int, n: int, delta: float, lr: float,
                       dev_msg_idx: int, dev_msg_val: int, msg_ld: int, hip_stream: int = 0) -> int:
    """ddef_ef_compress_static on device addresses given as integers; returns the library's code."""
    return int(load().ddef_ef_compress_static(C.c_void_p(int(dev_e)), C.c_void_p(int(dev_g)), int(ld), int(d), int(n),
                                              float(delta), float(lr), C.c_void_p(int(dev_msg_idx)),
                                              C.c_void_p(int(dev_msg_val)), int(msg_ld),
                                              C.c_void_p(int(hip_stream)) if hip_stream else None))


def corner_compression_only(v_g_bits: float, a_bps: float, t_comp_s: float) -> float:
    delta = C.c_double()
    rc = load().ddef_corner_compression_only(float(v_g_bits), float(a_bps), float(t_comp_s), C.byref(delta))
    if rc != OK:
        raise DdefError(rc, "ddef_corner_compression_only")
    return float(delta.value)


def corner_delay_only(v_g_bits: float, a_bps: float, b_s: float, t_comp_s: float, tau_max: int) -> int:
    tau = C.c_uint32()
    rc = load().ddef_corner_delay_only(float(v_g_bits), float(a_bps), float(b_s), float(t_comp_s), int(tau_max),
                                       C.byref(tau))
    if rc != OK:
        raise DdefError(rc, "ddef_corner_delay_only")
    return int(tau.value)


def phi_prime(delta: float, tau: float) -> float:
    return float(load().ddef_phi_prime(float(delta), float(tau)))


def phi(delta: float, tau: float) -> float:
    return float(load().ddef_phi(float(delta), float(tau)))


def t_avg_model(tau: int, delta: float, v_g_bits: float, a_bps: float, b_s: float, t_comp_s: float) -> float:
    return float(load().ddef_t_avg_model(int(tau), float(delta), float(v_g_bits), float(a_bps), float(b_s),
                                         float(t_comp_s)))


def t_avg_simulate(tau: int, delta: float, v_g_bits: float, a_bps: float, b_s: float, t_comp_s: float,
                   iterations: int) -> float:
    return float(load().ddef_t_avg_simulate(int(tau), float(delta), float(v_g_bits), float(a_bps), float(b_s),
                                            float(t_comp_s), int(iterations)))


class DecoLut:
    """Look-up table of Section 4.5 (ddef_lut_*)."""

    def __init__(self, v_g_bits, a_min_bps, a_max_bps, points, b_s, t_comp_s):
        self._lib = load()
        h = C.c_void_p()
        rc = self._lib.ddef_lut_build(float(v_g_bits), float(a_min_bps), float(a_max_bps), int(points),
                                      float(b_s), float(t_comp_s), C.byref(h))
        if rc != OK:
            raise DdefError(rc, "ddef_lut_build")
        self._h = h

    def query(self, a_bps: float):
        """(tau, delta, from_table) or None when DeCo has no candidate."""
        tau, delta, hit = C.c_uint32(), C.c_double(), C.c_int()
        rc = self._lib.ddef_lut_query(self._h, float(a_bps), C.byref(tau), C.byref(delta), C.byref(hit))
        if rc == EINVAL:
            return None
        if rc != OK:
            raise DdefError(rc, "ddef_lut_query")
        return int(tau.value), float(delta.value), bool(hit.value)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ddef_lut_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _f32(a) -> Tuple[np.ndarray, "C._Pointer"]:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


class Context:
    """One ddef_ctx.  Methods carry the C names without the prefix and raise on error codes;
    `raw_*` variants return the code instead (for error-path tests)."""

    def __init__(self, d: int, n: int, tau_max: int, queue_form: bool = False):
        self._lib = load()
        self.d, self.n, self.tau_max = int(d), int(n), int(tau_max)
        self.queue_form = bool(queue_form)
        h = _ctx()
        init = self._lib.ddef_init_queue if self.queue_form else self._lib.ddef_init
        rc = init(self.d, self.n, self.tau_max, C.byref(h))
        if rc != OK:
            raise DdefError(rc, "ddef_init_queue" if self.queue_form else "ddef_init")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ddef_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, rc: int, what: str):
        if rc != OK:
            raise DdefError(rc, what)

    # ---- set-up -------------------------------------------------------------------------
    def set_stream(self, hip_stream: Optional[int]):
        self._check(self._lib.ddef_set_stream(self._h, C.c_void_p(hip_stream or 0)), "ddef_set_stream")

    def set_problem(self, lam, xstar, x0, seed: int, noise_kind: int, noise_scale: float):
        lam, lp = _f32(lam)
        xstar, sp = _f32(xstar)
        x0, xp = _f32(x0)
        for a in (lam, xstar, x0):
            if a.shape != (self.d,):
                raise ValueError("problem vectors must have length d")
        self._check(self._lib.ddef_set_problem(self._h, lp, sp, xp, int(seed), int(noise_kind),
                                               float(noise_scale)), "ddef_set_problem")

    def set_tau(self, tau: int):
        self._check(self._lib.ddef_set_tau(self._h, int(tau)), "ddef_set_tau")

    def set_heterogeneity(self, zeta: float):
        self._check(self._lib.ddef_set_heterogeneity(self._h, float(zeta)), "ddef_set_heterogeneity")

    def set_compressor(self, kind: int):
        self._check(self._lib.ddef_set_compressor(self._h, int(kind)), "ddef_set_compressor")

    def set_composed(self, rand_ratio: float):
        self._check(self._lib.ddef_set_composed(self._h, float(rand_ratio)), "ddef_set_composed")

    def set_option(self, option: int, value: int):
        self._check(self._lib.ddef_set_option(self._h, int(option), int(value)), "ddef_set_option")

    # ---- the step -----------------------------------------------------------------------
    def grad(self):
        self._check(self._lib.ddef_grad(self._h), "ddef_grad")

    def load_grad(self, worker: int, g):
        g, gp = _f32(g)
        if g.shape != (self.d,):
            raise ValueError("gradient must have length d")
        self._check(self._lib.ddef_load_grad(self._h, int(worker), gp), "ddef_load_grad")

    def ef_compress(self, delta: float, lr: float):
        self._check(self._lib.ddef_ef_compress(self._h, float(delta), float(lr)), "ddef_ef_compress")

    def aggregate(self):
        self._check(self._lib.ddef_aggregate(self._h), "ddef_aggregate")

    def apply_delayed(self, lr: float):
        self._check(self._lib.ddef_apply_delayed(self._h, float(lr)), "ddef_apply_delayed")

    def step(self, delta: float, lr: float):
        self._check(self._lib.ddef_step(self._h, float(delta), float(lr)), "ddef_step")

    def device_info(self) -> dict:
        cu, wave, clk, mclk, bus = (C.c_uint32() for _ in range(5))
        lds, mem = C.c_uint64(), C.c_uint64()
        name = C.create_string_buffer(64)
        self._check(self._lib.ddef_device_info(self._h, C.byref(cu), C.byref(wave), C.byref(lds), C.byref(mem),
                                               C.byref(clk), C.byref(mclk), C.byref(bus), name, 64), "ddef_device_info")
        return {"arch": name.value.decode(), "compute_units": cu.value, "wave_size": wave.value,
                "lds_bytes_per_cu": lds.value, "memory_bytes": mem.value, "clock_khz": clk.value,
                "memory_clock_khz": mclk.value, "memory_bus_bits": bus.value}

    def get_snapshot(self, age: int) -> np.ndarray:
        return self._get(self._lib.ddef_get_snapshot, "ddef_get_snapshot", int(age))

    def set_snapshot(self, age: int, x) -> None:
        a = np.ascontiguousarray(x, dtype=np.float32)
        if a.shape != (self.d,):
            raise ValueError("snapshot must have d entries")
        self._check(self._lib.ddef_set_snapshot(self._h, int(age), a.ctypes.data_as(_f32p)), "ddef_set_snapshot")

    def set_step_index(self, t: int) -> None:
        self._check(self._lib.ddef_set_step_index(self._h, int(t)), "ddef_set_step_index")

    def graph_replays(self) -> int:
        n = C.c_uint64()
        self._check(self._lib.ddef_graph_replays(self._h, C.byref(n)), "ddef_graph_replays")
        return int(n.value)

    def sync(self):
        self._check(self._lib.ddef_sync(self._h), "ddef_sync")

    # raw return codes, for error-path tests
    def raw(self, name: str, *args) -> int:
        return int(getattr(self._lib, "ddef_" + name)(self._h, *args))

    # ---- inspection ---------------------------------------------------------------------
    @property
    def t(self) -> int:
        t = C.c_uint64()
        self._check(self._lib.ddef_step_index(self._h, C.byref(t)), "ddef_step_index")
        return int(t.value)

    def _get(self, fn, what, *args) -> np.ndarray:
        out = np.empty(self.d, dtype=np.float32)
        self._check(fn(self._h, *args, out.ctypes.data_as(_f32p)), what)
        return out

    def get_model(self):
        return self._get(self._lib.ddef_get_model, "ddef_get_model")

    def set_model(self, x):
        x, xp = _f32(x)
        self._check(self._lib.ddef_set_model(self._h, xp), "ddef_set_model")

    def get_error(self, worker: int):
        return self._get(self._lib.ddef_get_error, "ddef_get_error", int(worker))

    def set_error(self, worker: int, e):
        e, ep = _f32(e)
        self._check(self._lib.ddef_set_error(self._h, int(worker), ep), "ddef_set_error")

    def get_grad(self, worker: int):
        return self._get(self._lib.ddef_get_grad, "ddef_get_grad", int(worker))

    def get_update(self):
        return self._get(self._lib.ddef_get_update, "ddef_get_update")

    def get_message(self, worker: int):
        k = C.c_uint64()
        self._check(self._lib.ddef_get_message(self._h, int(worker), None, None, C.byref(k)), "ddef_get_message")
        idx = np.empty(k.value, dtype=np.uint32)
        val = np.empty(k.value, dtype=np.float32)
        if k.value:
            self._check(self._lib.ddef_get_message(self._h, int(worker), idx.ctypes.data_as(_u32p),
                                                   val.ctypes.data_as(_f32p), C.byref(k)), "ddef_get_message")
        return idx, val

    def objective(self) -> float:
        """f(x_t) = (1/n) sum_i f_i(x_t) of the synthetic quadratics at the current iterate."""
        f = C.c_double()
        self._check(self._lib.ddef_objective(self._h, C.byref(f)), "ddef_objective")
        return float(f.value)

    def get_message_codes(self, worker: int):
        """(packed 4-bit codes, block steps) of the last message under the composed compressor."""
        k = C.c_uint64()
        self._check(self._lib.ddef_get_message_codes(self._h, int(worker), None, None, C.byref(k)),
                    "ddef_get_message_codes")
        codes = np.zeros((k.value + 1) // 2, dtype=np.uint8)
        steps = np.zeros((k.value + 255) // 256, dtype=np.float32)
        if k.value:
            self._check(self._lib.ddef_get_message_codes(self._h, int(worker),
                                                         codes.ctypes.data_as(C.POINTER(C.c_uint8)),
                                                         steps.ctypes.data_as(_f32p), C.byref(k)),
                        "ddef_get_message_codes")
        return codes, steps

    def get_threshold(self, worker: int):
        T, r = C.c_uint32(), C.c_uint64()
        self._check(self._lib.ddef_get_threshold(self._h, int(worker), C.byref(T), C.byref(r)), "ddef_get_threshold")
        return int(T.value), int(r.value)

    def get_filter_state(self, worker: int):
        """(next bound pattern, candidates caught, searched whole row) of the last selection."""
        b, m, a = C.c_uint32(), C.c_uint32(), C.c_uint32()
        self._check(self._lib.ddef_get_filter_state(self._h, int(worker), C.byref(b), C.byref(m), C.byref(a)),
                    "ddef_get_filter_state")
        return int(b.value), int(m.value), bool(a.value)

    def full_select_count(self) -> int:
        cnt = C.c_uint64()
        self._check(self._lib.ddef_full_select_count(self._h, C.byref(cnt)), "ddef_full_select_count")
        return int(cnt.value)

    # ---- measurement --------------------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(self._lib.ddef_profile_enable(self._h, 1 if on else 0), "ddef_profile_enable")

    def copy_probe(self) -> int:
        """Launch the plain copy yardstick once; returns the bytes it reads (= writes)."""
        b = C.c_uint64()
        self._check(self._lib.ddef_copy_probe(self._h, C.byref(b)), "ddef_copy_probe")
        return int(b.value)

    def profile_read(self):
        """{kernel name: (launches, total_ms)} since profiling was switched on."""
        out = {}
        for s in range(self._lib.ddef_profile_slots()):
            name, cnt, ms = C.c_char_p(), C.c_uint64(), C.c_double()
            self._check(self._lib.ddef_profile_read(self._h, s, C.byref(name), C.byref(cnt), C.byref(ms)),
                        "ddef_profile_read")
            out[name.value.decode()] = (int(cnt.value), float(ms.value))
        return out
