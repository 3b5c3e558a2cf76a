"""ctypes front end of the CPU oracle (test infrastructure, not part of the product).

Only tests/, the smoke check and the benchmark's cpu_baseline leg import this package.  It
never imports the GPU binding.  `build()` compiles oracle/ddef_oracle.cpp with g++ into
oracle/libddef_oracle.so; the functions below only marshal numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ddef_oracle.cpp")
_LIB = os.path.join(_HERE, "libddef_oracle.so")

# -ffp-contract=off: every fp32 operation rounds on its own (no fused multiply-add).
CXXFLAGS = ["-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
            "-pthread"]


def build(force: bool = True) -> str:
    if _prebuilt:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", *CXXFLAGS, _SRC, "-o", _LIB])
    return _LIB


_lib = None
_prebuilt = False


def use_library(path: str) -> None:
    """Load this build of the oracle instead of oracle/libddef_oracle.so (before first use).
    For the test that compiles copies of the source with mistakes planted in them and checks
    that the pins notice."""
    global _LIB, _prebuilt
    if _lib is not None:
        raise RuntimeError("the oracle library is already loaded")
    _LIB, _prebuilt = path, True


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not _prebuilt:
        build(force=False)
    L = C.CDLL(_LIB)
    u32p, f32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_float), C.POINTER(C.c_uint64)
    vp = C.c_void_p
    sig = {
        "oracle_philox4x32_10": (None, [u32p, u32p, u32p]),
        "oracle_neg2ln_uniform": (C.c_float, [C.c_uint32]),
        "oracle_unit_circle_point": (None, [C.c_uint32, f32p, f32p]),
        "oracle_noise_z": (C.c_float, [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int]),
        "oracle_noise_fill": (None, [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64,
                                     C.c_int, f32p]),
        "oracle_k_from_delta": (C.c_uint64, [C.c_double, C.c_uint64]),
        "oracle_topk": (None, [f32p, C.c_uint64, C.c_uint64, u32p, u32p, u64p]),
        "oracle_create": (vp, [C.c_uint64, C.c_uint32, C.c_uint32]),
        "oracle_destroy": (None, [vp]),
        "oracle_set_threads": (None, [vp, C.c_int]),
        "oracle_set_problem": (None, [vp, f32p, f32p, f32p, C.c_uint64, C.c_int, C.c_float]),
        "oracle_set_tau": (None, [vp, C.c_uint32]),
        "oracle_step_index": (C.c_uint64, [vp]),
        "oracle_grad": (None, [vp]),
        "oracle_load_grad": (None, [vp, C.c_uint32, f32p]),
        "oracle_ef_compress": (None, [vp, C.c_double, C.c_float]),
        "oracle_aggregate": (None, [vp]),
        "oracle_apply_delayed": (None, [vp]),
        "oracle_step": (None, [vp, C.c_double, C.c_float]),
        "oracle_get_model": (None, [vp, f32p]),
        "oracle_set_model": (None, [vp, f32p]),
        "oracle_get_snapshot": (None, [vp, C.c_uint64, f32p]),
        "oracle_get_error": (None, [vp, C.c_uint32, f32p]),
        "oracle_set_error": (None, [vp, C.c_uint32, f32p]),
        "oracle_get_grad": (None, [vp, C.c_uint32, f32p]),
        "oracle_message_size": (C.c_uint64, [vp, C.c_uint32]),
        "oracle_get_message": (None, [vp, C.c_uint32, u32p, f32p]),
        "oracle_get_update": (None, [vp, f32p]),
        "oracle_get_threshold": (None, [vp, C.c_uint32, u32p, u64p]),
        "oracle_queue_run": (None, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_double,
                                    C.c_float, f32p, f32p, f32p, C.c_uint64, C.c_int, C.c_float,
                                    f32p, f32p]),
        "oracle_randk_indices": (None, [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64, u32p]),
        "oracle_randk_permute": (C.c_uint64, [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64]),
        "oracle_murmur_fmix32": (C.c_uint32, [C.c_uint32]),
        "oracle_set_compressor": (None, [vp, C.c_int]),
        "oracle_set_composed": (None, [vp, C.c_double]),
        "oracle_objective": (C.c_double, [vp]),
        "oracle_quantize4": (None, [f32p, C.c_uint64, C.POINTER(C.c_uint8), f32p, f32p]),
        "oracle_get_message_codes": (None, [vp, C.c_uint32, C.POINTER(C.c_uint8), f32p]),
        "oracle_set_heterogeneity": (None, [vp, C.c_float]),
        "oracle_phi_prime": (C.c_double, [C.c_double, C.c_double]),
        "oracle_deco_noniid": (C.c_int, [C.c_double] * 4 + [u32p, C.POINTER(C.c_double)]),
        "oracle_queue_create": (vp, [C.c_uint64, C.c_uint32, C.c_uint32]),
        "oracle_queue_destroy": (None, [vp]),
        "oracle_queue_set_tau": (None, [vp, C.c_uint32]),
        "oracle_queue_set_heterogeneity": (None, [vp, C.c_float]),
        "oracle_queue_set_problem": (None, [vp, f32p, f32p, f32p, C.c_uint64, C.c_int, C.c_float]),
        "oracle_queue_step": (None, [vp, C.c_double, C.c_float]),
        "oracle_queue_get_model": (None, [vp, f32p]),
        "oracle_queue_get_update": (None, [vp, f32p]),
        "oracle_queue_get_error": (None, [vp, C.c_uint32, f32p]),
        "oracle_queue_message_size": (C.c_uint64, [vp, C.c_uint32]),
        "oracle_queue_get_message": (None, [vp, C.c_uint32, u32p, f32p]),
        "oracle_phi": (C.c_double, [C.c_double, C.c_double]),
        "oracle_delta_star": (C.c_double, [C.c_double] * 5),
        "oracle_deco": (C.c_int, [C.c_double] * 4 + [u32p, C.POINTER(C.c_double)]),
        "oracle_t_avg_closed_form": (C.c_double, [C.c_double] * 6),
        "oracle_t_avg_recurrence": (C.c_double, [C.c_uint32] + [C.c_double] * 5 + [C.c_uint64]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _u32(a):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint32))


# ---- stateless helpers -------------------------------------------------------------
def philox4x32_10(ctr, key):
    c, cp = _u32(ctr)
    k, kp = _u32(key)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(cp, kp, out.ctypes.data_as(C.POINTER(C.c_uint32)))
    return out


def neg2ln_uniform(w: int) -> float:
    return float(lib().oracle_neg2ln_uniform(C.c_uint32(w)))


def unit_circle_point(w: int):
    c, s = C.c_float(), C.c_float()
    lib().oracle_unit_circle_point(C.c_uint32(w), C.byref(c), C.byref(s))
    return c.value, s.value


def noise_z(seed, t, worker, j, kind) -> float:
    return float(lib().oracle_noise_z(seed, t, worker, j, kind))


def noise_fill(seed, t, worker, j0, count, kind) -> np.ndarray:
    out = np.empty(count, dtype=np.float32)
    lib().oracle_noise_fill(seed, t, worker, j0, count, kind, out.ctypes.data_as(C.POINTER(C.c_float)))
    return out


def k_from_delta(delta: float, d: int) -> int:
    return int(lib().oracle_k_from_delta(float(delta), int(d)))


def topk(p, k):
    """Indices (ascending) of the top-k of p under (|v| desc, index asc); also (T, r)."""
    p, pp = _f32(p)
    idx = np.empty(k, dtype=np.uint32)
    T, r = C.c_uint32(), C.c_uint64()
    lib().oracle_topk(pp, p.shape[0], k, idx.ctypes.data_as(C.POINTER(C.c_uint32)),
                      C.byref(T), C.byref(r))
    return idx, T.value, r.value


def queue_run(lam, xstar, x0, n, tau, T, delta, lr, seed, noise_kind, noise_scale, trajectory=False):
    lam, lp = _f32(lam)
    xstar, sp = _f32(xstar)
    x0, xp = _f32(x0)
    d = lam.shape[0]
    xf = np.empty(d, dtype=np.float32)
    traj = np.empty((T + 1, d), dtype=np.float32) if trajectory else None
    tp = traj.ctypes.data_as(C.POINTER(C.c_float)) if trajectory else None
    lib().oracle_queue_run(d, n, tau, T, float(delta), float(lr), lp, sp, xp, seed, noise_kind,
                           float(noise_scale), tp, xf.ctypes.data_as(C.POINTER(C.c_float)))
    return (xf, traj) if trajectory else xf


def randk_indices(seed, t, worker, d, k) -> np.ndarray:
    """Coordinates the Random-k sparsifier keeps for (seed, t, worker), ascending."""
    out = np.empty(k, dtype=np.uint32)
    lib().oracle_randk_indices(int(seed), int(t), int(worker), int(d), int(k),
                               out.ctypes.data_as(C.POINTER(C.c_uint32)))
    return out


def randk_permute(seed, t, worker, d, m) -> int:
    return int(lib().oracle_randk_permute(int(seed), int(t), int(worker), int(d), int(m)))


def quantize4(values):
    """4-bit block quantiser of a message: (packed codes, block steps, decoded values)."""
    v, vp_ = _f32(values)
    k = v.size
    codes = np.zeros((k + 1) // 2, dtype=np.uint8)
    steps = np.zeros((k + 255) // 256, dtype=np.float32)
    deq = np.zeros(k, dtype=np.float32)
    lib().oracle_quantize4(vp_, k, codes.ctypes.data_as(C.POINTER(C.c_uint8)),
                           steps.ctypes.data_as(C.POINTER(C.c_float)), deq.ctypes.data_as(C.POINTER(C.c_float)))
    return codes, steps, deq


def murmur_fmix32(h: int) -> int:
    return int(lib().oracle_murmur_fmix32(C.c_uint32(h)))


def phi(delta, tau):
    return float(lib().oracle_phi(float(delta), float(tau)))


def phi_prime(delta, tau):
    return float(lib().oracle_phi_prime(float(delta), float(tau)))


def deco_noniid(v_g, a, b, t_comp):
    tau, delta = C.c_uint32(), C.c_double()
    rc = lib().oracle_deco_noniid(float(v_g), float(a), float(b), float(t_comp), C.byref(tau), C.byref(delta))
    if rc != 0:
        return None
    return int(tau.value), float(delta.value)


HETEROGENEITY_KEY = 0xFFFFFFFFFFFFFFFE     # the step key the per-worker optimum shifts are drawn under


def delta_star(tau, v_g, a, b, t_comp):
    return float(lib().oracle_delta_star(float(tau), float(v_g), float(a), float(b), float(t_comp)))


def deco(v_g, a, b, t_comp):
    tau, delta = C.c_uint32(), C.c_double()
    rc = lib().oracle_deco(float(v_g), float(a), float(b), float(t_comp), C.byref(tau), C.byref(delta))
    if rc != 0:
        return None
    return int(tau.value), float(delta.value)


def t_avg_closed_form(tau, delta, v_g, a, b, t_comp):
    return float(lib().oracle_t_avg_closed_form(float(tau), float(delta), float(v_g), float(a),
                                                float(b), float(t_comp)))


def t_avg_recurrence(tau, delta, v_g, a, b, t_comp, E):
    return float(lib().oracle_t_avg_recurrence(int(tau), float(delta), float(v_g), float(a),
                                               float(b), float(t_comp), int(E)))


def lut_build(v_g, a_min, a_max, points, b, t_comp):
    """Section 4.5, pre-computation: DeCo at `points` bandwidths spaced evenly over [a_min, a_max]
    for the measured latency b.  Returns a list of (bandwidth, (tau, delta) or None)."""
    table = []
    for i in range(points):
        a = a_min + (a_max - a_min) * i / (points - 1)
        table.append((a, deco(v_g, a, b, t_comp)))
    return table


def lut_query(table, v_g, b, t_comp, a):
    """Section 4.5, runtime lookup: inside the recorded range the entry of the nearest sample
    bandwidth, outside it the online computation.  Returns (tau, delta, from_table) or None."""
    a_min, a_max = table[0][0], table[-1][0]
    if a_min <= a <= a_max:
        nearest = min(range(len(table)), key=lambda i: (abs(table[i][0] - a), -i))
        if table[nearest][1] is not None:
            return table[nearest][1] + (True,)
    online = deco(v_g, a, b, t_comp)
    return None if online is None else online + (False,)


class Oracle:
    """Normative (ring-form) DD-EF-SGD state on the CPU."""

    def __init__(self, d: int, n: int, tau_max: int, threads: int = 1):
        self.d, self.n, self.tau_max = int(d), int(n), int(tau_max)
        self._h = C.c_void_p(lib().oracle_create(self.d, self.n, self.tau_max))
        lib().oracle_set_threads(self._h, int(threads))

    def close(self):
        if self._h:
            lib().oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_problem(self, lam, xstar, x0, seed, noise_kind, noise_scale):
        _, lp = _f32(lam)
        _, sp = _f32(xstar)
        _, xp = _f32(x0)
        lib().oracle_set_problem(self._h, lp, sp, xp, int(seed), int(noise_kind), float(noise_scale))

    def set_tau(self, tau):
        lib().oracle_set_tau(self._h, int(tau))

    def set_heterogeneity(self, zeta):
        """Non-IID workers: worker i's optimum is x* + zeta * u_i, u_i a fixed standard normal vector."""
        lib().oracle_set_heterogeneity(self._h, float(zeta))

    def set_compressor(self, kind):
        """0: Top-k (default), 1: Random-k, 2: composed (Random-k, Top-k inside it, 4-bit codes)."""
        lib().oracle_set_compressor(self._h, int(kind))

    def set_composed(self, rand_ratio):
        """Share of the coordinates the Random-k stage of the composed compressor keeps."""
        lib().oracle_set_composed(self._h, float(rand_ratio))

    def get_message_codes(self, w):
        """Wire form of worker w's last composed message: packed 4-bit codes and block steps."""
        k = int(lib().oracle_message_size(self._h, int(w)))
        codes = np.zeros((k + 1) // 2, dtype=np.uint8)
        steps = np.zeros((k + 255) // 256, dtype=np.float32)
        lib().oracle_get_message_codes(self._h, int(w), codes.ctypes.data_as(C.POINTER(C.c_uint8)),
                                       steps.ctypes.data_as(C.POINTER(C.c_float)))
        return codes, steps

    @property
    def t(self):
        return int(lib().oracle_step_index(self._h))

    def grad(self):
        lib().oracle_grad(self._h)

    def load_grad(self, worker, g):
        _, gp = _f32(g)
        lib().oracle_load_grad(self._h, int(worker), gp)

    def ef_compress(self, delta, lr):
        lib().oracle_ef_compress(self._h, float(delta), float(lr))

    def aggregate(self):
        lib().oracle_aggregate(self._h)

    def apply_delayed(self):
        lib().oracle_apply_delayed(self._h)

    def step(self, delta, lr):
        lib().oracle_step(self._h, float(delta), float(lr))

    def _get_vec(self, fn, *args):
        out = np.empty(self.d, dtype=np.float32)
        fn(self._h, *args, out.ctypes.data_as(C.POINTER(C.c_float)))
        return out

    def get_model(self):
        return self._get_vec(lib().oracle_get_model)

    def objective(self):
        """f(x_t) = (1/n) sum_i f_i(x_t) of the synthetic quadratics, in double."""
        return float(lib().oracle_objective(self._h))

    def set_model(self, x):
        _, xp = _f32(x)
        lib().oracle_set_model(self._h, xp)

    def get_snapshot(self, step):
        return self._get_vec(lib().oracle_get_snapshot, int(step))

    def get_error(self, w):
        return self._get_vec(lib().oracle_get_error, int(w))

    def set_error(self, w, e):
        _, ep = _f32(e)
        lib().oracle_set_error(self._h, int(w), ep)

    def get_grad(self, w):
        return self._get_vec(lib().oracle_get_grad, int(w))

    def get_update(self):
        return self._get_vec(lib().oracle_get_update)

    def get_message(self, w):
        k = int(lib().oracle_message_size(self._h, int(w)))
        idx = np.empty(k, dtype=np.uint32)
        val = np.empty(k, dtype=np.float32)
        lib().oracle_get_message(self._h, int(w), idx.ctypes.data_as(C.POINTER(C.c_uint32)),
                                 val.ctypes.data_as(C.POINTER(C.c_float)))
        return idx, val

    def get_threshold(self, w):
        T, r = C.c_uint32(), C.c_uint64()
        lib().oracle_get_threshold(self._h, int(w), C.byref(T), C.byref(r))
        return int(T.value), int(r.value)


class QueueOracle:
    """Algorithm 1 as printed, one iteration at a time: workers at the current x, the server
    applying the message sent tau iterations earlier (constant tau)."""

    def __init__(self, d: int, n: int, tau: int):
        self.d, self.n, self.tau = int(d), int(n), int(tau)
        self._h = C.c_void_p(lib().oracle_queue_create(self.d, self.n, self.tau))

    def close(self):
        if self._h:
            lib().oracle_queue_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_problem(self, lam, xstar, x0, seed, noise_kind, noise_scale):
        _, lp = _f32(lam)
        _, sp = _f32(xstar)
        _, xp = _f32(x0)
        lib().oracle_queue_set_problem(self._h, lp, sp, xp, int(seed), int(noise_kind), float(noise_scale))

    def set_tau(self, tau):
        self.tau = int(tau)
        lib().oracle_queue_set_tau(self._h, self.tau)

    def set_heterogeneity(self, zeta):
        lib().oracle_queue_set_heterogeneity(self._h, float(zeta))

    def step(self, delta, lr):
        lib().oracle_queue_step(self._h, float(delta), float(lr))

    def _vec(self, fn, *args):
        out = np.empty(self.d, dtype=np.float32)
        fn(self._h, *args, out.ctypes.data_as(C.POINTER(C.c_float)))
        return out

    def get_model(self):
        return self._vec(lib().oracle_queue_get_model)

    def get_update(self):
        return self._vec(lib().oracle_queue_get_update)

    def get_error(self, w):
        return self._vec(lib().oracle_queue_get_error, int(w))

    def get_message(self, w):
        k = int(lib().oracle_queue_message_size(self._h, int(w)))
        idx = np.empty(k, dtype=np.uint32)
        val = np.empty(k, dtype=np.float32)
        lib().oracle_queue_get_message(self._h, int(w), idx.ctypes.data_as(C.POINTER(C.c_uint32)),
                                       val.ctypes.data_as(C.POINTER(C.c_float)))
        return idx, val
