"""The allocation-free entry point ddef_ef_compress_static against ddef_ef_compress: same error
buffers and gradients in, bit-identical messages and residuals out, on two calls in a row (the
second on a smaller problem, so that whatever the first left in the shared work memory is in the
way), through the C-ABI.  The caller's device buffers and stream come straight from the HIP runtime
(the one the library itself runs on), through ctypes."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

F32 = np.float32


class Hip:
    """The few HIP runtime calls a caller of the entry point needs: buffers, copies, a stream."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")
        self.owned = []

    def ok(self, rc, what):
        assert rc == 0, f"{what} failed with HIP error {rc}"

    def malloc(self, nbytes):
        p = C.c_void_p()
        self.ok(self.lib.hipMalloc(C.byref(p), C.c_size_t(nbytes)), "hipMalloc")
        self.owned.append(p)
        return p

    def upload(self, array):
        a = np.ascontiguousarray(array)
        p = self.malloc(a.nbytes)
        self.ok(self.lib.hipMemcpy(p, C.c_void_p(a.ctypes.data), C.c_size_t(a.nbytes), C.c_int(1)), "hipMemcpy")
        return p

    def download(self, p, shape, dtype):
        out = np.empty(shape, dtype=dtype)
        self.ok(self.lib.hipMemcpy(C.c_void_p(out.ctypes.data), p, C.c_size_t(out.nbytes), C.c_int(2)), "hipMemcpy")
        return out

    def stream(self):
        s = C.c_void_p()
        self.ok(self.lib.hipStreamCreateWithFlags(C.byref(s), C.c_uint(1)), "hipStreamCreateWithFlags")
        return s

    def sync(self):
        self.ok(self.lib.hipDeviceSynchronize(), "hipDeviceSynchronize")

    def release(self, stream=None):
        self.sync()
        if stream is not None:
            self.lib.hipStreamDestroy(stream)
        for p in self.owned:
            self.lib.hipFree(p)
        self.owned = []


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


def reference(ddef, e, g, delta, lr):
    """ddef_ef_compress on a context that was handed the same e and g."""
    n, d = e.shape
    zero = np.zeros(d, dtype=F32)
    c = ddef.Context(d, n, 0)
    c.set_problem(np.ones(d, dtype=F32), zero, zero, 0, 0, 0.0)
    c.set_tau(0)
    c.set_option(ddef.OPT_FORCE_FULL_SELECT, 0)
    for i in range(n):
        c.set_error(i, e[i])
        c.load_grad(i, g[i])
    c.ef_compress(delta, lr)
    out = [(c.get_message(i), c.get_error(i)) for i in range(n)]
    c.close()
    return out


def static_call(ddef, hip, e, g, delta, lr, pad, side_stream=False):
    n, d = e.shape
    ld = (d + 3) // 4 * 4 + 4 * pad
    k = ddef.k_from_delta(delta, d)
    msg_ld = k + 5
    e_rows = np.zeros((n, ld), dtype=F32)
    g_rows = np.zeros((n, ld), dtype=F32)
    e_rows[:, :d] = e
    g_rows[:, :d] = g
    e_dev, g_dev = hip.upload(e_rows), hip.upload(g_rows)
    idx_dev = hip.upload(np.full((n, msg_ld), 0x7FFFFFFF, dtype=np.uint32))
    val_dev = hip.upload(np.full((n, msg_ld), -1.0, dtype=F32))
    hip.sync()
    # the null stream, or a stream of the caller's own
    stream = hip.stream() if side_stream else None
    rc = ddef.ef_compress_static(e_dev.value, g_dev.value, ld, d, n, delta, lr, idx_dev.value, val_dev.value, msg_ld,
                                 stream.value if stream is not None else 0)
    assert rc == ddef.OK, ddef.strerror(rc)
    hip.sync()
    idx = hip.download(idx_dev, (n, msg_ld), np.uint32)
    val = hip.download(val_dev, (n, msg_ld), F32)
    res = hip.download(e_dev, (n, ld), F32)
    hip.release(stream)
    assert np.all(idx[:, k:] == 0x7FFFFFFF) and np.all(val[:, k:] == -1.0)      # nothing past k was written
    return [((idx[i, :k].copy(), val[i, :k].copy()), res[i, :d].copy()) for i in range(n)]


def make_inputs(seed, n, d, ties):
    rng = np.random.default_rng(seed)
    e = (rng.standard_t(3, size=(n, d)) * 0.05).astype(F32)
    g = rng.standard_normal((n, d)).astype(F32)
    if ties:                       # many equal magnitudes around the threshold, both signs
        e[:, ::7] = F32(0.25)
        e[:, 3::14] = F32(-0.25)
        g[:, ::7] = 0
        g[:, 3::14] = 0
    return e, g


def test_static_entry_point_matches_ef_compress_twice_in_a_row():
    from paper_2507_17346_amd import binding as ddef
    ddef.load()
    hip = Hip()
    # first call: several tiles and chunks, a ragged tail, ties at the threshold; second: smaller
    # in d, n and k, straight after it (on a stream of the caller's own); third: a handful of entries;
    # fourth: as many workers as the work memory holds, over what the smaller calls left in it
    cases = [(11, 3, 300_017, 0.06, True, 2), (12, 2, 70_001, 0.003, False, 0), (13, 1, 5, 0.4, False, 1),
             (14, 64, 9_001, 0.02, True, 1)]
    for seed, n, d, delta, ties, pad in cases:
        e, g = make_inputs(seed, n, d, ties)
        lr = 0.05
        got = static_call(ddef, hip, e, g, delta, lr, pad, side_stream=(seed == 12))
        want = reference(ddef, e, g, delta, lr)
        for i in range(n):
            (gi, gv), ge = got[i]
            (wi, wv), we = want[i]
            assert np.array_equal(gi, wi), (d, i, "indices")
            assert np.array_equal(bits(gv), bits(wv)), (d, i, "values")
            assert np.array_equal(bits(ge), bits(we)), (d, i, "residual")


def test_static_entry_point_rejects_what_it_cannot_hold():
    from paper_2507_17346_amd import binding as ddef
    ddef.load()
    hip = Hip()
    p = hip.upload(np.zeros(1024, dtype=F32)).value
    q = hip.upload(np.zeros(1024, dtype=np.uint32)).value
    r = hip.upload(np.zeros(1024, dtype=F32)).value
    call = lambda **kw: ddef.ef_compress_static(**{**dict(dev_e=p, dev_g=p, ld=1024, d=1000, n=1, delta=0.01, lr=0.05,
                                                          dev_msg_idx=q, dev_msg_val=r, msg_ld=1024), **kw})
    assert call() == ddef.OK
    assert call(n=65) == ddef.EINVAL                                   # more workers than the work memory holds
    assert call(d=2 ** 32 - 9000, ld=2 ** 32 - 9000 + 8, n=8) == ddef.EINVAL   # more chunks than it holds
    assert call(ld=999) == ddef.EINVAL and call(ld=1002) == ddef.EINVAL
    assert call(dev_e=p + 4) == ddef.EINVAL
    assert call(msg_ld=9) == ddef.EINVAL and call(delta=0.0) == ddef.EINVAL and call(dev_g=0) == ddef.EINVAL
    hip.release()
