"""The allocation-free entry point ddef_ef_compress_static against ddef_ef_compress: same error
buffers and gradients in, bit-identical messages and residuals out, on two calls in a row (the
second on a smaller problem, so that whatever the first left in the shared work memory is in the
way), through the C-ABI.  torch only provides the caller's device buffers and the stream."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

F32 = np.float32


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


def static_call(ddef, torch, e, g, delta, lr, pad, side_stream=False):
    n, d = e.shape
    ld = (d + 3) // 4 * 4 + 4 * pad
    k = ddef.k_from_delta(delta, d)
    msg_ld = k + 5
    dev = torch.device("cuda:0")
    e_t = torch.zeros((n, ld), dtype=torch.float32, device=dev)
    g_t = torch.zeros((n, ld), dtype=torch.float32, device=dev)
    e_t[:, :d] = torch.from_numpy(e).to(dev)
    g_t[:, :d] = torch.from_numpy(g).to(dev)
    idx_t = torch.full((n, msg_ld), 0x7FFFFFFF, dtype=torch.int32, device=dev)
    val_t = torch.full((n, msg_ld), -1.0, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    # the null stream, or a stream of the caller's own
    owner = torch.cuda.Stream(device=dev) if side_stream else torch.cuda.current_stream()
    stream = owner.cuda_stream
    rc = ddef.ef_compress_static(e_t.data_ptr(), g_t.data_ptr(), ld, d, n, delta, lr, idx_t.data_ptr(),
                                 val_t.data_ptr(), msg_ld, stream)
    assert rc == ddef.OK, ddef.strerror(rc)
    torch.cuda.synchronize()
    idx = idx_t.cpu().numpy().view(np.uint32)
    val = val_t.cpu().numpy()
    assert np.all(idx[:, k:] == 0x7FFFFFFF) and np.all(val[:, k:] == -1.0)      # nothing past k was written
    return [((idx[i, :k].copy(), val[i, :k].copy()), e_t[i, :d].cpu().numpy()) for i in range(n)]


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
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2507_17346_amd import binding as ddef
    ddef.load()
    # first call: several tiles and chunks, a ragged tail, ties at the threshold; second: smaller
    # in d, n and k, straight after it on the same stream
    cases = [(11, 3, 300_017, 0.06, True, 2), (12, 2, 70_001, 0.003, False, 0), (13, 1, 5, 0.4, False, 1)]
    for seed, n, d, delta, ties, pad in cases:
        e, g = make_inputs(seed, n, d, ties)
        lr = 0.05
        got = static_call(ddef, torch, e, g, delta, lr, pad, side_stream=(seed == 12))
        want = reference(ddef, e, g, delta, lr)
        for i in range(n):
            (gi, gv), ge = got[i]
            (wi, wv), we = want[i]
            assert np.array_equal(gi, wi), (d, i, "indices")
            assert np.array_equal(bits(gv), bits(wv)), (d, i, "values")
            assert np.array_equal(bits(ge), bits(we)), (d, i, "residual")


def test_static_entry_point_rejects_what_it_cannot_hold():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2507_17346_amd import binding as ddef
    ddef.load()
    buf = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    out_i = torch.zeros(1024, dtype=torch.int32, device="cuda:0")
    out_v = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    p, q, r = buf.data_ptr(), out_i.data_ptr(), out_v.data_ptr()
    call = lambda **kw: ddef.ef_compress_static(**{**dict(dev_e=p, dev_g=p, ld=1024, d=1000, n=1, delta=0.01, lr=0.05,
                                                          dev_msg_idx=q, dev_msg_val=r, msg_ld=1024), **kw})
    assert call() == ddef.OK
    assert call(n=65) == ddef.EINVAL                                   # more workers than the work memory holds
    assert call(d=2 ** 32 - 9000, ld=2 ** 32 - 9000 + 8, n=8) == ddef.EINVAL   # more chunks than it holds
    assert call(ld=999) == ddef.EINVAL and call(ld=1002) == ddef.EINVAL
    assert call(dev_e=p + 4) == ddef.EINVAL
    assert call(msg_ld=9) == ddef.EINVAL and call(delta=0.0) == ddef.EINVAL and call(dev_g=0) == ddef.EINVAL
    torch.cuda.synchronize()
