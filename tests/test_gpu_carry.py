"""GPU parity of the carried-codebook path (DLC_FLAG_CARRY_CODEBOOK): a sequence of payloads through one context
against the same sequence through the oracle, container by container, byte for byte.

The oracle chain is its own: call k is given the counts the oracle itself reported for call k-1; nothing the GPU
produced goes into it.
"""
import numpy as np
import pytest

import dlc_workloads as W
import oracle
from gpu_util import to_device

pytestmark = pytest.mark.gpu

R = 512


def _batch(T, B, D, seed, sigma=0.02, dtype=np.float32, rows=80, shift=0.0):
    rng = np.random.default_rng(seed)
    table = (rng.standard_normal((rows, D)) * sigma + shift).astype(np.float32)
    idx = rng.integers(0, rows, (T, B))
    x = table[idx] * (1 + np.arange(T, dtype=np.float32)[:, None, None])
    return x.astype(dtype)


class _Chain:
    """one context with the flag; compress() returns (container bytes, sizes, reconstruction)"""

    def __init__(self, shape, dtype, S, Rr=R, LMAX=12):
        import torch
        from paper_2407_04272_amd import binding as b
        self.b = b
        T, B, D = shape
        dt = b.F16 if np.dtype(dtype) == np.float16 else b.F32
        self.cfg = b.make_config(dt, T, B, D, Rr, S, LMAX, b.FLAG_CARRY_CODEBOOK)
        self.ctx = b.Context(self.cfg)
        self.cap = b.dlc_compress_bound(self.cfg)
        self.d_out = torch.zeros(self.cap + 64, dtype=torch.uint8, device="cuda")
        self.d_sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")

    def compress(self, x, ebs):
        import torch
        d = to_device(x)
        self.ctx.set_error_bounds(eb=ebs)
        self.d_out.fill_(0xA5)
        assert self.ctx.compress(d, self.d_out, self.d_sizes, capacity=self.cap) == 0
        assert self.ctx.sync_status() == 0
        sizes = self.d_sizes.cpu().numpy().astype(np.uint64)
        total = int(sizes[0])
        out = self.d_out.cpu().numpy()
        assert np.all(out[self.cap:] == 0xA5)
        rec = torch.full_like(d, 7.0)
        assert self.ctx.decompress(self.d_out, total, rec) == 0
        assert self.ctx.sync_status() == 0
        return out[:total].copy(), sizes, rec.cpu().numpy()


def _same(g, o, x, what):
    data, sizes, rec = g
    assert o.rc == 0, what
    assert data.size == o.data.size, (what, data.size, o.data.size)
    diff = np.nonzero(data != o.data)[0]
    assert diff.size == 0, f"{what}: first differing byte {diff[:8]} of {data.size}"
    assert np.array_equal(sizes, o.sizes), what
    rc, orec = oracle.decompress(o.data, x.shape, x.dtype)
    assert rc == 0
    u = np.uint32 if x.dtype == np.float32 else np.uint16
    assert np.array_equal(rec.view(u), orec.view(u)), what


CASES = [  # T, B, D, S, eb, dtype
    (1, 256, 16, 256, 1e-3, np.float32),     # less than one group
    (2, 37, 13, 64, 2e-3, np.float32),       # ragged: B*D = 481 not a multiple of 4 (scalar loads), partial group
    (3, 1000, 50, 256, 2e-3, np.float32),    # several groups and a partial last one
    (5, 700, 48, 128, 1e-3, np.float32),
    (2, 2048, 64, 64, 5e-4, np.float32),     # long codes: chunks that do not fit their LDS words are walked twice
    (3, 900, 40, 256, 4e-3, np.float16),     # half precision: many escapes (records written by the second walk)
    (2, 512, 32, 128, 2e-3, np.float16),
]


@pytest.mark.parametrize("T,B,D,S,eb,dtype", CASES)
def test_chain_matches_the_oracle(T, B, D, S, eb, dtype):
    print("carried chain", T, B, D, S, eb, np.dtype(dtype).name, flush=True)
    ebs = (np.float32(eb) * (1 + np.arange(T, dtype=np.float32))).astype(np.float32)
    ch = _Chain((T, B, D), dtype, S)
    prev = None
    for k in range(4):
        x = _batch(T, B, D, 100 * k + B + D, dtype=dtype)
        if k == 2:
            x.reshape(-1)[::211] = 1e4 if dtype == np.float32 else 6e4     # true escapes
            x.reshape(-1)[5] = np.nan
        if k == 3:
            x.reshape(-1)[::2999] = -3e4                                   # a few per group: records kept on the way
        g = ch.compress(x, ebs)
        o = oracle.compress(x, ebs, R, S, 12, carry_hist=prev, want_hist=True)
        _same(g, o, x, f"call {k}")
        prev = o.hist


def test_new_bounds_start_a_new_chain():
    T, B, D, S = 3, 600, 32, 128
    ch = _Chain((T, B, D), np.float32, S)
    e1 = np.full(T, 2e-3, np.float32)
    e2 = np.full(T, 1e-3, np.float32)
    x0, x1, x2, x3 = (_batch(T, B, D, s) for s in (1, 2, 3, 4))
    o0 = oracle.compress(x0, e1, R, S, 12, want_hist=True)
    _same(ch.compress(x0, e1), o0, x0, "first call")
    o1 = oracle.compress(x1, e1, R, S, 12, carry_hist=o0.hist, want_hist=True)
    _same(ch.compress(x1, e1), o1, x1, "carried")
    # a changed bound: the symbols mean something else now, the call builds its own codebook
    o2 = oracle.compress(x2, e2, R, S, 12, want_hist=True)
    _same(ch.compress(x2, e2), o2, x2, "after new bounds")
    o3 = oracle.compress(x3, e2, R, S, 12, carry_hist=o2.hist, want_hist=True)
    _same(ch.compress(x3, e2), o3, x3, "carried again")


def test_payload_unlike_the_previous_one():
    """Nothing of the new payload has a code: every element becomes an escape, bit-exact and still in order."""
    T, B, D, S = 2, 300, 16, 64
    ch = _Chain((T, B, D), np.float32, S)
    ebs = np.full(T, 1e-3, np.float32)
    x0 = _batch(T, B, D, 7)
    x1 = _batch(T, B, D, 8, shift=0.3)
    o0 = oracle.compress(x0, ebs, R, S, 12, want_hist=True)
    _same(ch.compress(x0, ebs), o0, x0, "first")
    o1 = oracle.compress(x1, ebs, R, S, 12, carry_hist=o0.hist, want_hist=True)
    g1 = ch.compress(x1, ebs)
    _same(g1, o1, x1, "all escapes")
    assert np.array_equal(g1[2].view(np.uint32), x1.view(np.uint32))
    # and back to ordinary data: the counts of the all-escape call carry nothing but the escape
    x2 = _batch(T, B, D, 9)
    o2 = oracle.compress(x2, ebs, R, S, 12, carry_hist=o1.hist, want_hist=True)
    _same(ch.compress(x2, ebs), o2, x2, "after all escapes")


def test_small_alphabet_and_constant_table():
    T, B, D, S = 2, 256, 16, 64
    ch = _Chain((T, B, D), np.float32, S, Rr=64, LMAX=8)
    ebs = np.array([1e-3, 1.0], np.float32)            # table 1: one symbol
    prev = None
    for k in range(3):
        x = _batch(T, B, D, 20 + k)
        g = ch.compress(x, ebs)
        o = oracle.compress(x, ebs, 64, S, 8, carry_hist=prev, want_hist=True)
        _same(g, o, x, f"call {k}")
        prev = o.hist


def test_wide_alphabet_chain():
    """Radius 2048 and bins much narrower than the data: most symbols lie outside the 255-symbol window around bin 0
    (counted and looked up one by one), and chunks are far longer than their LDS words."""
    T, B, D, S = 2, 1024, 32, 128
    ch = _Chain((T, B, D), np.float32, S, Rr=2048, LMAX=12)
    ebs = np.array([2e-5, 1e-4], np.float32)
    prev = None
    for k in range(3):
        x = _batch(T, B, D, 40 + k, sigma=0.01)
        g = ch.compress(x, ebs)
        o = oracle.compress(x, ebs, 2048, S, 12, carry_hist=prev, want_hist=True)
        _same(g, o, x, f"call {k}")
        prev = o.hist


def test_workload3_consecutive_iterations_full_size():
    """The benchmark shape: iteration i+1 coded with iteration i's codebook, byte for byte against the oracle."""
    import torch
    from paper_2407_04272_amd import binding as b
    print("workload 5 forward payloads, 128 x 8192 x 128, two iterations", flush=True)
    gen = W.Workload5(device="cuda")
    f0 = gen.step()[0].clone()
    f1 = gen.step()[0].clone()
    T, B, D = f0.shape
    lo = f0.amin(dim=(1, 2)).cpu().numpy()
    hi = f0.amax(dim=(1, 2)).cpu().numpy()
    ebs = (0.03 * (hi - lo)).astype(np.float32)
    ctx = b.Context(b.make_config(b.F32, T, B, D, chunk_symbols=256, flags=b.FLAG_CARRY_CODEBOOK))
    ctx.set_error_bounds(eb=ebs)
    out = torch.zeros(f0.numel() * 4, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")
    prev = None
    for k, d in enumerate((f0, f1)):
        assert ctx.compress(d, out, sizes) == 0 and ctx.sync_status() == 0
        total = int(sizes[0].item())
        data = out[:total].cpu().numpy()
        rec = torch.empty_like(d)
        assert ctx.decompress(out, total, rec) == 0 and ctx.sync_status() == 0
        x = d.cpu().numpy()
        print("oracle, iteration", k, flush=True)
        o = oracle.compress(x, ebs, carry_hist=prev, want_hist=True)
        assert o.rc == 0 and o.data.size == data.size and np.array_equal(o.data, data), k
        assert np.array_equal(o.sizes, sizes.cpu().numpy().astype(np.uint64))
        err = (d.double() - rec.double()).abs().amax(dim=(1, 2)).cpu().numpy()
        assert np.all(err <= ebs.astype(np.float64) * (1 + 1e-6))
        prev = o.hist


def test_f16_ties_on_the_single_pass_path():
    from test_oracle_quantizer import half_tie_payload
    x, ebs = half_tie_payload()
    ch = _Chain(x.shape, np.float16, 128)
    prev = None
    for k in range(2):
        g = ch.compress(x, ebs)
        o = oracle.compress(x, ebs, R, 128, 12, carry_hist=prev, want_hist=True)
        _same(g, o, x, f"call {k}")
        prev = o.hist


def test_periodic_reclassification_in_a_carried_run():
    """Every fourth iteration the tables are classified again from the current payload (dlc_stats, then
    dlc_set_error_bounds with those statistics); in between the schedule alone moves the bounds.  Statistics,
    classes, bounds and containers against the oracle; the carried chain starts anew whenever a bound changed."""
    from paper_2407_04272_amd import binding as b
    T, B, D, S = 4, 512, 32, 128
    ch = _Chain((T, B, D), np.float32, S)
    p = b.ControllerParams(mode=0, decay_kind=b.DECAY_STEPWISE, global_eb=2e-3, alpha=5.0 / 3.0, beta=3.0, h_large=0.0,
                           h_small=0.05, decay_start=0, decay_len=6, decay_steps=2, reserved=0, decay_mult0=2.0,
                           eb_min=0.0, eb_max=0.0, rel_floor=0.0)
    op = oracle.ControllerParams(**{f[0]: getattr(p, f[0]) for f in p._fields_})
    probe = np.full(T, 2e-3, np.float32)
    st = ost = None
    prev_hist, prev_eb = None, None
    classes, carried_calls, fresh_calls = [], 0, 0
    for it in range(12):
        x = _batch(T, B, D, 300 + it, rows=300)
        if it < 6:                                  # early on the rows of this table merge once quantised ...
            x[2] = x[2, :1] + np.random.default_rng(it).standard_normal((B, D)).astype(np.float32) * np.float32(1e-5)
        x[1, B // 2:] = x[1, :B // 2]               # (a table with repeated rows throughout)
        if it % 4 == 0:                             # ... so its class changes at a later re-classification
            st = ch.ctx.stats(to_device(x), probe)
            ost = oracle.stats(x, probe)
            for t in range(T):
                assert (st[t].n_unique_raw, st[t].n_unique_quant, st[t].min, st[t].max) == \
                       (ost[t].n_unique_raw, ost[t].n_unique_quant, ost[t].min, ost[t].max), (it, t)
        ebs, cls = ch.ctx.set_error_bounds(stats=st, params=p, iteration=it)
        oeb, ocls = oracle.controller(ost, op, it)
        assert np.array_equal(ebs.view(np.uint32), oeb.view(np.uint32)) and np.array_equal(cls, ocls), it
        classes.append(tuple(int(c) for c in cls))
        carried = prev_eb is not None and np.array_equal(prev_eb.view(np.uint32), oeb.view(np.uint32))
        carried_calls += carried
        fresh_calls += not carried
        o = oracle.compress(x, oeb, R, S, 12, carry_hist=prev_hist if carried else None, want_hist=True)
        _same(ch.compress(x, ebs), o, x, f"iteration {it}")
        prev_hist, prev_eb = o.hist, oeb
    assert len(set(classes)) >= 2                   # a re-classification did change a class
    assert carried_calls >= 4 and fresh_calls >= 3  # both kinds of call were exercised


def test_many_small_tables_both_paths():
    """600 tables of two groups each: the codebook kernels build four tables per work-group (a wavefront each, the
    whole work-group for the tables with more than 64 used symbols), the decoder runs work-groups of two wavefronts.
    Tables of one symbol, of a few, of a wide alphabet and with escapes; the default path and a chain of three calls
    on the single-pass path, each against the oracle."""
    T, B, D, S = 600, 32, 64, 64             # 2048 elements a table = 1 group of 64 x 64 symbols, half of a second
    rng = np.random.default_rng(99)
    ebs = np.full(T, 2e-3, np.float32)

    def batch(k):
        x = (rng.standard_normal((T, B, D)) * 0.01).astype(np.float32)
        x[0:600:7] *= 40.0                   # wide alphabets: more than 64 used symbols
        x[3:600:50] = 0.25                   # one symbol
        x[5:600:50, :, ::2] = 0.0            # two or three symbols
        x[9:600:31, 2, 3] = 1e6              # an escape
        if k == 2:
            x[11:600:13] *= 25.0             # other tables turn wide: symbols without a carried code
        return x

    x0 = batch(0)
    from gpu_util import DeviceRun
    g = DeviceRun(x0, ebs, S=S)
    o = oracle.compress(x0, ebs, R, S, 12)
    assert g.status == 0 and o.rc == 0 and np.array_equal(g.sizes, o.sizes) and np.array_equal(g.data, o.data)
    st, rec = g.decompress()
    rc, orec = oracle.decompress(o.data, x0.shape, x0.dtype)
    assert st == 0 and rc == 0 and np.array_equal(rec.view(np.uint32), orec.view(np.uint32))
    ch = _Chain((T, B, D), np.float32, S)
    prev = None
    for k in range(3):
        x = batch(k)
        gk = ch.compress(x, ebs)
        ok = oracle.compress(x, ebs, R, S, 12, carry_hist=prev, want_hist=True)
        _same(gk, ok, x, f"many tables, call {k}")
        prev = ok.hist


# ------------------------------------------------------------------------------------------------
# DLC_FLAG_SAMPLE_CODEBOOK: the same single-pass kernels, the codebook from a few groups of the payload itself
# ------------------------------------------------------------------------------------------------
def _sampled(x, ebs, S, n_calls=1, Rr=R, LMAX=12):
    import torch
    from paper_2407_04272_amd import binding as b
    T, B, D = x.shape
    f16 = x.dtype == np.float16
    cfg = b.make_config(b.F16 if f16 else b.F32, T, B, D, Rr, S, LMAX, b.FLAG_SAMPLE_CODEBOOK)
    ctx = b.Context(cfg)
    ctx.set_error_bounds(eb=ebs)
    cap = b.dlc_compress_bound(cfg)
    out = torch.zeros(cap + 64, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")
    d = to_device(x)
    for _ in range(n_calls):
        out.fill_(0xA5)
        assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
    sz = sizes.cpu().numpy().astype(np.uint64)
    h = out.cpu().numpy()
    assert np.all(h[cap:] == 0xA5)
    rec = torch.full_like(d, 7.0)
    assert ctx.decompress(out, int(sz[0]), rec) == 0 and ctx.sync_status() == 0
    return (h[:int(sz[0])].copy(), sz, rec.cpu().numpy()), ctx


@pytest.mark.parametrize("T,B,D,S,eb,dtype", CASES + [
    (2, 8192, 128, 256, 2e-3, np.float32),   # 64 groups a table: groups 0, 16, 32, 48 are the sample
    (3, 4096, 64, 64, 2e-3, np.float32),     # 64 groups of 4096 elements: sixteen sampled
    (2, 5000, 100, 128, 3e-3, np.float16),   # 62 groups, the last ragged; stride 7
])
def test_sampled_codebook_matches_the_oracle(T, B, D, S, eb, dtype):
    x = _batch(T, B, D, 17 * B + D, dtype=dtype, rows=max(80, B // 4))
    x.reshape(-1)[::1013] = 6e4 if dtype == np.float16 else 1e9
    ebs = (np.float32(eb) * (1 + np.arange(T, dtype=np.float32))).astype(np.float32)
    g, _ = _sampled(x, ebs, S, n_calls=2)    # (the second call finds what the first left in the workspace)
    _same(g, oracle.compress(x, ebs, R, S, 12, sample_codebook=True), x, "sampled codebook")


def test_sampled_codebook_symbols_outside_the_sample_become_escapes():
    T, B, D, S = 2, 8192, 128, 256
    rng = np.random.default_rng(5)
    x = (rng.integers(-2, 3, (T, B, D)) * 4e-3).astype(np.float32)       # five symbols
    flat = x.reshape(T, -1)
    flat[:, 16384 * 5:16384 * 7] = (rng.integers(-40, 41, (T, 16384 * 2)) * 4e-3).astype(np.float32)  # groups 5, 6: eighty-one
    ebs = np.full(T, 2e-3, np.float32)
    g, ctx = _sampled(x, ebs, S)
    o = oracle.compress(x, ebs, R, S, 12, sample_codebook=True)
    _same(g, o, x, "symbols outside the sample")
    assert o.data.size > oracle.compress(x, ebs, R, S, 12).data.size
    hist = ctx.read_histogram()              # the counts the codebook was built from: the sample's
    assert np.array_equal(hist.astype(np.uint64), oracle.sample_histogram(x, ebs, R, S))
    ln, code = ctx.read_codebook()           # and the codebook the container was coded with: theirs, the escape counted once more
    for t in range(T):
        h = hist[t].astype(np.uint64)
        h[0] += 1
        oln, ocode, _, _ = oracle.codebook(h, 12)
        assert np.array_equal(ln[t], oln) and np.array_equal(code[t][oln > 0], ocode[oln > 0].astype(np.uint16))


def test_sampled_codebook_workload3_full_size():
    """The whole workload-3 payload (128 x 8192 x 128): sizes against the oracle on the first tables, the bound on all."""
    import torch
    from paper_2407_04272_amd import binding as b
    w = W.workload3(device="cuda")
    x = w.payload
    T, B, D = x.shape
    flat = x.reshape(T, -1)
    rng_t = (flat.max(dim=1).values - flat.min(dim=1).values).cpu().numpy()
    ebs = (0.03 * rng_t).astype(np.float32)
    cfg = b.make_config(b.F32, T, B, D, R, 256, 12, b.FLAG_SAMPLE_CODEBOOK)
    ctx = b.Context(cfg)
    ctx.set_error_bounds(eb=ebs)
    cap = b.dlc_compress_bound(cfg)
    out = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")
    assert ctx.compress(x, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
    sz = sizes.cpu().numpy().astype(np.uint64)
    rec = torch.empty_like(x)
    assert ctx.decompress(out, int(sz[0]), rec) == 0 and ctx.sync_status() == 0
    err = (rec.double() - x.double()).abs().reshape(T, -1).max(dim=1).values.cpu().numpy()
    assert np.all(err <= ebs.astype(np.float64))
    nt = 6
    xs = x[:nt].cpu().numpy()
    o = oracle.compress(xs, ebs[:nt], R, 256, 12, sample_codebook=True)
    assert o.rc == 0 and np.array_equal(sz[1:1 + nt], o.sizes[1:1 + nt])
    rc, orec = oracle.decompress(o.data, xs.shape, np.float32)
    assert rc == 0 and np.array_equal(rec[:nt].cpu().numpy().view(np.uint32), orec.view(np.uint32))


def test_sampled_codebook_workload4_f16_full_size():
    """Workload 4 in half precision at its full size (64 x 16384 x 128, escapes in the percent range): the whole
    container against the oracle's, byte for byte."""
    import torch
    from paper_2407_04272_amd import binding as b
    w = W.workload4(device="cuda")
    d = w.meta["payload_f16"]
    del w
    T, B, D = d.shape
    lo = d.float().amin(dim=(1, 2)).cpu().numpy()
    hi = d.float().amax(dim=(1, 2)).cpu().numpy()
    ebs = np.maximum(0.03 * (hi - lo), np.float32(2.0 ** -10) * (hi - lo)).astype(np.float32)
    cfg = b.make_config(b.F16, T, B, D, R, 256, 12, b.FLAG_SAMPLE_CODEBOOK)
    ctx = b.Context(cfg)
    ctx.set_error_bounds(eb=ebs)
    cap = b.dlc_compress_bound(cfg)
    out = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")
    assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
    sz = sizes.cpu().numpy().astype(np.uint64)
    rec = torch.empty_like(d)
    assert ctx.decompress(out, int(sz[0]), rec) == 0 and ctx.sync_status() == 0
    x = d.cpu().numpy()
    print("oracle at full size", flush=True)
    o = oracle.compress(x, ebs, R, 256, 12, sample_codebook=True)
    assert o.rc == 0 and o.data.size == int(sz[0]) and np.array_equal(o.sizes, sz)
    assert np.array_equal(o.data, out[:int(sz[0])].cpu().numpy())
    rc, orec = oracle.decompress(o.data, x.shape, np.float16)
    assert rc == 0 and np.array_equal(rec.cpu().numpy().view(np.uint16), orec.view(np.uint16))
