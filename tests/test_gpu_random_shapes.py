"""A seeded sweep of small random geometries through every compress path, each against the oracle byte for byte."""
import numpy as np
import pytest

import oracle
from gpu_util import to_device

pytestmark = pytest.mark.gpu



def _one(rng, k, large=False, force_mode=None):
    import torch
    from paper_2407_04272_amd import binding as b
    T = int(rng.integers(1, 7))
    B = int(rng.choice([1, 3, 17, 64, 130, 257, 700, 2100]))
    D = int(rng.choice([1, 4, 7, 16, 20, 48, 64, 132]))
    S = int(rng.choice([64, 128, 256]))
    R, LMAX = 512, 12
    if large:  # many groups per table (several items per work-group), many tables, other alphabets and code lengths
        T = int(rng.choice([2, 9, 40, 530]))
        B = int(rng.choice([4096, 20000])) if T < 100 else int(rng.choice([64, 300]))
        D = int(rng.choice([16, 64, 100]))
        R, LMAX = [(64, 8), (64, 12), (512, 10), (512, 12), (2048, 12)][int(rng.integers(0, 5))]
    f16 = bool(rng.integers(0, 2))
    mode = int(rng.integers(0, 3))           # 0 default, 1 single-pass chain, 2 row matching
    if force_mode is not None:
        mode = force_mode                    # 3: single pass with the codebook of a sample of the payload
    if mode == 2 and D % 4 != 0:
        mode = 0
    n = int(rng.choice([1, 1, 2, 3])) if mode != 2 or T * 3 <= 65535 else 1
    dtype = np.float16 if f16 else np.float32
    sigma = float(rng.choice([1e-3, 0.02, 0.5]))
    eb = np.float32(sigma * rng.choice([0.02, 0.1, 0.4, 3.0]) * (8.0 if f16 else 1.0))
    ebs = (eb * (1 + np.arange(T, dtype=np.float32) % 3)).astype(np.float32)
    print(f"random shape {k}: n={n} T={T} B={B} D={D} S={S} R={R} LMAX={LMAX} {np.dtype(dtype).name} mode={mode} eb={eb:g}", flush=True)
    flags = [0, b.FLAG_CARRY_CODEBOOK, b.FLAG_ROW_MATCH, b.FLAG_SAMPLE_CODEBOOK][mode]
    # what the next allocation gets is not zero: a context must not rely on fresh memory
    junk = torch.full((48 << 20,), 0xA5, dtype=torch.uint8, device="cuda")
    del junk
    torch.cuda.empty_cache()
    cfg = b.make_config(b.F16 if f16 else b.F32, T, B, D, R, S, LMAX, flags, num_dest=n)
    ctx = b.Context(cfg)
    ctx.set_error_bounds(eb=ebs)
    cap = b.dlc_compress_bound(cfg)
    stride = (cap // n) & ~255 if n > 1 else cap
    out = torch.zeros(cap + 64, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + n * T + (n if n > 1 else 0), dtype=torch.int64, device="cuda")
    prev = [None] * n
    for call in range({1: 3, 3: 2}.get(mode, 1)):  # (a context with a sampled codebook keeps nothing from call to call)
        rows = max(1, B // 3)
        table = (rng.standard_normal((n, T, rows, D)) * sigma).astype(np.float32)
        idx = rng.integers(0, rows, (n, T, B))
        x = np.take_along_axis(table, idx[..., None], axis=2).astype(dtype)     # repeated rows
        x.reshape(-1)[::int(rng.choice([53, 911, 7]))] = 6e4 if f16 else 1e9    # escapes: some, few, very many
        d = to_device(x if n > 1 else x[0])
        out.fill_(0xA5)
        assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
        h = out.cpu().numpy()
        sz = sizes.cpu().numpy().astype(np.uint64)
        assert np.all(h[cap:] == 0xA5)
        rec = torch.full_like(d, 7.0)
        assert ctx.decompress(out, cap if n > 1 else int(sz[0]), rec) == 0 and ctx.sync_status() == 0
        r = rec.cpu().numpy().reshape(x.shape)
        u = np.uint16 if f16 else np.uint32
        for p in range(n):
            o = oracle.compress(x[p], ebs, R, S, LMAX, carry_hist=prev[p] if mode == 1 else None,
                                want_hist=(mode == 1), row_match=(True if mode == 2 else None),
                                sample_codebook=(mode == 3))
            assert o.rc == 0
            nbytes = int(sz[1 + n * T + p]) if n > 1 else int(sz[0])
            got = h[p * stride:p * stride + nbytes]
            assert nbytes == o.data.size and np.array_equal(got, o.data), (k, call, p)
            rc, orec = oracle.decompress(o.data, x[p].shape, dtype)
            assert rc == 0 and np.array_equal(r[p].view(u), orec.view(u)), (k, call, p)
            if mode == 1:
                prev[p] = o.hist
        # the same container through the entry point that takes no context
        if n * T <= b.STATIC_MAX_TABLES:
            rec2 = torch.full_like(d, 7.0)
            status = torch.full((1,), 99, dtype=torch.int32, device="cuda")
            assert b.dlc_decompress_static(cfg, out, cap if n > 1 else int(sz[0]), rec2, status) == 0
            torch.cuda.synchronize()
            assert int(status.item()) == 0 and torch.equal(rec.view(torch.int16 if f16 else torch.int32),
                                                           rec2.view(torch.int16 if f16 else torch.int32)), (k, call)
        # the statistics of the same payload (one destination: a table's statistics are over its whole batch)
        if n == 1 and call == 0 and R == 512:
            st = ctx.stats(d, ebs)
            ost = oracle.stats(x[0], ebs)
            for t in range(T):
                a, c = st[t], ost[t]
                assert (a.n_unique_raw, a.n_unique_quant, a.n_rows) == (c.n_unique_raw, c.n_unique_quant, c.n_rows), (k, t)
                assert np.float32(a.min).view(np.uint32) == np.float32(c.min).view(np.uint32), (k, t)
                assert np.float32(a.max).view(np.uint32) == np.float32(c.max).view(np.uint32), (k, t)


def test_random_geometries():
    rng = np.random.default_rng(20240704)
    for k in range(150):
        _one(rng, k)


def test_random_larger_geometries():
    rng = np.random.default_rng(20240705)
    for k in range(24):
        _one(rng, k, large=True)


def test_random_geometries_sampled_codebook():
    rng = np.random.default_rng(20240706)
    for k in range(80):
        _one(rng, k, force_mode=3)


def test_random_larger_geometries_sampled_codebook():
    rng = np.random.default_rng(20240707)
    for k in range(14):
        _one(rng, k, large=True, force_mode=3)
