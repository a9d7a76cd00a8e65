"""dlc_decompress_static (the entry point that allocates nothing) against dlc_decompress, through the C ABI."""
import numpy as np
import pytest

import oracle
from gpu_util import to_device

pytestmark = pytest.mark.gpu

R = 512


def _container(x, ebs, S, flags=0, num_dest=1):
    import torch
    from paper_2407_04272_amd import binding as b
    T, B, D = x.shape
    dt = b.F16 if x.dtype == np.float16 else b.F32
    cfg = b.make_config(dt, T // num_dest, B, D, R, S, 12, flags, num_dest)
    ctx = b.Context(cfg)
    cap = b.dlc_compress_bound(cfg)
    d = to_device(x)
    out = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T + (num_dest if num_dest > 1 else 0), dtype=torch.int64, device="cuda")
    ctx.set_error_bounds(eb=ebs)
    assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
    nbytes = cap if num_dest > 1 else int(sizes[0].item())
    return cfg, ctx, d, out, nbytes


def _both_ways(cfg, ctx, d, out, nbytes, expect=0):
    import torch
    from paper_2407_04272_amd import binding as b
    rec0 = torch.full_like(d, 7.0)
    rec1 = torch.full_like(d, 7.0)
    status = torch.full((1,), 99, dtype=torch.int32, device="cuda")
    assert ctx.decompress(out, nbytes, rec0) == 0
    assert ctx.sync_status() == expect
    assert b.dlc_decompress_static(cfg, out, nbytes, rec1, status) == 0
    torch.cuda.synchronize()
    assert int(status.item()) == expect
    u = torch.int32 if d.dtype == torch.float32 else torch.int16
    if expect == 0:
        assert torch.equal(rec0.view(u), rec1.view(u))
    return rec1


def _lookups(T, B, D, seed, dtype):
    rng = np.random.default_rng(seed)
    table = (rng.standard_normal((T, 40, D)) * 0.03).astype(np.float32)
    idx = rng.integers(0, 40, (T, B))
    return np.stack([table[t][idx[t]] for t in range(T)]).astype(dtype)


def test_two_calls_in_a_row_the_second_smaller():
    from paper_2407_04272_amd import binding as b
    for (T, B, D, S, dtype, flags) in ((6, 3000, 32, 256, np.float32, 0), (3, 130, 16, 64, np.float32, 0),
                                         (4, 700, 40, 128, np.float16, b.FLAG_ROW_MATCH), (2, 70, 8, 64, np.float16, 0)):
        print("no-alloc decompress", T, B, D, S, np.dtype(dtype).name, flags, flush=True)
        x = _lookups(T, B, D, 5 * T + B, dtype)
        x[0, 1, 2] = 3.0e4                                  # an escape
        ebs = np.full(T, 2e-3 if dtype == np.float32 else 8e-3, np.float32)
        cfg, ctx, d, out, nbytes = _container(x, ebs, S, flags)
        rec = _both_ways(cfg, ctx, d, out, nbytes)
        o = oracle.compress(x, ebs, R, S, 12, row_match=bool(flags))
        rc, orec = oracle.decompress(o.data, x.shape, x.dtype)
        u = np.uint32 if dtype == np.float32 else np.uint16
        assert rc == 0 and np.array_equal(rec.cpu().numpy().view(u), orec.view(u))


def test_several_destinations():
    x = _lookups(8, 900, 16, 77, np.float32)
    ebs = np.full(2, 1e-3, np.float32)
    cfg, ctx, d, out, nbytes = _container(x, ebs, 128, num_dest=4)
    _both_ways(cfg, ctx, d, out, nbytes)


def test_a_bad_container_is_reported_and_the_next_call_is_clean():
    import torch
    from paper_2407_04272_amd import binding as b
    x = _lookups(5, 2000, 32, 9, np.float32)
    ebs = np.full(5, 1e-3, np.float32)
    cfg, ctx, d, out, nbytes = _container(x, ebs, 256)
    bad = out.clone()
    bad[128 + 16:128 + 20] = torch.tensor([200, 0, 0, 0], dtype=torch.uint8)   # the directory claims escapes the payload lacks
    _both_ways(cfg, ctx, d, bad, nbytes, expect=b.ECORRUPT)
    hdr = out.clone()
    hdr[0] ^= 1                                             # not a container at all
    _both_ways(cfg, ctx, d, hdr, nbytes, expect=b.ECORRUPT)
    _both_ways(cfg, ctx, d, out, nbytes)                    # (what the bad calls left behind does not matter)


def test_limits_and_arguments():
    import torch
    from paper_2407_04272_amd import binding as b
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    big = b.make_config(b.F32, b.STATIC_MAX_TABLES + 1, 8, 4, R, 64, 12)
    rec = torch.zeros((b.STATIC_MAX_TABLES + 1) * 32, dtype=torch.float32, device="cuda")
    assert b.dlc_decompress_static(big, buf, buf.numel(), rec, status) == b.ELIMIT
    assert "maximum" in b.dlc_strerror(b.ELIMIT)
    ok = b.make_config(b.F32, 4, 8, 4, R, 64, 12)
    small = torch.zeros(8, dtype=torch.float32, device="cuda")
    assert b.dlc_decompress_static(ok, buf, buf.numel(), small, status) == b.ECAPACITY
    assert b.dlc_decompress_static(ok, buf, 64, rec, status) == b.ECORRUPT
    torch.cuda.synchronize()


def test_decompress_under_graph_capture():
    """Both decompress entry points recorded into a HIP graph (they keep no per-call state on the host and allocate
    nothing) and replayed with other containers in the same buffer: every replay against the eager result."""
    import torch
    from paper_2407_04272_amd import binding as b
    T, B, D, S = 4, 1500, 32, 128
    ebs = np.full(T, 2e-3, np.float32)
    payloads = [_lookups(T, B, D, 31 + k, np.float32) for k in range(3)]
    cfg = b.make_config(b.F32, T, B, D, R, S, 12)
    ctx = b.Context(cfg)
    ctx.set_error_bounds(eb=ebs)
    cap = b.dlc_compress_bound(cfg)
    out = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    sizes = torch.zeros(1 + T, dtype=torch.int64, device="cuda")
    rec0 = torch.zeros((T, B, D), dtype=torch.float32, device="cuda")
    rec1 = torch.zeros_like(rec0)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    d = to_device(payloads[0])
    assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        # once outside the capture: the first call on a device looks up the fixed array's address
        assert ctx.decompress(out, cap, rec0) == 0 and b.dlc_decompress_static(cfg, out, cap, rec1, status) == 0
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            assert ctx.decompress(out, cap, rec0) == 0
            assert b.dlc_decompress_static(cfg, out, cap, rec1, status) == 0
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for k, x in enumerate(payloads):
        d = to_device(x)                                                  # eager work between the replays
        assert ctx.compress(d, out, sizes, capacity=cap) == 0 and ctx.sync_status() == 0
        want = torch.zeros_like(rec0)
        assert ctx.decompress(out, cap, want) == 0 and ctx.sync_status() == 0
        rec0.fill_(7.0)
        rec1.fill_(7.0)
        status.fill_(99)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert ctx.sync_status() == 0 and int(status.item()) == 0, k
        assert torch.equal(rec0.view(torch.int32), want.view(torch.int32)), k
        assert torch.equal(rec1.view(torch.int32), want.view(torch.int32)), k
        o = oracle.compress(x, ebs, R, S, 12)
        rc, orec = oracle.decompress(o.data, x.shape, np.float32)
        assert rc == 0 and np.array_equal(want.cpu().numpy().view(np.uint32), orec.view(np.uint32)), k
