"""GPU: ps_push_noalloc (the push that allocates nothing: fixed scratch array in device memory) against ps_push
on a twin server, through the C ABI: the stored values must be the same bit for bit (same kernels, other
scratch), the owner map and every counter equal - on two calls in a row, the second with fewer keys, which finds
the first call's contents in the scratch.  Both orders of push; sizes beyond the limit are refused and change
nothing."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _zipf_keys(rng, K, n, s=1.1):
    p = np.arange(1, K + 1, dtype=np.float64) ** -s
    p /= p.sum()
    return rng.permutation(K)[rng.choice(K, size=n, p=p)].astype(np.int64)


@pytest.mark.parametrize("K,L,W,sequential,sizes", [(5000, 100, 4, 0, (50000, 3000)), (5000, 100, 4, 1, (20000, 700)),
                                                    (500600, 400, 8, 0, (106496, 4097)), (777, 130, 7, 0, (262144, 65)),
                                                    (64, 1, 1, 0, (1000, 1))])
def test_push_noalloc_equals_push(K, L, W, sequential, sizes):
    import torch
    from paper_2002_00655_amd import ps as P
    print(f"case K={K} L={L} W={W} sequential={sequential} sizes={sizes}", flush=True)
    rng = np.random.default_rng(K + L)
    dev = torch.device("cuda")
    a, b = P.ParameterServer(K, L, W), P.ParameterServer(K, L, W)
    for s in (a, b):
        s.set_option(P.OPT_PUSH_SEQUENTIAL, sequential)
    all_keys = torch.arange(K, device=dev)
    init = torch.from_numpy(rng.standard_normal((K, L)).astype(np.float32)).to(dev) if K * L <= 10 ** 7 else None
    if init is not None:
        a.push(all_keys, init)
        b.push(all_keys, init)
    some = torch.from_numpy(rng.integers(0, K, size=min(K, 300))).to(dev)
    a.localize(some, W - 1)
    b.localize(some, W - 1)
    for n in sizes:
        keys = _zipf_keys(rng, K, n) if K <= 10 ** 4 else rng.integers(0, K, size=n)
        kt = torch.from_numpy(np.ascontiguousarray(keys)).to(dev)
        deltas = torch.from_numpy(rng.standard_normal((n, L)).astype(np.float32)).to(dev)
        worker = int(rng.integers(0, W))
        a.push(kt, deltas, worker)
        b.push_noalloc(kt, deltas, worker)
        va, vb = a.pull(all_keys).cpu().numpy(), b.pull(all_keys).cpu().numpy()
        assert np.array_equal(va.view(np.uint32), vb.view(np.uint32)), f"values differ after a call with {n} keys"
        assert a.stats() == b.stats()
        assert torch.equal(a.owner(), b.owner())
    a.status()
    b.status()


def test_push_noalloc_limits():
    import torch
    from paper_2002_00655_amd import ps as P
    dev = torch.device("cuda")
    srv = P.ParameterServer(1000, 1024, 2)
    before = srv.pull(torch.arange(1000, device=dev)).cpu().numpy()
    # too many keys
    n = 262145
    with pytest.raises(P.PSError) as e:
        srv.push_noalloc(torch.zeros(n, dtype=torch.int64, device=dev), torch.ones((n, 1024), device=dev), 0)
    assert e.value.code == P.PS_ELIMIT
    # few enough keys, but too many partial sums: ceil(n / 64) * value_len > 2^20
    n = 64 * 1024 + 1
    with pytest.raises(P.PSError) as e:
        srv.push_noalloc(torch.zeros(n, dtype=torch.int64, device=dev), torch.ones((n, 1024), device=dev), 0)
    assert e.value.code == P.PS_ELIMIT
    assert np.array_equal(srv.pull(torch.arange(1000, device=dev)).cpu().numpy(), before)
    assert srv.stats()["push_local"] == 0 and srv.stats()["push_remote"] == 0
    # at the limit it works
    n = 64 * 1024
    keys = torch.arange(n, device=dev) % 1000
    srv.push_noalloc(keys, torch.ones((n, 1024), device=dev), 0)
    got = srv.pull(torch.arange(1000, device=dev)).cpu().numpy()
    counts = np.bincount(np.arange(n) % 1000, minlength=1000).astype(np.float32)
    assert np.array_equal(got, np.repeat(counts[:, None], 1024, axis=1))
    srv.status()
