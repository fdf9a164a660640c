"""Helpers shared by the GPU parity tests: run one workload through the CPU
oracle and through the HIP library with the same seeded inputs."""
import numpy as np


def oracle_epochs(prec, w, rb, cb, blocked, schedule, epochs=1, lr=None, lam=None):
    from oracle.oracle import Oracle
    br, bc, bv, bp = blocked
    W = int(max(int(np.asarray(s)[:, 0].max()) for s in schedule)) + 1
    orc = Oracle(prec, w.m + w.n, w.rank, W)
    orc.push(np.arange(w.m), w.W0)
    orc.push(w.m + np.arange(w.n), w.H0)
    for _ in range(epochs):
        orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, schedule, w.lr if lr is None else lr, w.lam if lam is None else lam)
    return orc


def gpu_epochs(w, rb, cb, blocked, schedule, epochs=1, lr=None, lam=None, options=()):
    import torch
    from paper_2002_00655_amd import ps as P
    br, bc, bv, bp = blocked
    W = int(max(int(np.asarray(s)[:, 0].max()) for s in schedule)) + 1
    srv = P.ParameterServer(w.m + w.n, w.rank, W)
    for opt, value in options:
        srv.set_option(opt, value)
    dev = torch.device("cuda")
    srv.push(torch.arange(w.m, device=dev), torch.from_numpy(w.W0).to(dev))
    srv.push(w.m + torch.arange(w.n, device=dev), torch.from_numpy(w.H0).to(dev))
    srv.mf_load_ratings(w.m, w.n, torch.from_numpy(br).to(dev), torch.from_numpy(bc).to(dev), torch.from_numpy(bv).to(dev),
                        rb, cb, bp)
    for _ in range(epochs):
        srv.mf_sgd_epoch(schedule, w.lr if lr is None else lr, w.lam if lam is None else lam)
    srv.status()
    return srv


def gpu_values(srv):
    import torch
    return srv.pull(torch.arange(srv.K, device="cuda")).cpu().numpy()


def compare_state(orc, srv, exact, atol=1e-4):
    """Owner map and counters bit-exact; values bit-exact or within atol."""
    got, want = gpu_values(srv), orc.pull(np.arange(orc.K))
    assert np.array_equal(srv.owner().cpu().numpy(), orc.owner()), "owner map differs"
    assert srv.stats() == orc.stats(), (srv.stats(), orc.stats())
    if exact:
        bad = np.flatnonzero((got != want.astype(np.float32)).any(axis=1))
        assert bad.size == 0, f"{bad.size} keys differ, first {bad[:5]}"
    else:
        err = np.abs(got.astype(np.float64) - want.astype(np.float64)).max()
        print(f"  max abs difference to the oracle: {err:.3e}", flush=True)
        assert err <= atol, f"max abs difference {err}"
    return got, want
