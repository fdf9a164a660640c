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


def check_handoff_order(order):
    """The order an epoch with hand-over reports, int32 [d_row, d_col, 2] of (column block, workers that had it
    before): every worker has every column block once, and the visit numbers of a column block are 0 .. d_row-1."""
    order = np.asarray(order)
    d_row, d_col, _ = order.shape
    for w in range(d_row):
        assert np.array_equal(np.sort(order[w, :, 0]), np.arange(d_col)), f"worker {w}: {order[w, :, 0]}"
    for c in range(d_col):
        visits = order[:, :, 1][order[:, :, 0] == c]
        assert np.array_equal(np.sort(visits), np.arange(d_row)), f"column block {c}: {visits}"


def replay_schedule(order, rng=None):
    """Strata for mf_sgd_epoch that agree with a reported order: task (w, w, c) comes after worker w's previous task
    and after the previous visit of column block c.  Without rng: the earliest stratum for every task (tasks of a
    stratum then share no worker and no block).  With rng: one task per stratum, a random sequence that respects
    both orders."""
    order = np.asarray(order)
    d_row, d_col, _ = order.shape
    step_of = {}                                       # (column block, visit) -> (worker, step)
    for w in range(d_row):
        for s in range(d_col):
            step_of[(int(order[w, s, 0]), int(order[w, s, 1]))] = (w, s)
    if rng is None:
        level = np.zeros((d_row, d_col), dtype=np.int64)
        col_level = {}
        # visits of a column block in increasing order need the levels of earlier visits: go by (visit, worker)
        todo = sorted(step_of.items(), key=lambda kv: (kv[0][1], kv[1][0]))
        pending = list(todo)
        while pending:                                 # a few sweeps until all predecessors are known
            rest = []
            for (c, v), (w, s) in pending:
                ok_w = s == 0 or level[w, s - 1] > 0
                ok_c = v == 0 or (c, v - 1) in col_level
                if ok_w and ok_c:
                    lv = 1 + max(level[w, s - 1] if s else 0, col_level[(c, v - 1)] if v else 0)
                    level[w, s] = lv
                    col_level[(c, v)] = lv
                else:
                    rest.append(((c, v), (w, s)))
            assert len(rest) < len(pending), "the reported order has a cycle"
            pending = rest
        strata = []
        for lv in range(1, int(level.max()) + 1):
            ws, ss = np.nonzero(level == lv)
            strata.append(np.stack([ws, ws, order[ws, ss, 0]], axis=1).astype(np.int32))
        return strata
    done_w = np.zeros(d_row, dtype=np.int64)           # steps finished per worker
    done_c = np.zeros(d_col, dtype=np.int64)           # visits finished per column block
    strata = []
    while len(strata) < d_row * d_col:
        ready = [w for w in range(d_row) if done_w[w] < d_col and order[w, done_w[w], 1] == done_c[order[w, done_w[w], 0]]]
        assert ready, "the reported order has a cycle"
        w = int(rng.choice(ready))
        c = int(order[w, done_w[w], 0])
        strata.append(np.array([[w, w, c]], dtype=np.int32))
        done_w[w] += 1
        done_c[c] += 1
    return strata


def simulate_handoff(d_row, d_col, rng):
    """An order as an epoch with hand-over could report it, from block durations drawn at random: worker w keeps row
    block w; a worker that finishes gives its column block back and takes the first free one, in cyclic order after
    the one it had, that it has not had yet (first look: floor(w d_col / d_row))."""
    order = np.full((d_row, d_col, 2), -1, dtype=np.int32)
    held = np.zeros(d_col, dtype=bool)
    visits = np.zeros(d_col, dtype=np.int64)
    had = np.zeros((d_row, d_col), dtype=bool)
    start = [(w * d_col) // d_row for w in range(d_row)]
    step = np.zeros(d_row, dtype=np.int64)
    busy_until = np.zeros(d_row)                       # a worker with no block has busy_until = its waiting time
    holding = np.full(d_row, -1)
    now = 0.0
    while (step < d_col).any() or (holding >= 0).any():
        # workers without a block try to take one, in random order
        for w in rng.permutation(d_row):
            if holding[w] >= 0 or step[w] >= d_col or busy_until[w] > now:
                continue
            for k in range(d_col):
                c = (start[w] + k) % d_col
                if not held[c] and not had[w, c]:
                    held[c] = True; had[w, c] = True; holding[w] = c
                    order[w, step[w]] = (c, visits[c])
                    step[w] += 1
                    busy_until[w] = now + rng.uniform(0.5, 2.0)
                    break
        running = [w for w in range(d_row) if holding[w] >= 0]
        if not running:
            now += 0.1
            continue
        w = min(running, key=lambda x: busy_until[x])
        now = max(now, busy_until[w])
        c = holding[w]
        held[c] = False; visits[c] += 1; holding[w] = -1
        start[w] = (c + 1) % d_col
    return order
