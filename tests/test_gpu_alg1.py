"""Algorithm 1 on the GPU (galv_alg1_reduce + the windowed driver) against oracle/alg1.py."""
import struct
from fractions import Fraction

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

INF = 1 << 62


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    from oracle import alg1 as oracle_alg1
    from paper_2211_13878_amd import alg1, binding, workloads
    oracle.build()
    binding.load_library()
    torch.cuda.set_device(0)
    return dict(oracle_alg1=oracle_alg1, alg1=alg1, binding=binding, workloads=workloads)


def _reduce_expected(blocks, degrees, batch_sizes, base, state):
    """Sums, minimum and scan written out with Python integers."""
    n = len(batch_sizes)
    c_p = [[INF] * len(degrees) for _ in range(n)]
    for ip, pp in enumerate(degrees):
        for ib in range(n):
            vals = [int(v) for v in blocks[ip][ib]]
            c_p[ib][ip] = INF if any(v >= INF for v in vals) or sum(vals) >= INF else sum(vals)
    bsz, cost, pidx, bidx, stopped, nexp = state
    for ib in range(n):
        if stopped:
            break
        c_opt = min(c_p[ib])
        if c_opt >= INF:
            stopped = 1
            break
        nexp += 1
        if batch_sizes[ib] * cost > bsz * c_opt:
            bsz, cost, pidx, bidx = batch_sizes[ib], c_opt, c_p[ib].index(c_opt), base + ib
    return c_p, (bsz, cost, pidx, bidx, stopped, nexp)


@pytest.mark.parametrize("seed", range(6))
def test_reduce_kernel_chained_windows(env, seed):
    b = env["binding"]
    rng = np.random.default_rng(seed)
    degrees = [1, 2, 4, 8][: int(rng.integers(1, 5))]
    state_dev = torch.zeros(b.ALG1_STATE_BYTES, dtype=torch.uint8, device="cuda")
    state = (0, 1, -1, -1, 0, 0)
    base = 0
    for w in range(4):
        n = int(rng.integers(1, 40))
        big = seed == 5
        blocks = [rng.integers(1, (1 << 60) if big else 10_000, size=(n, pp)).astype(np.int64) for pp in degrees]
        p_inf = 0.02 if w < 2 else 0.3
        for blk in blocks:
            blk[rng.random(blk.shape) < p_inf] = INF
        if seed == 0 and w == 0:
            blocks[0][0, 0] = 0
        sizes = sorted(int(x) for x in rng.integers(1, 500, size=n))
        stage_cost = torch.from_numpy(np.concatenate([blk.reshape(-1) for blk in blocks])).cuda()
        c_p = torch.empty((n, len(degrees)), dtype=torch.int64, device="cuda")
        b.galv_alg1_reduce(degrees, stage_cost, torch.tensor(sizes, dtype=torch.int64, device="cuda"),
                           base, w == 0, c_p, state_dev)
        exp_cp, state = _reduce_expected(blocks, degrees, sizes, base, state)
        assert c_p.cpu().numpy().tolist() == exp_cp
        got = struct.unpack("<qqiiii", state_dev.cpu().numpy().tobytes())
        assert got == state, (w, got, state)
        base += n


def test_reduce_argument_errors(env):
    b = env["binding"]
    st = torch.zeros(b.ALG1_STATE_BYTES, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(3, dtype=torch.int64, device="cuda")
    bs = torch.ones(1, dtype=torch.int64, device="cuda")
    cp = torch.zeros((1, 2), dtype=torch.int64, device="cuda")
    with pytest.raises(b.GalvError) as e:
        b.galv_alg1_reduce([1, 0], sc[:1], bs, 0, True, cp, st)
    assert e.value.code == b.GALV_ERR_INVALID_ARG
    with pytest.raises(b.GalvError):
        b.galv_alg1_reduce([1] * 17, torch.zeros(17, dtype=torch.int64, device="cuda"), bs, 0, True,
                           torch.zeros((1, 17), dtype=torch.int64, device="cuda"), st)


def _compare(env, model, n_devices, budget, batch_sizes, window):
    exp = env["oracle_alg1"].optimize(model, n_devices, budget, batch_sizes)
    got = env["alg1"].optimize(model, n_devices, budget, batch_sizes, window=window)
    assert got.c_p.tolist() == exp["c_p"]
    assert (got.throughput, got.batch, got.pp, got.cost) == (exp["tpt"], exp["batch"], exp["pp"], exp["cost"])
    assert got.plans == exp["plans"]
    assert (got.n_explored, got.stopped) == (exp["n_explored"], exp["stopped"])
    return got


@pytest.mark.parametrize("n_layers,n_devices,budget,window", [
    (24, 8, 3000, 8), (24, 8, 3000, 5), (10, 8, 1500, 8), (3, 8, 1200, 4), (7, 4, 900, 3), (12, 2, 1500, 16),
    (6, 1, 1000, 8)])
def test_driver_matches_oracle(env, n_layers, n_devices, budget, window):
    counts = env["alg1"].strategy_counts(n_devices)
    assert counts == env["oracle_alg1"].strategy_counts(n_devices)
    model = env["workloads"].Alg1Model(100 + n_layers, n_layers, n_devices, counts)
    got = _compare(env, model, n_devices, budget, range(1, 400), window)
    assert got.stopped and got.n_explored >= 3 and got.throughput > 0


def test_driver_runs_out_of_batch_sizes_and_never_fits(env):
    counts = env["alg1"].strategy_counts(8)
    model = env["workloads"].Alg1Model(5, 16, 8, counts)
    got = _compare(env, model, 8, 3000, [1, 2, 3, 5, 8, 13], 4)       # ends inside a short window
    assert not got.stopped and got.n_explored == 6
    got = _compare(env, model, 8, 10, range(1, 20), 8)                # nothing fits at B = 1
    assert got.stopped and got.n_explored == 0 and got.throughput == Fraction(0) and got.plans is None
    got = _compare(env, model, 8, 3000, [], 8)
    assert got.n_explored == 0 and not got.stopped
