"""GPU parity of the kernel variants and grid decompositions that the launch heuristics do not pick at the shapes of the
other tests.  The test hook pamm_debug_set_plan forces them in-process; every forced configuration must give what
the fp64 oracle gives, at the bars of tests/test_gpu_parity.py:

  score kernel   every legal pair (generator fragments per wave, waves per workgroup), on a row length that is a
                 whole number of 128-byte windows and on one that is not, with one column block (the kernel decides
                 itself) and with several (records merged by the finalize kernel), both element types, with and
                 without the tolerance of Eq. 2
  contraction    512-column groups per wave 1..3, chunks of 16 / 64 / 4096 list positions, and the two counting sorts
                 (one workgroup; histogram + scatter) on the same batch -- all must give bit-identical sums, because the
                 sorted list does not depend on the decomposition and a generator's rows are summed in list order only
                 within a chunk (chunk boundaries move the partial sums, so across chunk sizes the bar is the oracle's)
  near-ties on rows that are nearly orthogonal to every generator (best |cosine| about 0.07 and 0.02), where the
                 fp32 score carries the largest relative error: f must be the fp64 decision down to the 1e-6 bar
"""
import itertools

import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads

pytestmark = pytest.mark.gpu

ELEM_ALPHA = 1e-5                                      # measured worst 2.9e-6 (rows of 16384 fp32 elements)
ELEM_BT = 5e-6                                         # measured worst 5.7e-7
ELEM_DW = {"f32": 5e-6, "bf16": 2.0 ** -8 + 5e-6}      # measured worst 6.9e-7 / 2.4e-3; 2^-8 is bf16's unit roundoff


@pytest.fixture(scope="module")
def pamm():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2506_02939_amd import pamm as p

    yield p
    p.debug_set_plan()


def _gap(ora):
    return np.where(ora.best > 0, (ora.best - ora.second) / np.where(ora.best > 0, ora.best, 1.0), 0.0)


def _check_compress(ora, got, eps):
    f = got.f.cpu().numpy()
    a = got.alpha.cpu().numpy().astype(np.float64)
    sure = _gap(ora) >= 1e-6
    assert np.array_equal(f[sure], ora.f[sure]), f"{int(np.sum(f[sure] != ora.f[sure]))} rows differ outside near-ties"
    same = f == ora.f
    if eps is not None:          # rows within 1e-6 ||X_i|| of the limit of Eq. 2 may fall either way
        lim = eps * ora.rownorm
        same &= np.abs(ora.resid - lim) > 1e-6 * ora.rownorm
        assert int(got.eta.item()) == ora.eta or not np.all(np.abs(ora.resid - lim) > 1e-6 * ora.rownorm)
    cnorm = np.sqrt((ora.C ** 2).sum(axis=1))
    with np.errstate(divide="ignore", invalid="ignore"):
        bound = np.where(cnorm[ora.f] > 0, ora.rownorm / cnorm[ora.f], 0.0)
    err = np.abs(a - ora.alpha)[same]
    assert np.all(err <= ELEM_ALPHA * bound[same] + 0.0), f"alpha off by {np.max(err / np.maximum(bound[same], 1e-300))}"


# ------------------------------------------------------------------------------------------ score kernel variants

SCORE_K = [24, 40, 100, 200, 300]          # widest block: 1, 2, 4, 8, 8 fragments; narrower ones give 2 .. 10 column blocks


def _score_cases():
    out = []
    for dn, n in (("bf16", 192), ("bf16", 200), ("f32", 96), ("f32", 100)):     # whole windows / a ragged last window
        for k in SCORE_K:
            out.append((dn, n, k))
    return out


@pytest.mark.parametrize("dn,n,k", _score_cases(), ids=[f"{c[0]}_n{c[1]}_k{c[2]}" for c in _score_cases()])
def test_every_score_kernel_variant(pamm, oracle, dn, n, k):
    base = "llama60m" if dn == "bf16" else "tiny"          # the bf16 recipe has bit-identical padding rows
    w = workloads.scaled(workloads.WORKLOADS[base], name="variants", seqs=3, seq_len=233, n=n, m=8, k=k, centres=max(8, k // 2))
    X, _ = workloads.generate(w)
    Xg = X.cuda()
    tg_max = 1
    while tg_max < 8 and 32 * tg_max < k:
        tg_max *= 2
    for eps in (None, 0.35):
        ora = oracle.compress(X, k, seed=4, eps=float("inf") if eps is None else eps)
        for tg, nw in itertools.product([t for t in (1, 2, 4, 8) if t <= tg_max], (2, 4, 8)):
            print(f"[variant] {dn} n={n} k={k} eps={eps} fragments/wave={tg} waves={nw} "
                  f"blocks={-(-k // (32 * tg))}", flush=True)
            pamm.debug_set_plan(score_tg=tg, score_nw=nw)
            try:
                got = pamm.compress(Xg, k, seed=4, eps=eps)
                torch.cuda.synchronize()
            finally:
                pamm.debug_set_plan()
            _check_compress(ora, got, eps)


# ------------------------------------------------------------------------------------------ contraction decompositions

@pytest.mark.parametrize("dn,m,k", [("bf16", 1544, 7), ("bf16", 5000, 70), ("f32", 1028, 33), ("bf16", 520, 2100)],
                         ids=["bf16_m1544_k7", "bf16_m5000_k70", "f32_m1028_k33", "bf16_m520_k2100"])
def test_contraction_decompositions_agree(pamm, oracle, dn, m, k):
    b, n = 9001, 64
    g = torch.Generator().manual_seed(77 + k)
    dt = torch.bfloat16 if dn == "bf16" else torch.float32
    C = torch.randn(k, n, generator=g).to(dt)
    dY = (0.1 * torch.randn(b, m, generator=g)).to(dt)
    # skewed group sizes, like padding rows that all map to one generator, and some rows with no weight
    f = torch.randint(0, k, (b,), generator=g, dtype=torch.int32)
    f[torch.rand(b, generator=g) < 0.3] = k // 2
    alpha = torch.rand(b, generator=g) + 0.5
    alpha[torch.rand(b, generator=g) < 0.1] = 0.0
    Bt_or, O_or = oracle.grad(oracle.to_f64(C), f.numpy(), alpha.numpy().astype(np.float64), dY)
    Bt_abs, O_abs = oracle.grad(np.abs(oracle.to_f64(C)), f.numpy(), alpha.numpy().astype(np.float64), dY.abs())
    Cg, fg, ag, dYg = C.cuda(), f.cuda(), alpha.cuda(), dY.cuda()
    by_chunk = {}
    for W, P, S in itertools.product((1, 2, 3), (0, 16, 64, 4096), (1, 16384)):
        print(f"[decomposition] {dn} m={m} k={k} column groups/wave={W} chunk={P or 'auto'} one-workgroup sort up to {S} rows",
              flush=True)
        pamm.debug_set_plan(contract_w=W, piece_rows=P, sort_one_rows=S)
        try:
            Bt = pamm.contract(fg, ag, dYg, k)
            dW = pamm.grad(Cg, fg, ag, dYg)
            torch.cuda.synchronize()
        finally:
            pamm.debug_set_plan()
        e_bt = np.abs(Bt.cpu().numpy().astype(np.float64) - Bt_or)
        e_dw = np.abs(dW.cpu().numpy().astype(np.float64) - O_or)
        assert np.all(e_bt <= ELEM_BT * Bt_abs), f"Btilde off by {np.max(e_bt / np.maximum(Bt_abs, 1e-300))}"
        assert np.all(e_dw <= ELEM_DW[dn] * O_abs), f"dW off by {np.max(e_dw / np.maximum(O_abs, 1e-300))}"
        # same chunk size: column groups per wave and the kind of counting sort must not change a single bit
        ref = by_chunk.setdefault((P, W if P == 0 else 0), (Bt.clone(), dW.clone()))      # auto chunks follow W
        assert torch.equal(Bt, ref[0]) and torch.equal(dW, ref[1]), "the decomposition changed the sums"


def test_sorted_list_is_in_increasing_row_order_within_each_generator(pamm):
    """The grouping is stable: behind the call, the workspace starts with the sorted list (16-byte entries: row number,
    weight bits, generator, 0), followed at the next 256-byte boundary after b + 16 entries by its length.  Checked for
    the one-workgroup sort, histogram + scatter, and the per-generator grouping kernels."""
    g = torch.Generator().manual_seed(5)
    for b, k, sort_one in ((6000, 37, 16384), (6000, 37, 1), (70001, 300, 1), (5000, 2100, 1)):
        m = 16
        f = torch.randint(0, k, (b,), generator=g, dtype=torch.int32)
        f[torch.rand(b, generator=g) < 0.4] = 3
        alpha = torch.rand(b, generator=g) + 0.5
        alpha[torch.rand(b, generator=g) < 0.2] = 0.0
        dY = torch.randn(b, m, generator=g).to(torch.bfloat16)
        pamm.debug_set_plan(sort_one_rows=sort_one)
        try:
            ws = torch.zeros(pamm.grad_workspace(b, 8, k, m, pamm.PAMM_BF16), dtype=torch.uint8, device="cuda")
            pamm.contract(f.cuda(), alpha.cuda(), dY.cuda(), k, ws=ws)
            torch.cuda.synchronize()
        finally:
            pamm.debug_set_plan()
        raw = ws.cpu().numpy()
        hdr_off = ((b + 16) * 16 + 255) // 256 * 256
        L = int(raw[hdr_off:hdr_off + 4].view(np.int32)[0])
        live = (alpha != 0).numpy()
        assert L == int(live.sum())
        ent = raw[:L * 16].view(np.int32).reshape(L, 4)
        rows, keys = ent[:, 0], ent[:, 2]
        assert np.all(np.diff(keys) >= 0), "the list is not sorted by generator"
        assert np.all((np.diff(rows) > 0) | (np.diff(keys) > 0)), "rows of one generator are not in increasing order"
        assert np.array_equal(np.sort(rows), np.nonzero(live)[0]) and np.array_equal(keys, f.numpy()[rows])
        assert np.array_equal(np.ascontiguousarray(ent[:, 1]).view(np.float32), alpha.numpy()[rows])


# ------------------------------------------------------------------------------------------ near-ties on low-score rows

@pytest.mark.parametrize("dn,n,cos", [("f32", 4096, 0.07), ("bf16", 4096, 0.07), ("f32", 8192, 0.07), ("bf16", 8192, 0.07),
                                      ("f32", 8192, 0.02), ("bf16", 8192, 0.02)],
                         ids=lambda v: str(v))
def test_near_ties_on_rows_far_from_every_generator(pamm, oracle, dn, n, cos):
    """Rows whose best |cosine| is only `cos` (the rest of the row is orthogonal to every generator) and whose two best
    generators score within 1e-4 .. 1e-7 of each other.  Here the fp32 score's relative error is largest (the dot
    product is a small difference of large terms), so this is where a too narrow second-look band would show."""
    g = torch.Generator().manual_seed(31 + n)
    k, rows_n = 12, 3000
    G = torch.randn(k, n, generator=g, dtype=torch.float64)
    Q, _ = torch.linalg.qr(G.T)                       # orthonormal generators: the designed scores are exact
    G = Q.T.contiguous()
    rows = [G[j].clone() for j in range(k)]
    for rep in range(rows_n):
        ja, jb = torch.randperm(k, generator=g)[:2].tolist()
        delta = 10.0 ** (-4 - 3 * torch.rand(1, generator=g, dtype=torch.float64).item())
        wv = torch.randn(n, generator=g, dtype=torch.float64)
        wv -= G.T @ (G @ wv)                          # orthogonal to every generator
        wv /= wv.norm()
        rows.append(cos * ((1 + delta) * G[ja] + (1 - delta) * G[jb]) / 2 ** 0.5 + wv)
    dt = torch.float32 if dn == "f32" else torch.bfloat16
    X = torch.stack(rows).to(dt)
    ora = oracle.compress(X, k, idx=np.arange(k, dtype=np.int32))
    gap = _gap(ora)[k:]
    best_cos = np.sqrt(ora.best[k:]) / ora.rownorm[k:]
    assert np.median(best_cos) < 1.5 * cos
    close = int(np.sum((gap >= 1e-6) & (gap < 2.0 ** -12)))
    assert close >= 30, f"only {close} rows ended up between the 1e-6 bar and the fp32 band"     # rounding to dt moves the gaps
    got = pamm.compress(X.cuda(), k, idx=torch.arange(k, dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    f = got.f.cpu().numpy()
    sure = _gap(ora) >= 1e-6
    wrong = int(np.sum(f[sure] != ora.f[sure]))
    print(f"[near-tie] {dn} n={n} cos={cos}: {close} rows between 1e-6 and 2^-12, {wrong} decided differently", flush=True)
    assert wrong == 0


# ------------------------------------------------------------------------------------------ the big tiles of C^T Btilde

@pytest.mark.parametrize("tile", ["256x128", "256x256"])
@pytest.mark.parametrize("form", ["f32", "bf16", "f32_m_by_n", "bf16_m_by_n"])
def test_big_tiles_of_the_small_product(pamm, oracle, form, tile):
    """At least 512 generators and a weight gradient of at least 512 blocks of 256 x 256: the product C^T Btilde takes
    the kernel built on the big-tile main loop, on 256 x 128 tiles (two workgroups per compute unit: what the library
    picks) and on 256 x 256 tiles (one; forced).  Ragged edges in both directions, 520 generators (padded to 544 with
    zero rows), all four output forms, against the oracle element by element."""
    w = workloads.scaled(workloads.WORKLOADS["llama7b_k1024"], name="big_tiles", seqs=2, seq_len=1024, n=4000, m=8200, k=520, centres=300)
    X, dY = workloads.generate(w)
    got = pamm.compress(X.cuda(), w.k, seed=3)
    torch.cuda.synchronize()
    f = got.f.cpu().numpy()
    a = got.alpha.cpu().numpy().astype(np.float64)
    C64 = oracle.to_f64(got.C.cpu())
    _, O = oracle.grad(C64, f, a, dY)
    _, O_abs = oracle.grad(np.abs(C64), f, np.abs(a), dY.abs())
    kw = dict(out_dtype=torch.bfloat16 if form.startswith("bf16") else torch.float32, transposed=form.endswith("m_by_n"))
    pamm.debug_set_plan(small_tiles=2 if tile == "256x256" else 0)
    try:
        dW = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), **kw)
        torch.cuda.synchronize()
    finally:
        pamm.debug_set_plan()
    res = dW.float().cpu().numpy().astype(np.float64)
    if kw["transposed"]:
        res = res.T
    bar = ELEM_DW["bf16"] + (2.0 ** -8 if form.startswith("bf16") else 0.0)        # + one rounding of the result itself
    err = np.abs(res - O)
    assert np.all(err <= bar * O_abs + 1e-30), f"dW off by {np.max(err / np.maximum(O_abs, 1e-300))}"
    assert np.linalg.norm(err) <= (2.0 ** -8 + (2.0 ** -9 if form.startswith("bf16") else 0.0)) * np.linalg.norm(O)


# ------------------------------------------------------------------------------------------ nearly identical rows

def test_nearly_identical_rows_stay_correct_and_affordable(pamm, oracle):
    """The method's own regime taken to the extreme: every row is one centre plus noise of relative size 1e-4, no two
    rows bit-identical.  All generators are then nearly parallel, every token has every generator within the fp32 band
    of its best, and each token is decided in fp64 among all of them.  f must still be the oracle's wherever the oracle's
    two best scores are 1e-6 apart, alpha within the bar, and the call must stay within a small multiple of a second."""
    import time

    g = torch.Generator().manual_seed(23)
    b, n, k = 4096, 512, 24
    centre = torch.randn(n, generator=g)
    X = (centre[None, :] * (1.0 + 0.5 * torch.rand(b, 1, generator=g)) + 1e-4 * centre.norm() / n ** 0.5 * torch.randn(b, n, generator=g))
    for dt in (torch.float32, torch.bfloat16):
        Xc = X.to(dt)
        ora = oracle.compress(Xc, k, seed=2)
        Xg = Xc.cuda()
        pamm.compress(Xg, k, seed=2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        got = pamm.compress(Xg, k, seed=2)
        torch.cuda.synchronize()
        dt_s = time.perf_counter() - t0
        _check_compress(ora, got, None)
        crowded = float(np.mean(_gap(ora) < 2.0 ** -12))
        print(f"[near-duplicates] {dt}: {crowded:.2f} of the rows within the fp32 band, compress took {dt_s * 1e3:.2f} ms", flush=True)
        assert dt_s < 0.5
