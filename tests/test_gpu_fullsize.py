"""GPU parity at the benchmark's full sizes and launch configuration: sampled rows (all N columns)
against the oracle, plus properties that hold at any size.  Inputs are generated on the GPU by the
same seeded recipe the benchmark uses; the sampled rows are copied to the host for the oracle."""
import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb
from paper_2401_14110_amd import inputs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
PROD = (5, 7, 15)
ACC = (4, 7, 7)


def sample_rows(M, n_random=24, seed=0):
    """First and last tile rows, tile-boundary rows, and pseudo-random rows."""
    rows = {0, 1, 2, 3, 63, 64, 65, M - 1, M - 2, M - 64, M // 2}
    rng = np.random.default_rng(seed + M)
    rows |= set(int(r) for r in rng.integers(0, M, n_random))
    return np.array(sorted(r for r in rows if 0 <= r < M))


def check_rows(ref, layer, C, qp, qa, rows, what, order=0):
    idx = torch.from_numpy(rows).to(DEV)
    A = layer["A"].index_select(0, idx).cpu().numpy()
    B = layer["B"].cpu().numpy()
    want = ref.gemm(A, B, ref.QFmt(*qp), ref.QFmt(*qa), order=order)
    got = C.index_select(0, idx).cpu().numpy()
    bad = got.view(np.uint32) != want.view(np.uint32)
    assert not bad.any(), "%s: %d mismatches in %d sampled rows, first %s: gpu %r oracle %r" % (
        what, int(bad.sum()), len(rows), np.argwhere(bad)[0], got[bad][0], want[bad][0])


def check_grid_property(C, qa):
    """Every output is a value of Q_acc: low mantissa bits clear, magnitude <= R_OF, zero is +0."""
    E, M, b, _ = qa
    w = C.view(torch.int32)
    low = (1 << (23 - M)) - 1
    assert int((w & low).ne(0).sum()) == 0
    rof = (2.0 - 2.0 ** -M) * 2.0 ** ((1 << E) - b - 1)
    assert float(C.abs().max()) <= rof
    nz = C[C != 0]
    if nz.numel():
        assert float(nz.abs().min()) >= 2.0 ** -b
    assert int((w == -2 ** 31).sum()) == 0                         # no negative zero


@pytest.fixture(scope="module")
def resnet50():
    return inputs.make_workload("resnet50", DEV)


@pytest.mark.parametrize("rnd", [0, 1])
def test_resnet50_layers_sampled_rows(ref, resnet50, rnd):
    seen = set()
    for l in resnet50:
        key = (l["M"], l["N"], l["K"])
        if key in seen:
            continue
        seen.add(key)
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, ACC, rnd)
        C = lb.gemm(l["A"], l["B"], qp, qa)
        C2 = lb.gemm(l["A"], l["B"], qp, qa)
        torch.cuda.synchronize()
        check_rows(ref, l, C, qp, qa, sample_rows(l["M"]), "resnet50 %s %s" % (l["name"], key))
        check_grid_property(C, qa)
        assert torch.equal(C.view(torch.int32), C2.view(torch.int32))              # deterministic
        assert int(C.ne(0).sum()) > C.numel() // 4
        del C, C2
    assert len(seen) == 21


def test_resnet50_layers_chunked_order(ref, resnet50):
    # the paper's own accumulation order (chunks of 16) and bias pair b_acc, b_prod = 10, 12 (Sec. 3.1)
    seen = set()
    for l in resnet50:
        key = (l["M"], l["N"], l["K"])
        if key in seen:
            continue
        seen.add(key)
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], (4, 7, 12), (4, 7, 10), 0)
        C = lb.gemm(l["A"], l["B"], qp, qa, order=1)
        torch.cuda.synchronize()
        check_rows(ref, l, C, qp, qa, sample_rows(l["M"], 12), "resnet50 chunk16 %s" % (key,), order=1)
        check_grid_property(C, qa)
        del C


def test_resnet50_layers_m4e3_operands(ref):
    # lba_gemm_in / lba_gemm_bwd_in as bench.py --in-fmt 3,4 runs them: the paper's M4E3 codes with per-tensor flex
    # biases, the quantizers' biases in real units; every distinct shape of the sweep (plain and mixed grids, 48 x 64
    # rounds, truncated and nearest-even products), and the OF plane of the recompute call on three of them
    layers = inputs.make_workload("resnet50", DEV, in_fmt=(3, 4))
    seen, mixed, planes_checked = set(), 0, 0
    for l in layers:
        key = (l["M"], l["N"], l["K"])
        if key in seen:
            continue
        seen.add(key)
        fa, fb = (3, 4, l["ta"]), (3, 4, l["tb"])
        rows = sample_rows(l["M"], 12)
        idx = torch.from_numpy(rows).to(DEV)
        A = l["A"].index_select(0, idx).cpu().numpy()
        B = l["B"].cpu().numpy()
        for rnd, order in ((0, 0), (1, 0), (0, 1)):
            qp, qa = PROD + (rnd,), ACC + (rnd,)
            plan = lb.lba_plan_query_in(l["M"], l["N"], l["K"], fa, fb, qp, qa, order)
            mixed += plan["kernel"] == 0 and plan["tail_blocks"] + plan["mid_blocks"] > 0
            C = lb.gemm_in(l["A"], l["B"], fa, fb, qp, qa, order=order)
            torch.cuda.synchronize()
            want = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), ref.QFmt(*qp), ref.QFmt(*qa), order=order)
            got = C.index_select(0, idx).cpu().numpy()
            bad = got.view(np.uint32) != want.view(np.uint32)
            assert not bad.any(), (key, rnd, order, int(bad.sum()), np.argwhere(bad)[0])
            if rnd == 0:
                check_grid_property(C, qa)
            del C
        if key in ((12544, 1024, 256), (50176, 128, 512), (3136, 512, 2048)):
            qp, qa = PROD + (0,), ACC + (0,)
            plan = lb.lba_plan_query_in(l["M"], l["N"], l["K"], fa, fb, qp, qa, 0, with_masks=3)
            assert plan["kernel"] == 0, plan
            C, of, _ = lb.gemm_in(l["A"], l["B"], fa, fb, qp, qa, planes=True, uf_plane=False)
            torch.cuda.synchronize()
            wc, wof, _ = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), ref.QFmt(*qp), ref.QFmt(*qa), planes=True)
            assert np.array_equal(C.index_select(0, idx).cpu().numpy().view(np.uint32), wc.view(np.uint32)), key
            assert np.array_equal(of.index_select(1, idx).cpu().numpy().view(np.uint32), wof), key
            planes_checked += 1
            del C, of
    assert len(seen) == 21 and planes_checked == 3 and mixed >= 30, (len(seen), planes_checked, mixed)


def test_resnet18_conv_config(ref):
    (l,) = inputs.make_workload("conv", DEV)
    assert (l["M"], l["N"], l["K"]) == (100352, 64, 576)
    for rnd in (0, 1):
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, ACC, rnd)
        C = lb.gemm(l["A"], l["B"], qp, qa)
        torch.cuda.synchronize()
        check_rows(ref, l, C, qp, qa, sample_rows(l["M"], 200), "conv")
        check_grid_property(C, qa)
        # a row permutation of A permutes the rows of C (chains are independent)
        perm = torch.randperm(l["M"], device=DEV, generator=torch.Generator(DEV).manual_seed(1))
        Cp = lb.gemm(l["A"].index_select(0, perm), l["B"], qp, qa)
        torch.cuda.synchronize()
        assert torch.equal(Cp.view(torch.int32), C.index_select(0, perm).view(torch.int32))


def test_bert_base_linears(ref):
    for l in inputs.make_workload("bert", DEV):
        for rnd in (0, 1):
            qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, ACC, rnd)
            C = lb.gemm(l["A"], l["B"], qp, qa)
            torch.cuda.synchronize()
            if l["name"] == "attn_out" and rnd == 0:               # one layer in full
                rows = np.arange(l["M"])
            else:
                rows = sample_rows(l["M"], 40)
            check_rows(ref, l, C, qp, qa, rows, "bert %s" % l["name"])
            check_grid_property(C, qa)


def test_accumulator_width_sweep_4096(ref):
    (l,) = inputs.make_workload("gemm4096", DEV)
    rows = sample_rows(4096, 8)
    for M in range(3, 11):
        for E in (4, 5, 6):
            acc = (E, M, (1 << (E - 1)) - 1)
            for rnd in ((0, 1) if (M in (3, 7, 10)) else (0,)):
                qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, acc, rnd)
                C = lb.gemm(l["A"], l["B"], qp, qa)
                torch.cuda.synchronize()
                check_rows(ref, l, C, qp, qa, rows, "sweep M%dE%d rnd%d" % (M, E, rnd))
                check_grid_property(C, qa)


def test_event_planes_full_512_and_slab_of_4096(ref):
    (l,) = inputs.make_workload("gemm4096", DEV)
    # a full 512^3 problem
    A = l["A"][:512, :512].contiguous(); B = l["B"][:512, :512].contiguous()
    for acc, rnd in (((4, 3, 7), 0), ((4, 7, 7), 0), ((6, 10, 31), 1)):
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, acc, rnd)
        C, of, uf = lb.gemm_bwd(A, B, qp, qa)
        torch.cuda.synchronize()
        wc, wof, wuf = ref.gemm_bwd(A.cpu().numpy(), B.cpu().numpy(), ref.QFmt(*qp), ref.QFmt(*qa))
        assert np.array_equal(C.cpu().numpy().view(np.uint32), wc.view(np.uint32))
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof)
        assert np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)
        assert torch.equal(lb.gemm(A, B, qp, qa).view(torch.int32), C.view(torch.int32))
    # the 4096^3 problem: both planes (17 GB), a 48-row slab against the oracle
    qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, (4, 7, 7), 0)
    C, of, uf = lb.gemm_bwd(l["A"], l["B"], qp, qa)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(0, 16), np.arange(2040, 2056), np.arange(4080, 4096)])
    idx = torch.from_numpy(rows).to(DEV)
    wc, wof, wuf = ref.gemm_bwd(l["A"].index_select(0, idx).cpu().numpy(), l["B"].cpu().numpy(),
                                ref.QFmt(*qp), ref.QFmt(*qa))
    assert np.array_equal(C.index_select(0, idx).cpu().numpy().view(np.uint32), wc.view(np.uint32))
    assert np.array_equal(of.index_select(1, idx).cpu().numpy().view(np.uint32), wof)
    assert np.array_equal(uf.index_select(1, idx).cpu().numpy().view(np.uint32), wuf)
    assert torch.equal(lb.gemm(l["A"], l["B"], qp, qa).view(torch.int32), C.view(torch.int32))


def test_diff_plane_full_512_and_slab_of_4096(ref):
    (l,) = inputs.make_workload("gemm4096", DEV)
    A = l["A"][:512, :512].contiguous(); B = l["B"][:512, :512].contiguous()
    for acc, rnd, order, eps2 in (((4, 3, 7), 0, 0, 0.25), ((4, 7, 7), 0, 1, 0.5), ((5, 7, 15), 0, 0, 0.25), ((4, 7, 7), 1, 0, 0.0)):
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, acc, rnd)
        C, diff = lb.gemm_bwd_diff(A, B, qp, qa, eps2, order=order)
        torch.cuda.synchronize()
        wc, wd = ref.gemm_diff(A.cpu().numpy(), B.cpu().numpy(), ref.QFmt(*qp), ref.QFmt(*qa), eps2, order=order)
        assert np.array_equal(C.cpu().numpy().view(np.uint32), wc.view(np.uint32)), (acc, rnd, order)
        assert np.array_equal(diff.cpu().numpy().view(np.uint32), wd), (acc, rnd, order)
    # the 4096^3 problem in the configuration the benchmark times: a 48-row slab against the oracle
    qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, (4, 7, 7), 0)
    C, diff = lb.gemm_bwd_diff(l["A"], l["B"], qp, qa, 0.25)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(0, 16), np.arange(2040, 2056), np.arange(4080, 4096)])
    idx = torch.from_numpy(rows).to(DEV)
    wc, wd = ref.gemm_diff(l["A"].index_select(0, idx).cpu().numpy(), l["B"].cpu().numpy(), ref.QFmt(*qp), ref.QFmt(*qa), 0.25)
    assert np.array_equal(C.index_select(0, idx).cpu().numpy().view(np.uint32), wc.view(np.uint32))
    assert np.array_equal(diff.index_select(1, idx).cpu().numpy().view(np.uint32), wd)
    assert 0.01 < np.unpackbits(wd.view(np.uint8)).mean() < 0.99


def _grad_check(got, want, scale, terms, what):
    tol = 2 * (terms + 1) * 2.0 ** -24 * scale + 1e-30
    err = np.abs(got - want)
    assert (err <= tol).all(), "%s: worst error / tolerance %.3g" % (what, float((err / tol).max()))
    # and far from a trivially passing bound: a dropped term would show
    assert float((err / tol).max()) < 0.5


def test_gradient_products_at_benchmark_sizes(ref):
    """lba_grad at the sizes bench.py --grad times, on sampled outputs: rows of dX (each needs all n of its
    rows) and columns n of dW (each needs all m of its columns), for the three estimators on the BERT-base
    attention-output linear, and rows of dX on the ResNet-18 conv configuration."""
    from oracle import lba_grad_ref as gref

    def sampled(layer, G, dX, dW, ste, qp, qa, what):
        M, N, K = layer["M"], layer["N"], layer["K"]
        fp, fa = ref.QFmt(*qp), ref.QFmt(*qa)
        rows = sample_rows(M, n_random=12)
        idx = torch.from_numpy(rows).to(DEV)
        A = layer["A"].index_select(0, idx).cpu().numpy(); Gs = G.index_select(0, idx).cpu().numpy()
        B = layer["B"].cpu().numpy()
        c = gref.coefficients(A, B, fp, fa, ste)
        wX, _ = gref.grad(Gs, A, B, fp, fa, ste, c=c)
        aX, _ = gref.grad_abs(Gs, A, B, fp, fa, ste, c=c)
        _grad_check(dX.index_select(0, idx).cpu().numpy(), wX, aX, N, what + " dX rows")
        if dW is not None:
            cols = sample_rows(N, n_random=4)[:12]
            jdx = torch.from_numpy(cols).to(DEV)
            A = layer["A"].cpu().numpy(); Bs = layer["B"].index_select(0, jdx).cpu().numpy()
            Gs = G.index_select(1, jdx).cpu().numpy()
            c = gref.coefficients(A, Bs, fp, fa, ste)
            _, wW = gref.grad(Gs, A, Bs, fp, fa, ste, c=c)
            _, aW = gref.grad_abs(Gs, A, Bs, fp, fa, ste, c=c)
            _grad_check(dW.index_select(0, jdx).cpu().numpy(), wW, aW, M, what + " dW columns")
        return int((~c).sum())

    layer = [l for l in inputs.make_workload("bert", DEV) if l["name"] == "attn_out"][0]
    # b = 16 puts R_OF near 1, where these sums (standard deviation about 0.55) overflow now and then
    qp, qa, _ = inputs.folded_formats(layer["ta"], layer["tb"], PROD, (4, 7, 16), 0)
    G = torch.from_numpy(np.random.default_rng(5).standard_normal((layer["M"], layer["N"])).astype(np.float32)).to(DEV)
    _, of, _ = lb.gemm_bwd(layer["A"], layer["B"], qp, qa, want_c=False, want_uf=False)
    last = lb.last_overflow(of, layer["K"])
    blocked = 0
    for ste in (lb.STE_IDENTITY, lb.STE_IMMEDIATE_OF, lb.STE_RECURSIVE_OF):
        dX, dW = lb.grad(G, layer["A"], layer["B"], ste, of_plane=of if ste == lb.STE_IMMEDIATE_OF else None,
                         last_of=last if ste == lb.STE_RECURSIVE_OF else None)
        torch.cuda.synchronize()
        blocked += sampled(layer, G, dX, dW, ste, qp, qa, "attn_out ste=%d" % ste)
    assert blocked > 0
    # ResNet-18 conv configuration (M = 100352): rows of dX, immediate estimator
    layer = inputs.make_workload("conv", DEV)[0]
    qp, qa, _ = inputs.folded_formats(layer["ta"], layer["tb"], PROD, ACC, 0)
    G = torch.from_numpy(np.random.default_rng(6).standard_normal((layer["M"], layer["N"])).astype(np.float32)).to(DEV)
    _, of, _ = lb.gemm_bwd(layer["A"], layer["B"], qp, qa, want_c=False, want_uf=False)
    dX, _ = lb.grad(G, layer["A"], layer["B"], lb.STE_IMMEDIATE_OF, of_plane=of, want_dw=False)
    torch.cuda.synchronize()
    sampled(layer, G, dX, None, lb.STE_IMMEDIATE_OF, qp, qa, "conv")


def test_brick_maps_and_premapped_gradients_at_benchmark_sizes(ref):
    """lba_gemm_bwd_ws / lba_grad_premapped at benchmark sizes: the maps the recompute kernel leaves (plain grid on the
    BERT linear, mixed grid on the ResNet-18 conv) equal the maps lba_grad_ws builds with its own pass over the same
    plane, byte for byte, and the gradients of lba_grad_premapped pass the sampled check against the oracle."""
    from oracle import lba_grad_ref as gref

    cases = []
    layer = [l for l in inputs.make_workload("bert", DEV) if l["name"] == "attn_out"][0]
    cases.append((layer, inputs.folded_formats(layer["ta"], layer["tb"], PROD, (4, 7, 16), 0)[:2], "attn_out"))   # overflows now and then
    layer = inputs.make_workload("conv", DEV)[0]
    cases.append((layer, inputs.folded_formats(layer["ta"], layer["tb"], PROD, (4, 7, 9), 0)[:2], "conv"))
    marked = 0
    for layer, (qp, qa), what in cases:
        M, N, K = layer["M"], layer["N"], layer["K"]
        need = lb.lba_grad_workspace_bytes(M, N, K)
        G = torch.from_numpy(np.random.default_rng(8).standard_normal((M, N)).astype(np.float32)).to(DEV)
        _, of, _, ws = lb.gemm_bwd_ws(layer["A"], layer["B"], qp, qa, want_c=False, want_uf=False)
        ws2 = torch.full((need,), 0x77, dtype=torch.uint8, device=DEV)
        eX, eW = lb.grad(G, layer["A"], layer["B"], lb.STE_IMMEDIATE_OF, of_plane=of, workspace=ws2)
        dX, dW = lb.grad_premapped(G, layer["A"], layer["B"], of, ws)
        torch.cuda.synchronize()
        assert torch.equal(ws[:need] != 0, ws2 != 0), what
        marked += int((ws[:need] != 0).sum())
        fp, fa = ref.QFmt(*qp), ref.QFmt(*qa)
        rows = sample_rows(M, n_random=8)
        idx = torch.from_numpy(rows).to(DEV)
        A = layer["A"].index_select(0, idx).cpu().numpy(); Gs = G.index_select(0, idx).cpu().numpy()
        B = layer["B"].cpu().numpy()
        c = gref.coefficients(A, B, fp, fa, lb.STE_IMMEDIATE_OF)
        wX, _ = gref.grad(Gs, A, B, fp, fa, lb.STE_IMMEDIATE_OF, c=c)
        aX, _ = gref.grad_abs(Gs, A, B, fp, fa, lb.STE_IMMEDIATE_OF, c=c)
        _grad_check(dX.index_select(0, idx).cpu().numpy(), wX, aX, N, what + " dX rows (premapped)")
        scale = float(eW.abs().max())
        assert float((dW - eW).abs().max()) <= 1e-4 * scale, what
    assert marked > 0
