"""Complete outputs at benchmark sizes: the checksum of every C the HIP library produces against the checksum
of the oracle's C, computed offline (tests/golden/full_digests.txt, written by tests/golden/make_full_digests.py
from oracle/ alone).  The inputs are regenerated here from the same seeds; their checksums are compared first,
so that a drift of the generator (it runs on the GPU here, on the CPU offline) cannot pass for a parity error:
an operand whose checksum differs is regenerated on the CPU, and if it still differs the test fails (a skip
would be no coverage at all).  Rows that carry plane checksums (of= uf= [of2= uf2=]) are run through the
recompute call (lba_gemm_bwd, or lba_gemm_bwd_chunked under the chunked order) and every plane is compared in
full as well."""
import os

import pytest
import torch

from paper_2401_14110_amd.digest import digest
from paper_2401_14110_amd import binding as lb
from paper_2401_14110_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLD = os.path.join(os.path.dirname(__file__), "golden", "full_digests.txt")
# (rounding, order, with planes) cases the golden file must hold per workload
WANT_CASES = {"conv": {(0, 0, True), (1, 0, False)}, "bert": {(0, 0, True), (0, 1, True)}, "gemm4096": {(0, 0, False), (0, 0, True)},
              "resnet50": {(0, 0, False), (1, 0, False), (0, 1, False), (0, 0, True)}}


def golden(name):
    rows = []
    for line in open(GOLD):
        f = line.split()
        if f and f[0] == name:
            rows.append(dict(layer=int(f[1]), M=int(f[2]), N=int(f[3]), K=int(f[4]),
                             qp=tuple(int(v) for v in f[5].split(",")), qa=tuple(int(v) for v in f[6].split(",")),
                             order=int(f[7]), dA=int(f[8], 16), dB=int(f[9], 16), dC=int(f[10], 16),
                             planes={t.split("=")[0]: int(t.split("=")[1], 16) for t in f[11:]}))
    return rows


def test_digest_function_is_the_same_on_both_devices():
    g = torch.Generator().manual_seed(3)
    x = torch.randint(0, 256, (100003,), dtype=torch.uint8, generator=g)
    f = torch.randn((777, 131), generator=g)
    assert digest(x) == digest(x.to(DEV)) and digest(f) == digest(f.to(DEV))
    y = x.clone(); y[5], y[6] = x[6], x[5]
    assert digest(y) != digest(x) or x[5] == x[6]
    f2 = f.clone(); f2[700, 100] = -f2[700, 100]
    assert digest(f2) != digest(f) and digest(f, chunk=1000) == digest(f)


@pytest.mark.parametrize("name", ["conv", "bert", "gemm4096", "resnet50"])
def test_complete_outputs_against_offline_oracle_checksums(name):
    rows = golden(name)
    assert rows, "no golden checksums for %s in tests/golden/full_digests.txt" % name
    cases = {(r["qp"][3], r["order"], bool(r["planes"])) for r in rows}
    assert WANT_CASES[name] <= cases, (name, cases)
    layers = inputs.make_workload(name, DEV)
    cpu_layers = None
    checked = 0
    for r in rows:
        l = layers[r["layer"]]
        assert (l["M"], l["N"], l["K"]) == (r["M"], r["N"], r["K"])
        A, B = l["A"], l["B"]
        if digest(A) != r["dA"] or digest(B) != r["dB"]:
            if cpu_layers is None:
                cpu_layers = inputs.make_workload(name, "cpu")
            A, B = cpu_layers[r["layer"]]["A"].to(DEV), cpu_layers[r["layer"]]["B"].to(DEV)
            assert digest(A) == r["dA"] and digest(B) == r["dB"], \
                "the input generator gives other codes on this host than where the golden file was made"
        # the golden row carries the folded formats the oracle ran with (the operand scales are part of them)
        what = (name, r["layer"], r["M"], r["N"], r["K"], r["qp"], r["qa"], r["order"])
        if r["planes"]:
            if r["order"] == 1:
                C, of, uf, of2, uf2 = lb.gemm_bwd_chunked(A, B, r["qp"], r["qa"])
                got = {"of": of, "uf": uf, "of2": of2, "uf2": uf2}
            else:
                C, of, uf = lb.gemm_bwd(A, B, r["qp"], r["qa"])
                got = {"of": of, "uf": uf}
            torch.cuda.synchronize()
            assert set(got) == set(r["planes"]), what
            for tag, plane in got.items():
                assert digest(plane) == r["planes"][tag], what + (tag,)
            del got, of, uf
        else:
            C = lb.gemm(A, B, r["qp"], r["qa"], order=r["order"])
            torch.cuda.synchronize()
        assert digest(C) == r["dC"], what
        del C
        checked += 1
    assert checked == len(rows)
