"""Complete outputs at benchmark sizes: the checksum of every C the HIP library produces against the checksum
of the oracle's C, computed offline (tests/golden/full_digests.txt, written by tests/golden/make_full_digests.py
from oracle/ alone).  The inputs are regenerated here from the same seeds; their checksums are compared first,
so that a drift of the generator (it runs on the GPU here, on the CPU offline) cannot pass for a parity error:
an operand whose checksum differs is regenerated on the CPU, and if it still differs the case is skipped."""
import os

import pytest
import torch

from digest import digest
from paper_2401_14110_amd import binding as lb
from paper_2401_14110_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLD = os.path.join(os.path.dirname(__file__), "golden", "full_digests.txt")


def golden(name):
    rows = []
    for line in open(GOLD):
        f = line.split()
        if f and f[0] == name:
            rows.append(dict(layer=int(f[1]), M=int(f[2]), N=int(f[3]), K=int(f[4]),
                             qp=tuple(int(v) for v in f[5].split(",")), qa=tuple(int(v) for v in f[6].split(",")),
                             order=int(f[7]), dA=int(f[8], 16), dB=int(f[9], 16), dC=int(f[10], 16)))
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
    if not rows:
        pytest.skip("no golden checksums for %s" % name)
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
            if digest(A) != r["dA"] or digest(B) != r["dB"]:
                pytest.skip("the input generator gives other codes on this host than where the golden file was made")
        # the golden row carries the folded formats the oracle ran with (the operand scales are part of them)
        C = lb.gemm(A, B, r["qp"], r["qa"], order=r["order"])
        torch.cuda.synchronize()
        assert digest(C) == r["dC"], (name, r["layer"], r["M"], r["N"], r["K"], r["qp"], r["qa"])
        checked += 1
    assert checked == len(rows)
