"""Writes tests/golden/full_digests.txt: checksums (paper_2401_14110_amd/digest.py) of the complete oracle outputs of the
benchmark configurations, with the checksums of the input codes they were computed from.  Calls only the
input generators and oracle/ (never the HIP library).  Run from the repository root:

    python tests/golden/make_full_digests.py [--redo] [conv bert gemm4096 resnet50]

Rows that the file already holds (same workload, layer, formats, order and the same set of checksums) are
kept as they are unless --redo is given.  Cases with planes also carry the checksums of the event planes of
the recompute (Sec. 4, App. C.3: one bit per FMAq step): of= / uf= for the first level and, under the chunked
order, of2= / uf2= for the second level.  The ResNet-50 sweep is 2.6e11 oracle MACs per case: several minutes
on 8 cores (layers with identical operands are computed once)."""
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

import torch  # noqa: E402

from paper_2401_14110_amd.digest import digest  # noqa: E402
from oracle import lba_ref  # noqa: E402
from paper_2401_14110_amd import inputs  # noqa: E402

PROD = (5, 7, 15)
ACC = (4, 7, 7)
# the paper's own bias pair b_acc, b_prod = 10, 12 with M7E4 for both formats (Sec. 3.1), its order: chunks of 16
PAPER_PROD, PAPER_ACC = (4, 7, 12), (4, 7, 10)
CASES = {  # workload -> [(product format, accumulator format, rounding, order, planes)]
    "conv": [(PROD, ACC, 0, 0, True), (PROD, ACC, 1, 0, False)],
    "bert": [(PROD, ACC, 0, 0, True), (PAPER_PROD, PAPER_ACC, 0, 1, True)],
    "gemm4096": [(PROD, ACC, 0, 0, False), (PROD, ACC, 0, 0, True)],
    "resnet50": [(PROD, ACC, 0, 0, False), (PROD, ACC, 1, 0, False), (PAPER_PROD, PAPER_ACC, 0, 1, False), (PROD, ACC, 0, 0, True)],
}


def row_key(fields):
    """workload, layer, qprod, qacc, order, and which checksums the row carries"""
    return (fields[0], fields[1], fields[5], fields[6], fields[7], tuple(f.split("=")[0] for f in fields[11:]))


def main():
    args = sys.argv[1:]
    redo = "--redo" in args
    names = [a for a in args if not a.startswith("--")] or ["conv", "bert", "gemm4096"]
    out = os.path.join(HERE, "full_digests.txt")
    old = {}
    if os.path.exists(out):
        for line in open(out):
            if line.strip() and not line.startswith("#"):
                old.setdefault(line.split()[0], []).append(line)
    for name in names:
        have = {} if redo else {row_key(line.split()): line for line in old.get(name, [])}
        layers = inputs.make_workload(name, "cpu")
        lines = []
        done = {}                                             # identical operands and formats: computed once
        for prod, acc, rnd, order, planes in CASES[name]:
            for i, l in enumerate(layers):
                qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], prod, acc, rnd)
                sqp, sqa = ",".join(map(str, qp)), ",".join(map(str, qa))
                tags = (("of", "uf", "of2", "uf2") if order == 1 else ("of", "uf")) if planes else ()
                key = (name, str(i), sqp, sqa, str(order), tags)
                if key in have:
                    lines.append(have[key])
                    continue
                t0 = time.time()
                dA, dB = digest(l["A"]), digest(l["B"])
                same = (dA, dB, l["M"], l["N"], l["K"], sqp, sqa, order, planes)
                if same not in done:
                    a, b = l["A"].numpy(), l["B"].numpy()
                    if planes:
                        res = lba_ref.gemm_bwd(a, b, lba_ref.QFmt(*qp), lba_ref.QFmt(*qa), order=order,
                                               nthreads=os.cpu_count(), level2=(order == 1))
                    else:
                        res = (lba_ref.gemm(a, b, lba_ref.QFmt(*qp), lba_ref.QFmt(*qa), order=order,
                                            nthreads=os.cpu_count()),)
                    done[same] = [digest(torch.from_numpy(r.view("int32") if r.dtype != "float32" else r)) for r in res]
                    del res
                d = done[same]
                extra = "".join("  %s=%016x" % (t, v) for t, v in zip(tags, d[1:]))
                lines.append("%s %d %d %d %d  %s %s %d  %016x %016x %016x%s\n" % (
                    name, i, l["M"], l["N"], l["K"], sqp, sqa, order, dA, dB, d[0], extra))
                print(lines[-1].strip(), "%.1f s" % (time.time() - t0), flush=True)
        old[name] = lines
        with open(out, "w") as f:
            f.write("# Checksums of complete oracle outputs (tests/golden/make_full_digests.py; oracle/lba_ref.cpp only).\n"
                    "# workload layer M N K  qprod(E,M,b,round) qacc(E,M,b,round) order  digest(A) digest(B) digest(C)"
                    "  [of= uf= [of2= uf2=] digests of the event planes]\n")
            for n in sorted(old):
                f.writelines(old[n])


if __name__ == "__main__":
    main()
