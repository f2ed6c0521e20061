"""The seeded input generators (shared by the HIP path's callers and the oracle's tests; they hold none
of the method's arithmetic): determinism, the FP8 casts against torch's, the scale rules, the layer lists."""
import numpy as np
import torch

from paper_2401_14110_amd import inputs


def test_counter_rng_is_deterministic_and_chunk_independent():
    a = inputs.normal(3, 1, 5000)
    b = inputs.normal(3, 1, 5000, chunk=777)
    assert torch.equal(a, b) and not torch.equal(a, inputs.normal(3, 2, 5000))
    assert abs(float(a.mean())) < 0.05 and abs(float(a.std()) - 1.0) < 0.05


def test_casts_match_torch_float8():
    x = torch.cat([inputs.normal(1, 0, 200000) * 30.0, torch.tensor([0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 1e-9,
                                                                      0.001953125 * 1.5, 17.0, 464.0, 1e6], dtype=torch.float64)])
    sat = x.clamp(-448.0, 448.0)
    want = sat.float().to(torch.float8_e4m3fn).view(torch.uint8)
    got = inputs.to_e4m3(x)
    same = got == want
    assert bool(same[sat.abs() > 0].all())                       # (torch keeps the sign of -0.0; so does the cast)
    inside = x.abs() <= 448.0
    assert torch.equal(inputs.to_fp8_code(x, 4, 3)[inside], got[inside])
    inside = x.abs() <= 57344.0                                  # binary8 E5M2 ends there (e = 31 is inf / NaN)
    assert torch.equal(inputs.to_fp8_code(x, 5, 2)[inside], x.float().to(torch.float8_e5m2).view(torch.uint8)[inside])
    assert int(inputs.to_fp8_code(x, 5, 2)[-1]) == 0x7F          # every code is finite here: saturation at the top code
    assert inputs.fp8_max(3, 4) == 31.0 and inputs.fp8_max(4, 3) == 480.0 and inputs.fp8_max(5, 2) == 114688.0


def test_scale_rules():
    x = inputs.normal(2, 0, 10000) * 0.02
    codes, t = inputs.quantize_tensor(x)
    mx = float(x.abs().max())
    assert mx * 2.0 ** t <= 448.0 < mx * 2.0 ** (t + 1)
    codes, bias = inputs.quantize_tensor_fp8(x, 3, 4)
    t = bias - 3
    assert mx * 2.0 ** t <= 31.0 < mx * 2.0 ** (t + 1)
    assert int(codes.max()) >= 0x70                               # the top binade is used


def test_layer_lists():
    l = inputs.resnet50_gemms()
    assert len(l) == 54 and sum(M * N * K for _, M, N, K in l) == 261707792384
    assert min(K for _, _, _, K in l) == 64 and max(K for _, _, _, K in l) == 4608
    assert [s[1:] for s in inputs.bert_base_gemms()] == [(4096, 2304, 768), (4096, 768, 768), (4096, 3072, 768), (4096, 768, 3072)]
    convs = inputs.resnet50_convs()
    assert len(convs) == 54
    for (_, M, N, K), (_, n, h, w_, c, cout, kh, kw, s_, p_) in zip(l, convs):
        oh, ow = (h + 2 * p_ - kh) // s_ + 1, (w_ + 2 * p_ - kw) // s_ + 1
        assert (M, N, K) == (n * oh * ow, cout, kh * kw * c)
    w = inputs.make_workload("config1")
    assert w[0]["A"].shape == (64, 256) and w[0]["ta"] == 0 and int(w[0]["A"].max()) >= 0x7E - 0x08


def test_checksum_function_and_golden_file():
    """paper_2401_14110_amd/digest.py (the checksum the full-size GPU checks use) on the CPU: position-sensitive, independent of
    the chunking; the golden file holds one row per GEMM of the benchmark configurations."""
    import os
    import torch
    from paper_2401_14110_amd.digest import digest
    g = torch.Generator().manual_seed(5)
    x = torch.randint(0, 256, (70001,), dtype=torch.uint8, generator=g)
    f = torch.randn((333, 77), generator=g)
    assert digest(x) == digest(x.clone()) and digest(f, chunk=1000) == digest(f) and digest(x, chunk=4097) == digest(x)
    y = x.clone(); y[11] ^= 1
    assert digest(y) != digest(x)
    z = f.clone().view(-1); z[[3, 4]] = z[[4, 3]]
    assert digest(z) != digest(f) or z[3] == z[4]
    assert digest(torch.zeros(5)) != digest(torch.zeros(6))                 # a missing word changes the sum
    rows = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "full_digests.txt")
    for line in open(path):
        t = line.split()
        if t and not line.startswith("#"):
            assert len(t) in (11, 13, 15) and all(len(v) == 16 for v in t[8:11])
            assert [v.split("=")[0] for v in t[11:]] == ["of", "uf", "of2", "uf2"][:len(t) - 11]
            assert all(len(v.split("=")[1]) == 16 for v in t[11:])
            assert (len(t) == 15) == (t[7] == "1" and len(t) > 11)         # chunked order with planes: four of them
            rows[t[0]] = rows.get(t[0], 0) + 1
    # conv: floor (with planes) and nearest-even; bert: floor / sequential and the paper's biases / chunked, with
    # planes; 4096^3: floor without and with planes; ResNet-50: floor (without and with planes), nearest-even and the
    # paper's biases under the chunked order
    assert rows == {"conv": 2, "bert": 8, "gemm4096": 2, "resnet50": 216}
