"""Seeded synthetic inputs for the LBA matrix product (shapes and value distributions only).

This module holds NO arithmetic of the method itself (no quantizer Q, no FMAq, no accumulation):
it only draws random tensors, scales them per tensor, and casts them to FP8 E4M3 codes.  It is the
one module that both the test oracle's callers and the HIP path's callers use, so that the two
sides see the same bytes.

Random numbers: a counter-based generator (the published splitmix64 finaliser applied to
seed/stream/index) followed by the Box-Muller transform, written with torch integer/float64 ops so
that it runs on the CPU or on the GPU.  Element i of stream s under seed z is a pure function of
(z, s, i): tensors can be generated in chunks and in any order.

Workload stand-ins.  The paper fine-tunes torchvision ResNets on ImageNet and BERT models on SQuAD
(Sec. 3.1-3.2, App. C); neither the datasets nor the weights exist here, so only layer SHAPES and
plausible value distributions are kept: ReLU(N(0,1)) activations with Kaiming-normal weights for
convolutions (as im2col GEMMs), N(0,1) activations with N(0, 0.02^2) weights for BERT linears.
"""
import math

import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB


def _s64(x):
    """Python int (mod 2^64) -> the same bits as a signed 64-bit value."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x, s):
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z):
    z = (z ^ _lsr(z, 30)) * _s64(_MUL1)
    z = (z ^ _lsr(z, 27)) * _s64(_MUL2)
    return z ^ _lsr(z, 31)


def _mix_py(z):
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _MUL1) & _MASK64
    z = ((z ^ (z >> 27)) * _MUL2) & _MASK64
    return z ^ (z >> 31)


def _stream_base(seed, stream):
    return _mix_py(_mix_py(seed * 2 + 1) ^ ((stream * 2 + 1) * _GOLDEN))


def uniform_bits(seed, stream, start, count, device="cpu"):
    """53-bit uniform integers (as int64) for counters start .. start+count-1."""
    base = _stream_base(seed, stream)
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    z = i * _s64(_GOLDEN) + _s64(base)
    return _lsr(_mix(z), 11)


def normal(seed, stream, n, device="cpu", chunk=1 << 24):
    """n independent N(0,1) draws (float64), Box-Muller on two counters per draw."""
    out = torch.empty(n, dtype=torch.float64, device=device)
    for lo in range(0, n, chunk):
        c = min(chunk, n - lo)
        b = uniform_bits(seed, stream, 2 * lo, 2 * c, device)
        u1 = (b[0::2] + 1).to(torch.float64) * (2.0 ** -53)     # (0, 1]
        u2 = b[1::2].to(torch.float64) * (2.0 ** -53)           # [0, 1)
        out[lo:lo + c] = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return out


def to_e4m3(x):
    """float64 tensor -> uint8 OCP E4M3 codes: round-to-nearest-even, saturating at +-448."""
    ax = x.abs().clamp(max=448.0)
    _, ex = torch.frexp(ax)                       # ax = f * 2^ex, f in [0.5, 1)
    e = (ex - 1).clamp(min=-6)                    # binade; below 2^-6 the grid is the subnormal one
    quantum = torch.ldexp(torch.ones_like(ax), e - 3)
    q = torch.round(ax / quantum)                 # half-to-even; exact division by a power of two
    v = q * quantum
    _, ex2 = torch.frexp(v)
    e2 = (ex2 - 1).clamp(min=-6)
    m = torch.round(v / torch.ldexp(torch.ones_like(v), e2 - 3)).to(torch.int64)   # 0..15
    normal_code = ((e2 + 7).to(torch.int64) << 3) + (m - 8)
    code = torch.where(m >= 8, normal_code, m)    # m < 8 only on the subnormal grid (e2 == -6)
    code = code + (torch.signbit(x).to(torch.int64) << 7)
    return code.to(torch.uint8)


def fp8_max(E, M):
    """Largest value of the 8-bit format (1 sign, E exponent, M mantissa bits, bias 2^(E-1) - 1, every
    code finite)."""
    return (2.0 - 2.0 ** -M) * 2.0 ** ((1 << E) - 1 - ((1 << (E - 1)) - 1))


def to_fp8_code(x, E, M):
    """float64 tensor -> uint8 codes of that format at its canonical bias: round-to-nearest-even,
    saturating at +-fp8_max(E, M).  (E, M) = (3, 4) is the paper's M4E3 weight / activation format."""
    bias = (1 << (E - 1)) - 1
    emin = 1 - bias
    ax = x.abs().clamp(max=fp8_max(E, M))
    _, ex = torch.frexp(ax)
    e = (ex - 1).clamp(min=emin)                  # below 2^emin the grid is the subnormal one
    q = torch.round(ax / torch.ldexp(torch.ones_like(ax), e - M))
    v = q * torch.ldexp(torch.ones_like(ax), e - M)
    _, ex2 = torch.frexp(v)
    e2 = (ex2 - 1).clamp(min=emin)                # a mantissa carry moves to the next binade
    m = torch.round(v / torch.ldexp(torch.ones_like(v), e2 - M)).to(torch.int64)    # 0 .. 2^(M+1) - 1
    normal_code = ((e2 + bias).to(torch.int64) << M) + (m - (1 << M))
    code = torch.where(m >= (1 << M), normal_code, m)
    code = code + (torch.signbit(x).to(torch.int64) << 7)
    return code.to(torch.uint8)


def quantize_tensor_fp8(x, E, M):
    """Per-tensor "flex-bias" cast (Sec. 3.1 of the paper): the largest integer exponent bias that keeps
    max|x| inside the format.  Returns (uint8 codes, bias): value(code) = (canonical value) * 2^(canonical - bias)."""
    mx = float(x.abs().max())
    top = fp8_max(E, M)
    t = 0
    if mx > 0.0 and math.isfinite(mx):
        t = math.floor(math.log2(top / mx))
        while mx * 2.0 ** (t + 1) <= top:
            t += 1
        while mx * 2.0 ** t > top:
            t -= 1
    codes = to_fp8_code(torch.ldexp(x, torch.tensor(t, device=x.device)), E, M)
    return codes, ((1 << (E - 1)) - 1) + t


def pow2_scale_exp(x):
    """Largest integer t with max|x| * 2^t <= 448 (the per-tensor power-of-two scale)."""
    mx = float(x.abs().max())
    if mx == 0.0 or not math.isfinite(mx):
        return 0
    t = math.floor(math.log2(448.0 / mx))
    while mx * 2.0 ** (t + 1) <= 448.0:
        t += 1
    while mx * 2.0 ** t > 448.0:
        t -= 1
    return t


def quantize_tensor(x, scale_mode="pow2"):
    """Per-tensor scale then cast.  Returns (uint8 codes, t) with codes ~ x * 2^t ('pow2') or
    x * 448/max|x| ('exact448', t = round(log2 of that scale))."""
    if scale_mode == "pow2":
        t = pow2_scale_exp(x)
        return to_e4m3(torch.ldexp(x, torch.tensor(t, device=x.device))), t
    if scale_mode == "exact448":
        mx = float(x.abs().max())
        s = 448.0 / mx if mx > 0 else 1.0
        return to_e4m3(x * s), int(round(math.log2(s)))
    raise ValueError(scale_mode)


def make_operand(kind, rows, cols, seed, stream, device="cpu", scale_mode="pow2", std=1.0,
                 row_chunk=None, in_fmt=None):
    """One operand matrix [rows, cols] of E4M3 codes.  kind: 'normal' N(0,std^2) or 'relu'
    ReLU(N(0,1)).  Returns (codes uint8 [rows, cols], t); with in_fmt = (E, M) the codes are of that
    format and t is its flex bias."""
    n = rows * cols
    x = normal(seed, stream, n, device=device)
    if kind == "relu":
        x = torch.clamp(x, min=0.0)
    elif kind == "normal":
        if std != 1.0:
            x = x * std
    else:
        raise ValueError(kind)
    if in_fmt is not None:
        codes, t = quantize_tensor_fp8(x, *in_fmt)
    else:
        codes, t = quantize_tensor(x, scale_mode)
    return codes.reshape(rows, cols), t


# ---------------------------------------------------------------------------------------------
# Layer shapes (M, N, K) as im2col / linear GEMMs
# ---------------------------------------------------------------------------------------------

def resnet50_gemms(batch=64, image=224):
    """(name, M, N, K) for every conv and the FC of a torchvision-style ResNet-50 forward pass
    (stride on the 3x3 conv of each bottleneck), each written as C[M,N] = A[M,K] . B[N,K]^T."""
    layers = []
    h = image // 2                                # conv1: 7x7 / 2
    layers.append(("conv1", batch * h * h, 64, 3 * 49))
    h = h // 2                                    # maxpool / 2
    inplanes = 64
    for si, (planes, blocks, stride) in enumerate(((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))):
        for bi in range(blocks):
            s = stride if bi == 0 else 1
            name = "layer%d.%d" % (si + 1, bi)
            layers.append((name + ".conv1", batch * h * h, planes, inplanes))            # 1x1
            ho = h // s
            layers.append((name + ".conv2", batch * ho * ho, planes, planes * 9))        # 3x3 / s
            layers.append((name + ".conv3", batch * ho * ho, planes * 4, planes))        # 1x1
            if bi == 0:
                layers.append((name + ".downsample", batch * ho * ho, planes * 4, inplanes))
            inplanes = planes * 4
            h = ho
    layers.append(("fc", batch, 1000, 2048))
    return layers


def resnet50_convs(batch=64, image=224):
    """The same layers as resnet50_gemms, in the same order, as convolution descriptors
    (name, n, h, w, c, cout, kh, kw, stride, pad) on NHWC activations; the FC layer is a 1x1 convolution
    on a 1x1 image."""
    layers = []
    layers.append(("conv1", batch, image, image, 3, 64, 7, 7, 2, 3))
    h = image // 4                                # after conv1 / 2 and maxpool / 2
    inplanes = 64
    for si, (planes, blocks, stride) in enumerate(((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))):
        for bi in range(blocks):
            s = stride if bi == 0 else 1
            name = "layer%d.%d" % (si + 1, bi)
            layers.append((name + ".conv1", batch, h, h, inplanes, planes, 1, 1, 1, 0))
            layers.append((name + ".conv2", batch, h, h, planes, planes, 3, 3, s, 1))
            ho = h // s
            layers.append((name + ".conv3", batch, ho, ho, planes, planes * 4, 1, 1, 1, 0))
            if bi == 0:
                layers.append((name + ".downsample", batch, h, h, inplanes, planes * 4, 1, 1, s, 0))
            inplanes = planes * 4
            h = ho
    layers.append(("fc", batch, 1, 1, 2048, 1000, 1, 1, 1, 0))
    return layers


def bert_base_gemms(batch=32, seq=128):
    m = batch * seq
    return [("qkv", m, 2304, 768), ("attn_out", m, 768, 768),
            ("ffn_in", m, 3072, 768), ("ffn_out", m, 768, 3072)]


def make_conv_workload(name, device="cpu"):
    """'resnet50' or 'conv' as convolutions on NHWC activation tensors (for lba_conv2d): a list of dicts
    (name, desc = (n, h, w, c, kh, kw, stride, pad), cout, M, N, K, X [n, h, w, c], B [cout, kh*kw*c], ta, tb).
    Value distributions as in make_workload; layers of equal tensor shape share data."""
    if name == "resnet50":
        convs, seed = resnet50_convs(64, 224), 2
    elif name == "conv":
        convs, seed = [("resnet18.layer1.conv", 32, 56, 56, 64, 64, 3, 3, 1, 1)], 1
    else:
        raise ValueError("no convolution form of workload %r" % name)
    cache_x, cache_b, out = {}, {}, []
    for (lname, n, h, w, c, cout, kh, kw, stride, pad) in convs:
        K = kh * kw * c
        oh, ow = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1
        if (n, h, w, c) not in cache_x:
            kind = "normal" if lname == "conv1" else "relu"
            X, ta = make_operand(kind, n * h * w, c, seed, 2 * len(cache_x), device=device)
            cache_x[(n, h, w, c)] = (X.view(n, h, w, c), ta)
        if (cout, K) not in cache_b:
            cache_b[(cout, K)] = make_operand("normal", cout, K, seed, 2 * len(cache_b) + 1, device=device,
                                              std=(2.0 / K) ** 0.5)
        X, ta = cache_x[(n, h, w, c)]
        B, tb = cache_b[(cout, K)]
        out.append(dict(name=lname, desc=(n, h, w, c, kh, kw, stride, pad), cout=cout, M=n * oh * ow, N=cout, K=K,
                        X=X, A=X, B=B, ta=ta, tb=tb))
    return out


def make_workload(name, device="cpu", in_fmt=None):
    """Operands of a named workload as a list of dicts (name, M, N, K, A, B, ta, tb): A [M,K] and
    B [N,K] uint8 codes on `device`, ta / tb the power-of-two scale exponents.  Layers of equal
    operand shape share data.  Workloads: 'resnet50' (ResNet-50 forward, batch 64, 224x224: 54 GEMMs),
    'conv' (ResNet-18 3x3 conv 64->64 at batch 32), 'bert' (BERT-base linears, 4096 tokens),
    'gemm4096' (4096^3, N(0,1) operands), 'config1' (M=N=64, K=256, N(0,1) operands scaled to
    max|x| = 448, seed 0), 'layer:MxNxK' (one GEMM of that shape with the ResNet-50 recipe: ReLU activations,
    He weights; for per-shape profiles).  With in_fmt = (E, M) the codes are of that 8-bit format and ta / tb are the
    per-tensor flex biases (for lba_gemm_in, with the quantizers' biases in real units)."""
    if name == "resnet50":
        layers = resnet50_gemms(batch=64, image=224)
        seed = 2
    elif name == "conv":
        layers = [("resnet18.layer1.conv", 32 * 56 * 56, 64, 576)]
        seed = 1
    elif name == "bert":
        layers = bert_base_gemms(32, 128)
        seed = 3
    elif name == "gemm4096":
        layers = [("gemm4096", 4096, 4096, 4096)]
        seed = 4
    elif name == "config1":
        layers = [("gemm64", 64, 64, 256)]
        seed = 0
    elif name.startswith("layer:"):
        M, N, K = (int(v) for v in name[6:].split("x"))
        layers = [(name, M, N, K)]
        seed = 3
    else:
        raise ValueError("unknown workload %r" % name)
    # one operand tensor per distinct (rows, K) and role: layers of equal shape share data
    cache_a, cache_b, out = {}, {}, []
    mode = "exact448" if name == "config1" else "pow2"
    for idx, (lname, M, N, K) in enumerate(layers):
        if (M, K) not in cache_a:
            if name == "resnet50":
                kind = "normal" if lname == "conv1" else "relu"
            elif name == "conv" or name.startswith("layer:"):
                kind = "relu"
            else:
                kind = "normal"
            cache_a[(M, K)] = make_operand(kind, M, K, seed, 2 * len(cache_a), device=device,
                                           scale_mode=mode, in_fmt=in_fmt)
        if (N, K) not in cache_b:
            if name in ("resnet50", "conv") or name.startswith("layer:"):
                std = (2.0 / K) ** 0.5
            elif name == "bert":
                std = 0.02
            else:
                std = 1.0
            cache_b[(N, K)] = make_operand("normal", N, K, seed, 2 * len(cache_b) + 1,
                                           device=device, std=std, scale_mode=mode, in_fmt=in_fmt)
        A, ta = cache_a[(M, K)]
        B, tb = cache_b[(N, K)]
        if mode == "exact448":
            ta = tb = 0                            # formats are given in code units there
        out.append(dict(name=lname, M=M, N=N, K=K, A=A, B=B, ta=ta, tb=tb))
    return out


def folded_formats(t_a, t_b, prod=(5, 7, 15), acc=(4, 7, 7), rnd=0):
    """Biases of (E, M, b) formats given in real units, moved into code units:
    codes = real * 2^(t_a+t_b) for a product, and Q_{M,E,b}(2^-T y) = 2^-T Q_{M,E,b-T}(y),
    so the library is called with b - T.  Returns ((E,M,b',round), (E,M,b',round), T)."""
    T = t_a + t_b
    return (prod[0], prod[1], prod[2] - T, rnd), (acc[0], acc[1], acc[2] - T, rnd), T
