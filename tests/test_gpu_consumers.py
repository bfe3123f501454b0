"""GPU parity of the packed-format consumers (full-matrix decompression, quantized-matrix times vector)
against the float64 oracle.  Decompression is compared bit for bit: the kernel's value is the float32 product
scale * (code - zero), which the oracle's float64 product rounds to exactly; for float16 output it is rounded
once more.  The matrix-vector product accumulates n float32 terms per row: with unit roundoff u = 6e-8 a sum
of n terms in any order is within about (log2 n + 3) u * sum|terms| of the exact one when it is formed as a
tree of partial sums (64 lanes x 32 columns x n/2048 segments here), i.e. < 2e-6 * sum|q x| at n = 49152;
the test allows 1e-5 * sum|q x| per row."""
import numpy as np
import pytest
import torch

from oracle import gptq_oracle as O

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _random_layer(r, n, bits, group, seed, ternary=False):
    rng = np.random.default_rng(seed)
    hi = 3 if ternary else (1 << bits)
    codes = rng.integers(0, hi, size=(r, n))
    G = n // group if group else 1
    scale = (rng.uniform(0.5, 2.0, size=(r, G)) * 0.01).astype(np.float32)
    zero = (np.ones((r, G)) if ternary else rng.integers(0, 1 << bits, size=(r, G))).astype(np.int32)
    return codes, scale, zero


CASES = [
    # bits, group, r, n, ternary
    (3, 0, 37, 1000, False),          # ragged n (not a multiple of 32), rows not a multiple of 8
    (3, 0, 64, 4096, False),
    (4, 0, 9, 2500, False),
    (2, 0, 16, 6144 + 32, False),     # more than one 2048-column segment per wavefront, ragged last segment
    (2, 128, 24, 2048, False),
    (4, 32, 8, 1024, False),
    (3, 64, 5, 640, False),
    (2, 8, 13, 520, True),            # ternary at group size 8
    (4, 16, 3, 272, False),
    (3, 1024, 10, 3072, False),
    (3, 0, 1, 1, False),
]


@pytest.mark.parametrize("bits,group,r,n,ternary", CASES)
def test_consumers_match_oracle(bits, group, r, n, ternary):
    import paper_2210_17323_amd as g
    _say(f"consumers bits={bits} group={group} r={r} n={n} ternary={ternary}")
    codes, scale, zero = _random_layer(r, n, bits, group, 7 * bits + n, ternary)
    words = O.pack_codes(codes, bits)
    Q64 = O.dequantize_packed(words, n, bits, scale, zero, group)
    wd = torch.from_numpy(words.view(np.int32)).cuda()
    sd, zd = torch.from_numpy(scale).cuda(), torch.from_numpy(zero).cuda()
    for dt in (torch.float32, torch.float16):
        out = torch.full((r, n + 3), 7.0, dtype=dt, device="cuda")[:, :n]      # a pitch that breaks 16-byte alignment
        g.gptq_dequantize_packed(wd, n, bits, sd, zd, group, out)
        want = Q64.astype(np.float32) if dt == torch.float32 else Q64.astype(np.float32).astype(np.float16)
        assert np.array_equal(out.cpu().numpy(), want), dt
        out2 = torch.empty((r, (n + 7) // 8 * 8), dtype=dt, device="cuda")[:, :n]   # aligned rows: the vector path
        g.gptq_dequantize_packed(wd, n, bits, sd, zd, group, out2)
        assert np.array_equal(out2.cpu().numpy(), want), dt
    rng = np.random.default_rng(n)
    for dt in (torch.float16, torch.float32):
        x = torch.from_numpy(rng.normal(size=n).astype(np.float32)).to(dt).cuda()
        y = torch.full((r,), 3.0, dtype=torch.float32, device="cuda")
        g.gptq_matvec_packed(wd, n, bits, sd, zd, group, x, y)
        x64 = x.double().cpu().numpy()
        want = O.matvec_packed(words, n, bits, scale, zero, group, x64)
        bound = 1e-5 * (np.abs(Q64) @ np.abs(x64)) + 1e-30
        err = np.abs(y.double().cpu().numpy() - want)
        _say(f"  matvec {dt}: max err / bound = {(err / bound).max():.3f}")
        assert np.all(err <= bound)
        if dt == torch.float16:             # a vector that does not start on a 16-byte boundary: same result
            xo = torch.empty(n + 1, dtype=dt, device="cuda")[1:]
            xo.copy_(x)
            y2 = torch.full((r,), 5.0, dtype=torch.float32, device="cuda")
            g.gptq_matvec_packed(wd, n, bits, sd, zd, group, xo, y2)
            assert np.all(np.abs(y2.double().cpu().numpy() - want) <= bound)


def test_consumers_after_the_solver():
    # the layer Alg. 1 produced, packed: decompression gives the solver's own Wq, the product gives Wq x
    import paper_2210_17323_amd as g
    from paper_2210_17323_amd import solver as S
    from workloads import configs
    lay = configs.scaled_twin(configs.config4()[0], 512, r=96, m=4096)      # 2-bit, group 128
    W, X = configs.materialize(lay, "cuda")
    H = S.new_hessian(lay.n)
    S.accumulate(H, X)
    U = S.cholesky_inverse(H, lay.percdamp)
    res = S.quantize(W, U, lay.bits, lay.grid, lay.block, lay.group, want_Wq=True, pack=True)
    out = torch.empty((lay.r, lay.n), dtype=torch.float32, device="cuda")
    g.gptq_dequantize_packed(res.packed, lay.n, lay.bits, res.scales, res.zeros, lay.group, out)
    assert torch.equal(out, res.Wq)
    x = torch.randn(lay.n, device="cuda", dtype=torch.float16)
    y = torch.empty(lay.r, dtype=torch.float32, device="cuda")
    g.gptq_matvec_packed(res.packed, lay.n, lay.bits, res.scales, res.zeros, lay.group, x, y)
    want = res.Wq.double() @ x.double()
    assert torch.allclose(y.double(), want, rtol=0, atol=float(1e-5 * (res.Wq.double().abs() @ x.double().abs()).max()))


def test_consumers_full_size_fc2_shape():
    # OPT-175B fc2 at 3 bits (12288 x 49152): sampled rows against the oracle
    import paper_2210_17323_amd as g
    r, n, bits = 12288, 49152, 3
    gen = torch.Generator(device="cuda").manual_seed(11)
    codes = torch.randint(0, 8, (r, n), dtype=torch.uint8, device="cuda", generator=gen)
    words = torch.empty((r, g.packed_words_per_row(n, bits)), dtype=torch.int32, device="cuda")
    g.gptq_pack(codes, bits, words)
    scale = (torch.rand((r, 1), device="cuda", generator=gen) * 0.01 + 0.005).float()
    zero = torch.randint(0, 8, (r, 1), dtype=torch.int32, device="cuda", generator=gen)
    x = torch.randn(n, device="cuda", generator=gen).half()
    y = torch.empty(r, dtype=torch.float32, device="cuda")
    g.gptq_matvec_packed(words, n, bits, scale, zero, 0, x, y)
    out = torch.empty((r, n), dtype=torch.float16, device="cuda")
    g.gptq_dequantize_packed(words, n, bits, scale, zero, 0, out)
    rows = np.array([0, 7, 8, 4099, 12287])
    wh = words[rows].cpu().numpy().view(np.uint32)
    assert np.array_equal(wh, O.pack_codes(codes[rows].cpu().numpy(), bits))
    sc, zr = scale[rows].cpu().numpy(), zero[rows].cpu().numpy()
    Q64 = O.dequantize_packed(wh, n, bits, sc, zr, 0)
    assert np.array_equal(out[rows].cpu().numpy(), Q64.astype(np.float32).astype(np.float16))
    x64 = x.double().cpu().numpy()
    want = O.matvec_packed(wh, n, bits, sc, zr, 0, x64)
    err = np.abs(y[rows].double().cpu().numpy() - want)
    bound = 1e-5 * (np.abs(Q64) @ np.abs(x64))
    _say(f"  fc2-shape matvec: max err / bound = {(err / bound).max():.3f}")
    assert np.all(err <= bound)


def test_consumers_empty_inputs():
    import paper_2210_17323_amd as g
    L = g.lib()
    y = torch.full((5,), 2.0, dtype=torch.float32, device="cuda")
    assert L.gptq_matvec_packed(None, 0, 5, 0, 3, None, None, 0, None, 0, y.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert torch.equal(y, torch.zeros(5, device="cuda"))               # an empty sum
    assert L.gptq_matvec_packed(None, 0, 0, 64, 3, None, None, 0, None, 0, None, None) == 0
    assert L.gptq_dequantize_packed(None, 0, 0, 64, 3, None, None, 0, None, 0, 64, None) == 0
