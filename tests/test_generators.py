"""The seeded input generators: determinism, tiling consistency, distribution sanity."""
import numpy as np
import torch

from workloads import configs, generators as g


def test_mix64_matches_big_integer_arithmetic():
    xs = [0, 1, 2, 12345678901234567, (1 << 63) + 5, (1 << 64) - 1]
    t = torch.tensor([g._s64(x) for x in xs], dtype=torch.int64)
    got = g._mix64(t).numpy().view(np.uint64)
    want = np.array([g.mix64_int(x) for x in xs], dtype=np.uint64)
    assert (got == want).all()


def test_tiles_agree_with_whole():
    whole = g.normal_tile(7, 3, 100, 0, 50, 0, 100)
    part = g.normal_tile(7, 3, 100, 10, 20, 30, 40)
    assert torch.equal(whole[10:30, 30:70], part)
    other = g.normal_tile(7, 4, 100, 0, 50, 0, 100)
    assert not torch.equal(whole, other)


def test_normal_moments():
    z = g.normal_tile(1, 1, 2000, 0, 500, 0, 2000).double()
    assert abs(z.mean().item()) < 5e-3
    assert abs(z.var().item() - 1.0) < 5e-3
    assert z.abs().max().item() <= 6.0
    kurt = (z ** 4).mean().item() / z.var().item() ** 2
    assert abs(kurt - 2.9) < 0.03          # Irwin-Hall(12): excess kurtosis -0.1


def test_config_layers_and_activations():
    lay = configs.config1()[0]
    W = lay.weights()
    X = lay.x.tile()
    assert W.shape == (256, 256) and W.dtype == torch.float32
    assert X.shape == (256, 4096) and X.dtype == torch.float32
    assert abs(W.std().item() - 0.02) < 1e-3
    rms = X.double().pow(2).mean(dim=1).sqrt()
    assert int((rms > 10).sum()) == 4       # the four x20 outlier channels
    fc2 = configs.scaled_twin(configs.config3()[1], 512, r=64)
    Xr = fc2.x.tile(ncols=2048)
    assert Xr.dtype == torch.float16 and (Xr >= 0).all()
    assert abs((Xr == 0).double().mean().item() - 0.6) < 0.01
    twin = configs.scaled_twin(configs.config2()[0], 512)
    assert twin.x.m == 8192 and twin.r == 512
    s = twin.x.scales()
    assert s.shape == (512,) and s.dtype == torch.float32
    assert abs(np.log(np.sort(s.numpy())[:-1]).std() - 0.5) < 0.06
    # a tile of a big layer can be produced alone
    big = configs.config3()[1]
    t = big.x.tile(row0=49000, nrows=4, col0=262000, ncols=8)
    assert t.shape == (4, 8)
