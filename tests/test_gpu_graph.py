"""A whole layer solve captured in a HIP graph: Hessian, damped factorisation, Alg. 1 (the calls fork onto the library's
helper streams and join back with events) and packing, recorded once on a capturing stream and replayed several times
with the program's own eager work and synchronisations between the replays.  Every replay must give the bits of the same
calls made eagerly on the same inputs.  The library records no memset nodes (it clears with kernels), and the test clears
its Hessian with a fill kernel as well."""
import pytest
import torch

from workloads import configs

pytestmark = pytest.mark.gpu


class _Buffers:
    def __init__(self, g, r, n, t, dtype, bits):
        dev = "cuda"
        self.X = torch.empty((n, t), dtype=dtype, device=dev)
        self.W = torch.empty((r, n), dtype=dtype, device=dev)
        self.H = torch.empty((n, n), dtype=torch.float32, device=dev)
        self.hws = torch.empty(max(g.gptq_hessian_accumulate_workspace_bytes(n, t, dtype), 256), dtype=torch.uint8, device=dev)
        self.cws = torch.empty(g.gptq_damp_cholesky_workspace_bytes(n), dtype=torch.uint8, device=dev)
        self.qws = torch.empty(g.gptq_quantize_layer_workspace_bytes(r, n, 128, 0), dtype=torch.uint8, device=dev)
        self.info = torch.zeros(1, dtype=torch.int32, device=dev)
        self.codes = torch.empty((r, n), dtype=torch.uint8, device=dev)
        self.scales = torch.empty((r, 1), dtype=torch.float32, device=dev)
        self.zeros = torch.empty((r, 1), dtype=torch.int32, device=dev)
        self.half = torch.empty(r, dtype=torch.float64, device=dev)
        self.packed = torch.empty((r, g.packed_words_per_row(n, bits)), dtype=torch.int32, device=dev)
        self.bits = bits

    def solve(self, g):
        self.H.zero_()
        self.half.zero_()
        g.gptq_hessian_accumulate(self.H, self.X, self.hws)
        g.gptq_damp_cholesky(self.H, 0.01, self.cws, self.info)
        g.gptq_quantize_layer(self.W, self.H, self.bits, g.GPTQ_GRID_MINMAX, 128, 0, self.codes, self.scales, self.zeros, self.qws,
                              None, self.half, from_factor=True)
        g.gptq_pack(self.codes, self.bits, self.packed)

    def results(self):
        return [t.clone() for t in (self.H, self.codes, self.scales, self.zeros, self.half, self.packed, self.info)]


@pytest.mark.parametrize("forced_split", [False, True])
def test_layer_solve_replays_from_a_graph(forced_split):
    import paper_2210_17323_amd as g
    g.lib()
    r, n, t, bits = 512, 2304, 4000, 3           # three outer blocks: look-ahead on the helper streams in both solvers
    base = configs.scaled_twin(configs.config3()[1], n, r=r, m=t)
    inputs = []
    for shift in range(3):
        x = type(base.x)(**{**base.x.__dict__, "tensor_id": base.x.tensor_id + 10 * shift})
        lay = type(base)(**{**base.__dict__, "tensor_id": base.tensor_id + 10 * shift, "x": x})
        inputs.append((lay.x.tile().cuda(), lay.weights().cuda()))
    prev = g.gptq_set_split_min_tiles(1 if forced_split else 0)
    try:
        eager = _Buffers(g, r, n, t, inputs[0][0].dtype, bits)
        want = []
        for X, W in inputs:
            eager.X.copy_(X); eager.W.copy_(W)
            eager.solve(g)                       # also the warm-up that creates the library's helper streams and events
            torch.cuda.synchronize()
            want.append(eager.results())
        assert int(want[0][6]) == 0

        b = _Buffers(g, r, n, t, inputs[0][0].dtype, bits)
        b.X.copy_(inputs[0][0]); b.W.copy_(inputs[0][1])
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            b.solve(g)
        torch.cuda.synchronize()
        for rep, k in enumerate((0, 1, 2, 1, 0)):
            print(f"graph replay {rep}: inputs {k}, forced_split={forced_split}", flush=True)
            b.X.copy_(inputs[k][0]); b.W.copy_(inputs[k][1])
            for out in (b.codes, b.packed, b.scales):        # stale results of the previous replay must not pass
                out.fill_(0)
            scratch = torch.randn(1 << 20, device="cuda").sum().item()      # eager work and a synchronisation in between
            assert scratch == scratch
            graph.replay()
            torch.cuda.synchronize()
            got = b.results()
            for name, a, w in zip(("H", "codes", "scales", "zeros", "half_E2", "packed", "info"), got, want[k]):
                assert torch.equal(a, w), f"replay {rep} (inputs {k}): {name} differs from the eager result"
    finally:
        g.gptq_set_split_min_tiles(prev)


def test_helper_streams_can_be_released_and_come_back():
    # the library's only state between calls: released, the next call recreates it and gives the same bits
    import paper_2210_17323_amd as g
    g.lib()
    r, n, t, bits = 256, 2304, 3000, 4
    lay = configs.scaled_twin(configs.config3()[1], n, r=r, m=t)
    b = _Buffers(g, r, n, t, torch.float16, bits)
    b.X.copy_(lay.x.tile().cuda()); b.W.copy_(lay.weights().cuda())
    b.solve(g)
    torch.cuda.synchronize()
    want = b.results()
    g.gptq_release_thread_resources()
    g.gptq_release_thread_resources()              # a second release finds nothing and is a no-op
    for out in (b.codes, b.packed):
        out.fill_(0)
    b.solve(g)
    torch.cuda.synchronize()
    for name, a, w in zip(("R", "codes", "scales", "zeros", "half_E2", "packed", "info"), b.results(), want):
        assert torch.equal(a, w), name
