"""The library only enqueues kernels on the stream it is given: no allocation, no memset, no synchronisation,
and every counter a kernel uses is reset by the kernels themselves.  Two consequences are checked here on a
whole layer step (quantizer forward on W and X, the three index products, quantizer backward on X and W):
the step gives bit-identical results on a side stream, and it can be captured into a HIP graph whose
replays - with other work and fresh inputs in between - give what the eager calls give.
"""
import numpy as np
import pytest

import cdl_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu

M, N, K = 700, 300, 260          # several tiles, ragged in every dimension, K not a multiple of 16
W_SPEC = (-7, 15, 0.02, 1.0e4)   # lo, n_levels, delta, alpha
X_SPEC = (0, 16, 0.25, 64.0)


class Layer:
    def __init__(self, seed):
        import paper_2501_09849_amd as cdl
        torch = gu.torch_mod()
        self.cdl, self.torch = cdl, torch
        rng = np.random.default_rng(seed)
        f32, i8 = torch.float32, torch.int8
        self.W = gu.dev((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
        self.X = gu.dev(np.abs(rng.standard_normal((M, K))).astype(np.float32))
        self.G = gu.dev(rng.standard_normal((M, N)).astype(np.float32))
        self.out = {
            "Wi": gu.empty(N * K, i8), "Xi": gu.empty(M * K, i8),
            "Wsoft": gu.empty(N * K, f32), "Xsoft": gu.empty(M * K, f32),
            "margW": gu.empty(W_SPEC[1], f32), "margX": gu.empty(X_SPEC[1], f32),
            "scal": gu.empty(8, f32),
            "Y": gu.empty((M, N), f32), "acc": gu.empty((M, N), torch.int32),
            "dXh": gu.empty((M, K), f32), "dWh": gu.empty((N, K), f32),
            "dX": gu.empty(M * K, f32), "dW": gu.empty(N * K, f32),
        }
        need = max(cdl.quantize_workspace_bytes(M * K, 16), cdl.quantize_workspace_bytes(N * K, 15),
                   cdl.qgemm_fwd_workspace_bytes(M, N, K), cdl.qgemm_bwd_workspace_bytes(M, N, K))
        self.ws = gu.workspace(need)

    def run(self):
        cdl, o, s = self.cdl, self.out, self.out["scal"]
        cdl.cdl_quantize_fwd(self.W, N * K, *W_SPEC, o["Wi"], o["Wsoft"], o["margW"], s[0:1], self.ws)
        cdl.cdl_quantize_fwd(self.X, M * K, *X_SPEC, o["Xi"], o["Xsoft"], o["margX"], s[1:2], self.ws)
        cdl.cdl_qgemm_fwd(o["Xi"], o["Wi"], M, N, K, X_SPEC[2], W_SPEC[2], o["acc"], o["Y"], self.ws)
        cdl.cdl_qgemm_bwd(self.G, o["Xi"], o["Wi"], M, N, K, X_SPEC[2], W_SPEC[2], o["dXh"], o["dWh"], self.ws)
        cdl.cdl_quantize_bwd(self.X, o["dXh"], M * K, *X_SPEC, o["dX"], s[4:5], s[5:6], self.ws)
        cdl.cdl_quantize_bwd(self.W, o["dWh"], N * K, *W_SPEC, o["dW"], s[2:3], s[3:4], self.ws)

    def scramble(self):
        """Other work on the same buffers between runs: every output is overwritten with junk."""
        for name, t in self.out.items():
            if t.dtype.is_floating_point:
                t.fill_(float("nan"))
            else:
                t.fill_(77)
        self.out["scal"].zero_()

    def results(self):
        self.torch.cuda.synchronize()
        return {k: v.detach().cpu().numpy().copy() for k, v in self.out.items()}


def same(a, b):
    for k in a:
        x, y = a[k], b[k]
        if k == "scal":
            x, y = x[:6], y[:6]
        assert np.array_equal(x, y, equal_nan=False), k


def test_step_on_a_side_stream_is_bit_identical():
    torch = gu.torch_mod()
    layer = Layer(seed=5)
    layer.scramble()
    layer.run()
    want = layer.results()
    side = torch.cuda.Stream()
    layer.scramble()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        layer.run()
    side.synchronize()
    same(layer.results(), want)


def test_step_replayed_from_a_graph_matches_eager_every_time():
    torch = gu.torch_mod()
    layer = Layer(seed=6)
    # warm-up on a side stream, then capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.run()
    rng = np.random.default_rng(9)
    for rep in range(4):
        if rep:
            # fresh inputs in the same buffers: the graph must read them, and size the limbs from them again
            layer.X.copy_(gu.dev(np.abs(rng.standard_normal((M, K))).astype(np.float32)))
            layer.G.copy_(gu.dev((rng.standard_normal((M, N)) * 10.0 ** rep).astype(np.float32)))
        layer.scramble()
        layer.run()
        want = layer.results()
        layer.scramble()
        torch.cuda.synchronize()
        graph.replay()
        same(layer.results(), want)
