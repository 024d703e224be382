"""The hot path inside a captured HIP graph: every replay must equal the eager
result bit for bit, with eager work and synchronisations between the replays
and with the activations changed in place between them (the calls only enqueue
kernels; nothing in them is a memset node or a host-side wait)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [dd.MODE_FUSED, dd.MODE_SERIAL, dd.MODE_TWO_STREAMS])
@pytest.mark.parametrize("rfmt", ["fp16", "int4"])
def test_graph_replays_equal_eager(mode, rfmt):
    K, N, k = 2048, 1536, 41
    p = Problem(workloads.weights(90, 0, 0, K, N), 3, rfmt=rfmt, alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    d = p.device()
    ws = dd.Workspace(K, N, k)
    try:
        ws.set_mode(mode)
        xs = [workloads.x_gauss_outliers(90, 0, 0, s, K) for s in range(4)]
        x_dev = torch.from_numpy(xs[0]).cuda()
        y_dev = torch.full((N,), float("nan"), dtype=torch.float16, device="cuda")
        stream = torch.cuda.Stream()

        def call(s=None):
            dd.decdec_gemv(p.desc, x_dev, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], k, y_dev, ws, s)

        eager = []
        for x in xs:                                   # eager results first (also checks the residual pointer once)
            x_dev.copy_(torch.from_numpy(x))
            call()
            torch.cuda.synchronize()
            eager.append(y_dev.cpu().numpy().copy())
            y_ref, sc = p.reference(x, k)
            assert_parity(eager[-1], y_ref, ws.read_selection(k)[0], sc, what=f"eager mode {mode} {rfmt}")

        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            call(stream)
        for rep in range(3):
            for i, x in enumerate(xs):
                x_dev.copy_(torch.from_numpy(x))
                y_dev.fill_(float("nan"))
                scratch = torch.randn(1 << 16, device="cuda").sum().item()   # unrelated eager work in between
                assert np.isfinite(scratch)
                g.replay()
                torch.cuda.synchronize()
                got = y_dev.cpu().numpy()
                assert np.array_equal(got.view(np.uint16), eager[i].view(np.uint16)), (rep, i)
                assert np.array_equal(ws.read_selection(k)[0], oracle.topk_abs(x, k))
    finally:
        ws.close()
