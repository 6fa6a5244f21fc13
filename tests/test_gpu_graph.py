"""The four calls of a pass enqueue kernels and event waits only (no allocation, no
synchronisation, no memset): a caller can record a whole pass into a HIP graph and replay it.
Every replay is compared with the eager pass on the same inputs, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest

import lq_synth
from tests import lq_harness as hx

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _lq():
    import paper_2407_10032_amd as lq
    lq.load()
    return lq


class _Pass:
    """Static buffers of one pass and the sequence of calls on them."""

    def __init__(self, lq, cfg, P):
        r, c, n = cfg.r, cfg.c, cfg.n_tokens
        self.lq, self.P = lq, P
        self.X = torch.empty((n, c), dtype=torch.float32, device="cuda")
        self.W = torch.empty((r, c), dtype=torch.float32, device="cuda")
        self.H = torch.empty((c, c), dtype=torch.float32, device="cuda")
        self.U = torch.empty((c, c), dtype=torch.float32, device="cuda")
        self.d = torch.empty(c, dtype=torch.float32, device="cuda")
        self.info = torch.zeros(1, dtype=torch.int32, device="cuda")
        self.grid = torch.empty(hx.grid_shape(P, r, c), dtype=torch.float32, device="cuda")
        self.Wq = torch.empty_like(self.W)
        self.codes = torch.empty((r, c), dtype=torch.uint8, device="cuda")
        self.loss = torch.empty(r, dtype=torch.float32, device="cuda")
        self.ws = lq.alloc_workspace(max(lq.lq_workspace_bytes(k, r, c, n, P) for k in range(4)))

    def run(self):
        lq, P = self.lq, self.P
        self.H.zero_()                      # a fill kernel, not a memset node
        self.Wq.copy_(self.W)
        lq.lq_hessian_accumulate(self.H, self.X, self.ws)
        lq.lq_cholesky_inv(self.H, P.damp, self.U, self.d, self.info, self.ws)
        lq.lq_fit_grid(self.W, self.d, P, self.grid, self.ws)
        lq.lq_quantize_layer(self.Wq, self.U, self.grid, P, self.codes, self.loss, self.ws)

    def results(self):
        torch.cuda.synchronize()
        return [t.clone() for t in (self.H, self.U, self.d, self.grid, self.Wq, self.codes, self.loss, self.info)]


@pytest.mark.parametrize("mode", ["nu", "aff"])
def test_a_pass_recorded_into_a_graph_replays_bit_identically(mode):
    lq = _lq()
    cfg = lq_synth.CONFIGS["c1"].scaled(r=384, c=512, n_tokens=2048)
    if mode == "aff":
        cfg = cfg.scaled(mode="aff", bits=4, group_size=128)
    P = hx.params_for(cfg)
    print(f"graph replay of a pass, {mode}", flush=True)
    ps = _Pass(lq, cfg, P)
    rng = np.random.default_rng(77)

    def new_inputs():
        ps.X.copy_(torch.from_numpy(rng.standard_normal((cfg.n_tokens, cfg.c)).astype(np.float32)))
        ps.W.copy_(torch.from_numpy((rng.standard_normal((cfg.r, cfg.c)) * 0.02).astype(np.float32)))

    new_inputs()
    ps.run()                                # eager once: one-time attribute calls, side streams
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ps.run()
    for rep in range(3):
        new_inputs()
        ps.run()
        eager = ps.results()
        for t in (ps.H, ps.U, ps.d, ps.grid, ps.Wq, ps.codes, ps.loss):
            t.fill_(0)                      # eager work between replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        replayed = ps.results()
        assert int(replayed[-1].item()) == 0
        for a, b in zip(eager, replayed):
            assert torch.equal(a, b), rep
