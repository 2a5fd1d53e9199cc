"""The three calls of the path recorded into a HIP graph (no allocation, no
host wait and no memset inside the library: its clears are kernels) and
replayed on changing inputs, every replay compared with the oracle; eager
work and synchronisations of the program run between the replays."""
import numpy as np
import pytest
import torch

from paper_2301_12187_amd import api, inputs
from gpu_common import compare, run_oracle

pytestmark = pytest.mark.gpu


# (the L=200 shape queues two gated pipelines and a device-side choice between them)
@pytest.mark.parametrize("cid,B", [(3, 24), (4, 6), (5, 2)])
def test_graph_replays_match_the_oracle(cid, B):
    cfg = inputs.CONFIGS[cid]
    dev = torch.device("cuda:0")
    batches = [inputs.make_batch(cfg, seed=s, B=B) for s in (31, 32, 33)]
    qi, qt = inputs.budgets(cfg, batches[0][2])
    Q = len(qi)
    buf = api.Buffers(B, cfg.L, cfg.P, Q)
    # static inputs of the graph
    Td = torch.zeros((B, cfg.L + 1, cfg.L + 1), dtype=torch.int32, device=dev)
    Id = torch.zeros((B, cfg.L + 1, cfg.L + 1), dtype=torch.float32, device=dev)
    qid = torch.from_numpy(qi).to(dev)
    qtd = torch.zeros((Q,), dtype=torch.int32, device=dev)

    def load(batch):
        T, I, base = batch
        _, qt_b = inputs.budgets(cfg, base)
        Td.copy_(torch.from_numpy(T))
        Id.copy_(torch.from_numpy(I))
        qtd.copy_(torch.from_numpy(qt_b))
        return T, I, qt_b

    load(batches[0])
    api.solve(Td, Id, qid, qtd, buf)                 # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.solve(Td, Id, qid, qtd, buf)
    for batch in (batches[1], batches[2], batches[0], batches[1]):
        T, I, qt_b = load(batch)
        buf.M.fill_(float("nan"))                    # eager work between replays
        buf.K.fill_(0xEE)
        buf.A.fill_(-9)
        buf.S.fill_(-9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        api.dpc_stage2_check(buf.workspace)
        g = dict(Topt=buf.Topt.cpu().numpy(), split=buf.split.cpu().numpy(), M=buf.M.cpu().numpy(),
                 K=buf.K.cpu().numpy(), A=buf.A.cpu().numpy(), S=buf.S.cpu().numpy(),
                 A_len=buf.A_len.cpu().numpy(), S_len=buf.S_len.cpu().numpy(),
                 obj=buf.obj.cpu().numpy(), lat=buf.lat.cpu().numpy(),
                 status=buf.status.cpu().numpy())
        compare(g, run_oracle(T, I, cfg.P, qi, qt_b, threads=8), cfg.L, f"replay of {cfg.name}")
