"""The whole step captured in a HIP graph.  Every entry point only enqueues kernels on the stream it is given (no
allocation, no memset node, no host synchronisation), so a capture of the four calls replays the step; each replay is
checked against the eager calls on the same inputs, bit for bit, with new inputs, eager work and synchronisations
between the replays.  The eager path is the one the other tests hold against the oracle."""
import pytest
import torch

import gpu_util as gu
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu


def fresh_inputs(w, seed):
    ws = synth.Workload(w.name, w.batch, w.heads, w.seq_valid, w.head_dim, w.dtype, w.cube_gain, 0, w.budget_lo,
                        w.budget_hi, seed=seed)
    Q, K, V = synth.gen_qkv(ws)
    return gu.up(Q), gu.up(K), gu.up(V), torch.from_numpy(synth.gen_budgets(ws)).to(gu.DEV)


def test_step_replays_from_a_hip_graph(usv):
    w = synth.Workload("graph_ragged", 2, 3, 29 * 64 - 21, 128, "bf16", 2.0, 0, 2, 12, seed=4401)
    B, Hh, N, d, nb, kmax = w.batch, w.heads, w.seq_len, w.head_dim, w.nb, w.kmax
    q, k, v, budgets = fresh_inputs(w, 4401)
    S = torch.empty((B, Hh, nb, nb), dtype=torch.float32, device=gu.DEV)
    idx = torch.empty((B, Hh, nb, kmax), dtype=torch.int32, device=gu.DEV)
    cnt = torch.empty((B, Hh, nb), dtype=torch.int32, device=gu.DEV)
    wo = torch.empty((B, Hh, nb), dtype=torch.int32, device=gu.DEV)
    out = torch.empty((B, Hh, N, d), dtype=torch.float32, device=gu.DEV)
    lse = torch.empty((B, Hh, N), dtype=torch.float32, device=gu.DEV)

    def step():
        usv.block_scores_static(q, k, S, seq_valid=w.seq_valid)
        usv.select_topk(S, budgets=budgets, kmax=kmax, seq_valid=w.seq_valid, idx=idx, cnt=cnt)
        usv.attn_work_order(cnt, kmax, idx=idx, out=wo)
        usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out=out, lse=lse, work_order=wo)

    def eager(qe, ke, ve, be):
        Se = usv.block_scores(qe, ke, seq_valid=w.seq_valid)
        ie, ce = usv.select_topk(Se, budgets=be, kmax=kmax, seq_valid=w.seq_valid)
        oe, le = usv.block_sparse_attn(qe, ke, ve, ie, ce, seq_valid=w.seq_valid, out_dtype=torch.float32, return_lse=True)
        return Se, ie, ce, oe, le

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # the first call on a device looks the static array up: outside the capture
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    other = synth.Workload("graph_other", 1, 2, 7 * 64, 64, "bf16", 2.0, 3, seed=4402)
    for rep in range(4):
        qn, kn, vn, bn = fresh_inputs(w, 4410 + rep)
        for dst, src in ((q, qn), (k, kn), (v, vn), (budgets, bn)):
            dst.copy_(src)
        for t in (S, out, lse):
            t.fill_(float("nan"))
        idx.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        Se, ie, ce, oe, le = eager(qn, kn, vn, bn)
        torch.cuda.synchronize()
        what = f"replay {rep}"
        assert torch.equal(S.view(torch.int32), Se.view(torch.int32)), what
        assert torch.equal(idx, ie) and torch.equal(cnt, ce), what
        assert torch.equal(torch.sort(wo, dim=-1).values, torch.arange(nb, dtype=torch.int32, device=gu.DEV).expand_as(wo)), what
        nv = w.seq_valid  # rows past it are padding: unspecified
        assert torch.equal(out[:, :, :nv].view(torch.int32), oe[:, :, :nv].view(torch.int32)), what
        assert torch.equal(lse[:, :, :nv].view(torch.int32), le[:, :, :nv].view(torch.int32)), what
        # the program's own eager work between replays: another shape through the same entry points (it shares the
        # static array of stage 1 with the graph)
        Qo, Ko, Vo = synth.gen_qkv(other)
        qo, ko, vo = gu.up(Qo), gu.up(Ko), gu.up(Vo)
        So = torch.empty((other.batch, other.heads, other.nb, other.nb), dtype=torch.float32, device=gu.DEV)
        usv.block_scores_static(qo, ko, So, seq_valid=other.seq_valid)
        io, co = usv.select_topk(So, k=other.keep, seq_valid=other.seq_valid)
        usv.block_sparse_attn(qo, ko, vo, io, co, seq_valid=other.seq_valid)
        torch.cuda.synchronize()
