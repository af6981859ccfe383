"""The whole step (selection, operand build, the three products) recorded once as a HIP graph and replayed: the
library allocates nothing, clears nothing with memset calls and never synchronises, so a capture holds exactly its
kernels.  Every replay is compared bit for bit with the eager calls on the same inputs, with eager work and
synchronisations between the replays and inputs that change from replay to replay."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import TOL, TOL_DV, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K,T,dtype", [(768, 768, 77, 300, "bf16"), (128, 384, 40, 415, "bf16"),
                                           (100, 260, 31, 129, "f32")])
def test_step_replays_from_a_graph(M, N, K, T, dtype):
    D, L = max(M, N), min(M, N)
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(M + N + K)

    def draw():
        scores = rng.standard_normal((1, D)).astype(np.float32)
        values = (rng.standard_normal((K, L)) * 0.02).astype(np.float32)
        X = rng.standard_normal((T, M)).astype(np.float32)
        dY = rng.standard_normal((T, N)).astype(np.float32)
        if dtype == "bf16":
            values, X, dY = synth.round_to_bf16(values), synth.round_to_bf16(X), synth.round_to_bf16(dY)
        return scores, values, X, dY

    host = draw()
    d_scores = torch.from_numpy(host[0]).cuda()
    d_val, d_X, d_dY = (to_dev(a, dtype) for a in host[1:])
    d_off = torch.empty((1, K), dtype=torch.int32, device="cuda")
    out = {"Y": torch.empty((T, N), dtype=tdtype, device="cuda"), "dX": torch.empty((T, M), dtype=tdtype, device="cuda"),
           "dV": torch.empty((K, L), dtype=torch.float32, device="cuda")}
    ws = dd.Workspace()
    use_prepared = dtype == "bf16"
    prepared = [dd.dd_prepare(torch.zeros(K, dtype=torch.int32, device="cuda"), d_val, M, N)] if use_prepared else [None]

    def step():
        dd.dd_select_diagonals(d_scores, K, offsets_out=d_off, ws=ws)
        if use_prepared:
            dd.dd_prepare(d_off[0], d_val, M, N, prepared=prepared[0])
            dd.dd_fwd(d_X, None, None, N, Y=out["Y"], prepared=prepared[0])
            dd.dd_bwd_input(d_dY, None, None, M, dX=out["dX"], prepared=prepared[0])
        else:
            dd.dd_fwd(d_X, d_off[0], d_val, N, Y=out["Y"], ws=ws)
            dd.dd_bwd_input(d_dY, d_off[0], d_val, M, dX=out["dX"], ws=ws)
        dd.dd_bwd_weight(d_X, d_dY, d_off[0], dValues=out["dV"], ws=ws)

    step()  # every buffer the step needs exists before the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for replay in range(4):
        if replay:  # new inputs in the same buffers
            host = draw()
            d_scores.copy_(torch.from_numpy(host[0]).cuda())
            for dst, a in zip((d_val, d_X, d_dY), host[1:]):
                dst.copy_(to_dev(a, dtype))
        for t in out.values():
            t.fill_(float("nan"))
        d_off.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = {k: v.clone() for k, v in out.items()}
        got_off = d_off.clone()
        for t in out.values():
            t.zero_()
        step()  # eager, on the same inputs
        torch.cuda.synchronize()
        assert torch.equal(got_off, d_off), f"replay {replay}"
        for k in out:
            assert torch.equal(got[k].view(torch.int32 if got[k].dtype == torch.float32 else torch.int16),
                               out[k].view(torch.int32 if got[k].dtype == torch.float32 else torch.int16)), (replay, k)
        offsets = orc.select(host[0], K)[0]
        assert np.array_equal(got_off[0].cpu().numpy(), offsets)
        assert rel_err(to_host(got["Y"]), orc.fwd(host[2], offsets, host[1], N)) <= TOL[dtype]
        assert rel_err(to_host(got["dX"]), orc.bwd_input(host[3], offsets, host[1], M)) <= TOL[dtype]
        assert rel_err(to_host(got["dV"]), orc.bwd_weight(host[2], host[3], offsets)) <= TOL_DV
