"""The entry points can be captured into a HIP graph: they allocate nothing, pass their descriptors by
value and record kernel launches only.  Every replay must reproduce the eager results bit for bit."""
import pytest
import torch

import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, ensure_built

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def test_forward_backward_and_linear_entry_points_replay_from_a_graph():
    fmt, step = gws.FMT_FP8_E4M3, 11
    shapes = [(768, 768), (96, 320), (40, 50)]
    descs, outs = [], []
    for i, (r, c) in enumerate(shapes):
        t = synth.make_tensor(700 + i, r, c, ld=(c + 7) // 8 * 8, device=DEV)
        nbr, nbc = synth.n_blocks(r, c)
        w_hat, scale, dbt = torch.zeros_like(t["w"]), torch.zeros(nbr, nbc, device=DEV), torch.zeros(nbr, nbc, device=DEV)
        dw = torch.zeros_like(t["g"])
        descs.append(gws.TensorDesc(rows=r, cols=c, seed=gws.gws_derive_seed(9, i), w=t["w"], w_hat=w_hat, bt=t["bt"],
                                    scale=scale, g=t["g"], dw=dw, dbt=dbt, ld=t["w"].stride(0)))
        outs += [w_hat, scale, dbt, dw]
    # a sampled-weight linear on the large tile (sampling kernel + GEMM), and the same with w_hat staged in a workspace
    M, K, N = 512, 256, 512
    x = synth.make_activation(710, M, K, device=DEV)
    tl = synth.make_tensor(711, K, N, bt=6.0, device=DEV, with_grad=False)
    lw_hat, lscale = torch.zeros_like(tl["w"]), torch.zeros(K // 32, N // 32, device=DEV)
    y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    dlin = gws.TensorDesc(rows=K, cols=N, seed=5, w=tl["w"], w_hat=lw_hat, bt=tl["bt"], scale=lscale)
    outs += [lw_hat, lscale, y]
    dbare = gws.TensorDesc(rows=K, cols=N, seed=5, w=tl["w"], bt=tl["bt"])
    ws = torch.zeros(gws.gws_linear_fwd_workspace_bytes(dbare), dtype=torch.uint8, device=DEV)
    y3 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    outs += [ws, y3]
    # the plain GEMM with the sampling of another weight riding in its launch
    y2 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    tn = synth.make_tensor(712, 768, 768, device=DEV, with_grad=False)
    n_hat, n_scale = torch.zeros_like(tn["w"]), torch.zeros(24, 24, device=DEV)
    dnext = gws.TensorDesc(rows=768, cols=768, seed=6, w=tn["w"], w_hat=n_hat, bt=tn["bt"], scale=n_scale)
    outs += [y2, n_hat, n_scale]
    # the weight gradient with dL/db_t, one kernel and with the tokens split through a workspace
    dy = (synth.make_activation(713, 1024, N, device=DEV).float() * 1e-3).to(torch.bfloat16)
    xb = synth.make_activation(714, 1024, K, device=DEV)
    gscale = torch.full((K // 32, N // 32), 1e-3, device=DEV)
    dgrad = [gws.TensorDesc(rows=K, cols=N, seed=7, scale=gscale, dw=torch.zeros(K, N, dtype=torch.bfloat16, device=DEV),
                            dbt=torch.zeros(K // 32, N // 32, device=DEV)) for _ in range(2)]
    gws_bytes = gws.gws_linear_bwd_w_workspace_bytes(dgrad[1], 1024)
    assert gws_bytes > 0
    gwork = torch.zeros(gws_bytes // 4, device=DEV)
    outs += [dgrad[0].dw, dgrad[0].dbt, dgrad[1].dw, dgrad[1].dbt]

    def run():
        gws.gws_linear_bwd_w(xb, dy, dgrad[0], step)
        gws.gws_linear_bwd_w_ws(xb, dy, dgrad[1], step, gwork)
        gws.gws_sample_fwd(descs, fmt, step)
        gws.gws_sample_bwd(descs, step)
        gws.gws_linear_fwd(x, dlin, y, fmt, step)
        gws.gws_linear_fwd_ws(x, dbare, y3, fmt, step, ws)
        gws.gws_gemm_bf16_sample_next(x, tl["w"], y2, dnext, fmt, step)

    run()                                      # eager reference (also the usual warm-up before a capture)
    torch.cuda.synchronize()
    ref = [o.clone() for o in outs]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        for o in outs:                         # eager work between the replays
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (o, r) in enumerate(zip(outs, ref)):
            assert torch.equal(o.view(torch.uint8), r.view(torch.uint8)), (replay, k)
        run()                                  # and an eager call of the same entry points in between
        torch.cuda.synchronize()
