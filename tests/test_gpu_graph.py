"""GPU: every device entry point can be captured into a HIP graph (no allocation, no synchronisation, no
memset nodes inside the library) and every replay reproduces the eager results, with unrelated eager work
and synchronisations between the replays."""
import pytest
import torch

from paper_2305_18513_amd import binding as sf
from tests.gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def test_captured_calls_replay_to_the_eager_results():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(0)
    n, rows, cols, k, H = 300_000, 900, 384, 38, 768
    x = torch.randn(n, generator=g, device="cuda") * 2
    p = torch.softmax(torch.randn(rows, cols, generator=g, device="cuda"), dim=1)
    lnx = torch.randn(640, H, generator=g, device="cuda")
    gamma, beta = torch.rand(H, generator=g, device="cuda") + 0.5, torch.rand(H, generator=g, device="cuda")
    dy = torch.randn(640, H, generator=g, device="cuda")
    w_prev = [torch.randn(m, generator=g, device="cuda") * 0.02 + 0.05 for m in (1000, 70000, 16384)]
    w_cur = [w + 1e-4 * torch.randn(w.numel(), generator=g, device="cuda") for w in w_prev]
    numel = [w.numel() for w in w_prev]

    out = {
        "codes": torch.empty(sf.packed_bytes(n, 4), dtype=torch.uint8, device="cuda"),
        "scales": torch.empty(sf.num_blocks(n, 64), device="cuda"),
        "deq": torch.empty(n, device="cuda"),
        "gelu_y": torch.empty(n, device="cuda"),
        "gelu_dx": torch.empty(n, device="cuda"),
        "vals": torch.empty(rows, k, device="cuda"),
        "idx": torch.empty(rows, k, dtype=torch.uint16, device="cuda"),
        "counts": torch.empty(rows, dtype=torch.int32, device="cuda"),
        "dense": torch.empty(rows, cols, device="cuda"),
        "sm_p": torch.empty(rows, cols, device="cuda"),
        "sm_v": torch.empty(rows, k, device="cuda"),
        "sm_i": torch.empty(rows, k, dtype=torch.uint16, device="cuda"),
        "gv": torch.empty(n // 10, device="cuda"),
        "gi": torch.empty(n // 10, dtype=torch.int32, device="cuda"),
        "gptr": torch.empty(sf.global_tile_ptr_len(n), dtype=torch.int32, device="cuda"),
        "gback": torch.empty(n, device="cuda"),
        "ln_y": torch.empty(640, H, device="cuda"),
        "mean": torch.empty(640, device="cuda"),
        "rstd": torch.empty(640, device="cuda"),
        "lv": torch.empty(640 * H // 10, device="cuda"),
        "li": torch.empty(640 * H // 10, dtype=torch.int32, device="cuda"),
        "lrow": torch.empty(641, dtype=torch.int32, device="cuda"),
        "ln_dx": torch.empty(640, H, device="cuda"),
        "ln_dx_dense": torch.empty(640, H, device="cuda"),
        "dgamma": torch.empty(H, device="cuda"),
        "dbeta": torch.empty(H, device="cuda"),
        "d": torch.empty(3, device="cuda"),
        "sm_ds": torch.empty(rows, cols, device="cuda"),
        "lq_y": torch.empty(640, H, device="cuda"),
        "lq_codes": torch.empty(640 * H // 2, dtype=torch.uint8, device="cuda"),
        "lq_scales": torch.empty(640 * H // 64, device="cuda"),
        "lq_dx": torch.empty(640, H, device="cuda"),
        "d_apply": torch.empty(3, device="cuda"),
        "w0": torch.empty_like(w_prev[0]), "w1": torch.empty_like(w_prev[1]), "w2": torch.empty_like(w_prev[2]),
    }
    w_apply = [out["w0"], out["w1"], out["w2"]]
    upd = [c - q for q, c in zip(w_prev, w_cur)]
    ws_delta = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    ws_apply = torch.empty_like(ws_delta)
    sf.layer_delta_plan(w_apply, upd, ws_apply)
    ws_pg = torch.empty(sf.prune_global_workspace(n), dtype=torch.uint8, device="cuda")
    ws_ln = torch.empty(sf.prune_global_workspace(640 * H), dtype=torch.uint8, device="cuda")
    ws_par = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    sf.layer_delta_plan(w_prev, w_cur, ws_delta)

    def calls():
        o = out
        sf.quant_pack(x, sf.Q_BLOCK, 4, 64, 0, o["codes"], o["scales"])
        sf.dequant_unpack(o["codes"], o["scales"], sf.Q_BLOCK, 4, 64, 0, o["deq"])
        sf.gelu_quant_pack(x, sf.Q_BLOCK, 4, 64, 0, o["gelu_y"], o["codes"], o["scales"])
        sf.gelu_backward_dequant(o["codes"], o["scales"], sf.Q_BLOCK, 4, 64, 0, o["deq"], o["gelu_dx"])
        sf.prune_scores(p, k, sf.PRUNE_TOPK, 0.0, o["vals"], o["idx"], o["counts"])
        sf.restore_scores(o["vals"], o["idx"], o["counts"], o["dense"])
        sf.softmax_prune(p, k, o["sm_p"], o["sm_v"], o["sm_i"])
        sf.prune_global(x, n // 10, o["gv"], o["gi"], True, o["gptr"], ws_pg)
        sf.restore_global(o["gv"], o["gi"], n // 10, o["gback"], o["gptr"])
        sf.layernorm_forward(lnx, gamma, beta, 1e-5, o["ln_y"], o["mean"], o["rstd"])
        sf.prune_global_standardized(lnx, o["mean"], o["rstd"], 640 * H // 10, o["lv"], o["li"], True, None, o["lrow"],
                                     ws_ln)
        sf.layernorm_backward_pruned(o["lv"], o["li"], o["lrow"], 640 * H // 10, o["rstd"], gamma, dy, o["ln_dx"])
        sf.layernorm_backward(lnx, o["mean"], o["rstd"], gamma, dy, o["ln_dx_dense"])
        sf.layernorm_param_grads(lnx, o["mean"], o["rstd"], dy, o["dgamma"], o["dbeta"], ws_par)
        sf.layer_delta_run(numel, sf.F32, sf.F32, False, 0.0, o["d"], ws_delta)
        sf.softmax_backward_pruned(o["vals"], o["idx"], None, p, o["sm_ds"])
        sf.layernorm_forward_quant_pack(lnx, gamma, beta, 1e-5, 4, 64, o["lq_y"], o["mean"], o["rstd"], o["lq_codes"],
                                        o["lq_scales"])
        sf.layernorm_backward_dequant(o["lq_codes"], o["lq_scales"], 4, 64, o["mean"], o["rstd"], gamma, dy, o["lq_dx"])
        for dst, src in zip(w_apply, w_prev):                      # the update is applied to a fresh copy every time
            dst.copy_(src)
        sf.layer_delta_apply_run(numel, sf.F32, sf.F32, 0.0, o["d_apply"], ws_apply)

    calls()
    torch.cuda.synchronize()
    eager = {name: t.clone() for name, t in out.items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    # pointer checks stay on: the library sees that the call's stream is capturing and skips the look-ups itself
    with torch.cuda.graph(graph, stream=side):
        calls()

    scratch = torch.empty(1 << 22, device="cuda")
    for replay in range(4):
        for t in out.values():
            t.view(torch.uint8).fill_(0xCD)                        # stale outputs must not survive a replay
        scratch.normal_()                                          # unrelated eager work between replays
        _ = float(scratch.sum())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in out.items():
            assert torch.equal(t.view(torch.uint8), eager[name].view(torch.uint8)), "replay %d: %s" % (replay, name)
