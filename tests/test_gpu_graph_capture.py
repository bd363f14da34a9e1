"""HIP-graph capture of the entry points built around the aggregation: none of them allocates or
synchronises the host, so a sequence of them can be captured once and replayed; every replay
(with eager work in between) must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

import blockgen as bg
from paper_2409_14939_amd import binding as B
from gpu_util import dev_i32

pytestmark = pytest.mark.gpu


def test_update_idmap_match_edge_capture_and_replay():
    rng = np.random.default_rng(5)
    blk = bg.random_block(rng, 700, 1500, 5.0, empty_frac=0.1, hub_rows=2, hub_deg=1300)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    feat, N = 100, 48
    f32 = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32)).cuda()
    X, G, W, b, dY = f32(blk.num_src, feat), f32(blk.num_dst, feat), f32(feat, N), f32(N), f32(blk.num_dst, N)
    score = f32(blk.num_edges)
    dst_gid, nbr_gid = (torch.from_numpy(a).cuda() for a in bg.hop_global_ids(blk, 3))
    prev_gid = torch.from_numpy(rng.permutation(4000)[:1800].astype(np.int64)).cuda()
    new_gid = torch.from_numpy(rng.permutation(4000)[:1500].astype(np.int64)).cuda()
    X_prev, X_load = f32(1800, feat), f32(1500, feat)
    print("case graph capture of update / idmap / match / edge entry points", flush=True)

    E, nd, ns = blk.num_edges, blk.num_dst, blk.num_src
    u8 = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
    i32 = lambda n: torch.empty(n, dtype=torch.int32, device="cuda")
    O = dict(
        H=G, Y=torch.empty(nd, N, device="cuda"), dH=torch.empty(nd, feat, device="cuda"),
        dW=torch.empty(feat, N, device="cuda"), db=torch.empty(N, device="cuda"),
        local=i32(E), uniq=torch.empty(nd + E, dtype=torch.int64, device="cuda"), res=i32(2),
        src_row=i32(1500), load_pos=i32(1500), load_gid=torch.empty(1500, dtype=torch.int64, device="cuda"), mres=i32(2),
        X_new=torch.empty(1500, feat, device="cuda"),
        alpha=torch.empty(E, device="cuda"), gw=torch.empty(E, device="cuda"), gs=torch.empty(E, device="cuda"),
        sc=torch.empty(E, device="cuda"), g_el=torch.empty(nd, device="cuda"), g_er=torch.empty(ns, device="cuda"),
    )
    el, er = f32(nd), f32(ns)
    plan = B.fastgl_block_plan_create(ip, ix, ns, B.PLAN_ALL | B.PLAN_PERM)
    ws_u, ws_i = u8(B.fastgl_update_bwd_workspace_bytes(nd, feat, N)), u8(B.fastgl_idmap_workspace_bytes(nd, E))
    ws_m, ws_e = u8(B.fastgl_match_workspace_bytes(1800, 1500)), u8(B.fastgl_edge_workspace_bytes(nd, E))
    # the number of rows Match asks to load is fixed by the inputs; learn it once, eagerly
    _, _, _, r = B.fastgl_match(prev_gid, new_gid, workspace=ws_m)
    n_load = int(r.cpu()[0])

    def step():
        B.fastgl_update_fwd(O["H"], W, b, True, O["Y"])
        B.fastgl_update_bwd(O["H"], W, O["Y"], dY, True, want=(), dH=O["dH"], dW=O["dW"], db=O["db"], workspace=ws_u)
        B.fastgl_idmap(dst_gid, nbr_gid, "ordered", O["local"], O["uniq"], O["res"], ws_i)
        B.fastgl_match(prev_gid, new_gid, O["src_row"], O["load_pos"], O["load_gid"], O["mres"], ws_m)
        B.fastgl_assemble_rows(X_prev, X_load, O["src_row"], n_load, out=O["X_new"])
        B.fastgl_edge_softmax_fwd(ip, score, O["alpha"], ws_e)
        B.fastgl_edge_weight_grad(ip, ix, ns, "sum", X, G, grad_w=O["gw"], workspace=ws_e)
        B.fastgl_edge_softmax_bwd(ip, O["alpha"], O["gw"], O["gs"], ws_e)
        B.fastgl_edge_score_fwd(ip, ix, el, er, 0.2, O["sc"])
        B.fastgl_edge_score_bwd(ip, ix, el, er, 0.2, O["gs"], plan=plan, grad_el=O["g_el"], grad_er=O["g_er"])

    outs = ["Y", "dH", "dW", "db", "local", "res", "src_row", "load_pos", "mres", "X_new", "alpha", "gw", "gs", "sc", "g_el", "g_er"]
    for k in outs:                                       # entries no call writes (the tail of load_pos) compare as zeros
        O[k].zero_()
    step()
    torch.cuda.synchronize()
    ref = {k: O[k].clone() for k in outs}
    U, nl = int(O["res"].cpu()[0]), n_load
    ref_uniq, ref_lgid = O["uniq"][:U].clone(), O["load_gid"][:nl].clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for k in outs:                                   # eager work between replays: wipe every output
            O[k].zero_()
        for wsx in (ws_u, ws_i, ws_m, ws_e):
            wsx.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(O[k], ref[k]), (rep, k)
        assert torch.equal(O["uniq"][:U], ref_uniq) and torch.equal(O["load_gid"][:nl], ref_lgid), rep
