"""The entry points under HIP graph capture (run with -m gpu on an MI355X).

ksa_prefill_fwd and ksa_prefill_bwd with caller workspaces and ksa_decode_fwd_static (no workspace at all) enqueue
kernels only: no allocation, no memset, no synchronisation.  A caller can therefore capture them into a graph.  The
graph is replayed several times with the program's own eager work and synchronisations in between, on changing input
data, and every replay is compared bit for bit with the eager calls on the same data.
"""
import sys

import pytest
import torch

import paper_2604_24432_amd as K
from paper_2604_24432_amd import synth

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_prefill_backward_and_static_decode_replay_from_a_graph():
    cfg = synth.KsaConfig("graph", 1, 8, 2, 128, 2048, 64, 8, 1, seed=6001)
    p = K.make_params(cfg.batch, cfg.n_text, cfg.chunk_len, cfg.n_summary, cfg.window_chunks, cfg.n_q_heads,
                      cfg.n_kv_heads, cfg.head_dim)
    lay = K.ksa_build_layout(p)
    lay.upload()                                   # the schedule's device copy: allocated here, not under capture
    data = []
    for i in range(3):                             # three sets of inputs, one per replay
        c = cfg.scaled(seed=cfg.seed + i)
        data.append([x.cuda() for x in synth.make_prefill_inputs(c)] + [synth.make_upstream_gradient(c).cuda()])
    q, k, v, g = (x.clone() for x in data[0])
    o, dq = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(k)
    lse = torch.empty((cfg.batch, cfg.n_q_heads, cfg.aug_len), dtype=torch.float32, device="cuda")
    ws = torch.empty(K.prefill_workspace_bytes(lay), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(K.prefill_bwd_workspace_bytes(lay), dtype=torch.uint8, device="cuda")

    # decode: four sequences on a 40-chunk context
    B, n_cap = 4, 64 * 40
    pd = K.make_params(B, n_cap, 64, 8, 1, 8, 2, 128)
    s_cap, rows = K.cache_geometry(pd)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    qd_all = [torch.randn((B, 8, 128), device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3)]
    kc = torch.randn((B, 2, rows, 128), device="cuda", generator=gen).to(torch.bfloat16)
    vc = torch.randn((B, 2, rows, 128), device="cuda", generator=gen).to(torch.bfloat16)
    pos = torch.tensor([n_cap - 1, 64 * 17 + 5, 64 * 3, 100], dtype=torch.int32, device="cuda")
    qd = qd_all[0].clone()
    od = torch.empty_like(qd)
    lsed = torch.empty((B, 8), dtype=torch.float32, device="cuda")

    def run_all():
        K.ksa_prefill_fwd(lay, q, k, v, o=o, lse=lse, workspace=ws)
        K.ksa_prefill_bwd(lay, q, k, v, o, lse, g, dq=dq, dk=dk, dv=dv, workspace=wsb)
        K.ksa_decode_fwd_static(pd, qd, kc, vc, pos, od, lse=lsed, n_splits=3)

    def set_inputs(i):
        for dst, src in zip((q, k, v, g), data[i]):
            dst.copy_(src)
        qd.copy_(qd_all[i])

    # eager results for each data set (the first call also resolves the static scratch array's address)
    want = []
    for i in range(3):
        set_inputs(i)
        run_all()
        torch.cuda.synchronize()
        want.append([t.clone() for t in (o, lse, dq, dk, dv, od, lsed)])

    set_inputs(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all()
    for i in (1, 2, 0, 1):
        # eager work of the program between the replays: new inputs, outputs cleared, an unrelated eager call
        set_inputs(i)
        for t in (o, lse, dq, dk, dv, od, lsed):
            t.zero_()
        K.ksa_decode_fwd(pd, qd_all[(i + 1) % 3], kc, vc, pos)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("o", "lse", "dq", "dk", "dv", "decode o", "decode lse"),
                                  (o, lse, dq, dk, dv, od, lsed), want[i]):
            assert torch.equal(got, ref), f"replay on data set {i}: {name} differs from the eager call"
        say(f"replay on data set {i}: identical to the eager calls")
