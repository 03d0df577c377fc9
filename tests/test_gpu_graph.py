"""The library allocates nothing, never synchronises and clears its buffers with kernels, so a call can be
captured into a HIP graph.  The graph is replayed several times with eager work and synchronisations in
between, and every replay must reproduce the eager result bit for bit (the path is deterministic)."""
import numpy as np
import pytest

from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,beta", [(I.FKL, 0.5), (I.JSD, 0.3)])
def test_captured_call_replays_bit_exactly(kind, beta):
    import torch
    from paper_2603_01875_amd import kdloss as K
    cfg = I.scaled(I.workload("fkl_bf16"), batch=2, seq=200, H_t=192, H_s=128, V=1544, kind=kind, beta=beta)
    data = I.generate(cfg)
    d = {k: G.to_device(data[k], cfg.dtype) for k in ("h_t", "W_t", "h_s", "W_s")}
    mask = torch.from_numpy(data["mask"]).cuda()
    p = K.make_params(cfg.T, cfg.H_t, cfg.H_s, cfg.V, kind, cfg.tau, beta, vocab_chunk=512)
    ws = K.alloc_workspace(p)
    outs = [dict(loss=torch.zeros(1, device="cuda"), ptl=torch.zeros(cfg.T, device="cuda"),
                 gh=torch.zeros(cfg.T, cfg.H_s, device="cuda", dtype=torch.bfloat16),
                 gW=torch.zeros(cfg.V, cfg.H_s, device="cuda", dtype=torch.bfloat16)) for _ in range(2)]

    def call(o):
        K.kd_loss_fwd_bwd_raw(p, d["h_t"], d["W_t"], d["h_s"], d["W_s"], mask, o["loss"], o["ptl"], o["gh"], o["gW"], ws)

    call(outs[0])                                   # eager reference (also warms up the kernels)
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in outs[0].items()}
    G.check(dict(loss=ref["loss"], per_token_loss=ref["ptl"], grad_h_s=ref["gh"], grad_W_s=ref["gW"]),
            G.run_oracle(cfg, data), "eager")

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(outs[1])
    for rep in range(3):
        for v in outs[1].values():
            v.fill_(7)                              # eager work between the replays; stale outputs would show
        ws.fill_(0x5a)                              # the workspace carries nothing from one call to the next
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(outs[1][k], ref[k]), f"replay {rep}: {k}"


def test_two_calls_on_two_streams_do_not_interfere():
    """The library keeps no state between calls: two problems enqueued on two streams (default
    priority), each with its own workspace, give the results they give one after the other."""
    import torch
    from paper_2603_01875_amd import kdloss as K
    cfgs = [I.scaled(I.workload("fkl_bf16"), batch=2, seq=300, H_t=256, H_s=128, V=8200),
            I.scaled(I.workload("jsd_bf16"), batch=1, seq=500, H_t=192, H_s=64, V=6152)]
    probs = []
    for cfg in cfgs:
        data = I.generate(cfg)
        d = {k: G.to_device(data[k], cfg.dtype) for k in ("h_t", "W_t", "h_s", "W_s")}
        d["mask"] = torch.from_numpy(data["mask"]).cuda()
        probs.append((cfg, d))
    seq = [K.kd_loss_fwd_bwd(d["h_t"], d["W_t"], d["h_s"], d["W_s"], d["mask"], tau=c.tau, kind=c.kind, beta=c.beta)
           for c, d in probs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    conc = [None, None]
    for rep in range(3):
        for i, (c, d) in enumerate(probs):
            with torch.cuda.stream(streams[i]):
                conc[i] = K.kd_loss_fwd_bwd(d["h_t"], d["W_t"], d["h_s"], d["W_s"], d["mask"], tau=c.tau, kind=c.kind,
                                            beta=c.beta)
        torch.cuda.synchronize()
        for a, b in zip(seq, conc):
            for k in ("loss", "per_token_loss", "grad_h_s", "grad_W_s"):
                assert torch.equal(a[k], b[k]), k
