"""The library allocates nothing and records no memset: its launch sequences can be captured in a
HIP graph.  Every replay is checked against the eager result, with eager work in between."""
import pytest
import torch

from helpers import upload
from paper_2105_13120_amd import inputs, rsa

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode,kw", [
    (rsa.MODE_FUSED, dict(B=2, Z=2, L=512, N=4, causal=True)),
    (rsa.MODE_FUSED, dict(B=1, Z=2, L=4096, N=4, causal=False, rank_begin=3, rank_end=4)),   # split key walk
    (rsa.MODE_FUSED, dict(B=1, Z=2, L=1024, N=4, causal=True, zigzag=True, A=128)),
    (rsa.MODE_STAGED, dict(B=1, Z=2, L=256, N=2, causal=False)),
    # the backward whose workspace is the library's static device array (its address is looked up by
    # the warm-up call, outside the capture)
    (rsa.MODE_FUSED, dict(B=1, Z=2, L=4096, N=4, causal=True, rank_begin=3, rank_end=4, static_ws=True)),
])
def test_forward_backward_under_graph_capture(mode, kw):
    kw = dict(kw)
    static_ws = kw.pop("static_ws", False)
    A = kw.pop("A", 64)
    cfg = inputs.RSAConfig("g", A=A, dtype="bf16", seed=61, **kw)
    x = inputs.make_inputs(cfg)
    Q, K, V, dO = (upload(x[k], "bf16") for k in ("Q", "K", "V", "dO"))
    rb, re = cfg.ranks
    desc = rsa.make_desc(K, cfg.N, causal=cfg.causal, rank_begin=rb, rank_end=re, mode=mode, zigzag=cfg.zigzag)
    wf = torch.empty(max(rsa.workspace_bytes(desc, False), 16), dtype=torch.uint8, device="cuda")
    wb = torch.empty(max(rsa.workspace_bytes(desc, True), 16), dtype=torch.uint8, device="cuda")

    def buffers():
        return dict(O=torch.empty_like(Q), LSE=torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda"),
                    dQ=torch.empty_like(Q), dK=torch.empty_like(K), dV=torch.empty_like(V))

    def run(b):
        rsa.forward(desc, Q, K, V, O=b["O"], LSE=b["LSE"], ws=wf)
        if static_ws:
            rsa.backward_static(desc, dO, Q, K, V, b["O"], b["LSE"], b["dQ"], b["dK"], b["dV"])
        else:
            rsa.backward(desc, dO, Q, K, V, b["O"], b["LSE"], dQ=b["dQ"], dK=b["dK"], dV=b["dV"], ws=wb)

    eager = buffers()
    run(eager)
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in eager.items()}

    g = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(g)                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(g)
    for replay in range(3):
        for v in g.values():
            v.fill_(float("nan")) if v.dtype != torch.float32 else v.fill_(-1.0)
        wf.fill_(0xFF); wb.fill_(0xFF)          # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(g[k], ref[k]), f"replay {replay}: {k} differs from the eager result"


def test_linformer_chain_under_graph_capture():
    """The Linformer entry points (projection, short-keys forward, one-kernel backward, projection
    backward) allocate nothing either: one pass captured and replayed three times."""
    B, Z, L, N, Kp, A = 1, 4, 2048, 4, 256, 64
    g = torch.Generator(device="cuda").manual_seed(7)
    rnd = lambda *shape, s=1.0: (torch.randn(shape, generator=g, device="cuda") * s).to(torch.bfloat16)
    Q, K, V, dO = (rnd(B, Z, L, A) for _ in range(4))
    E, F = rnd(L, Kp, s=L ** -0.5), rnd(L, Kp, s=L ** -0.5)
    desc = rsa.make_desc(K, N)
    ws = torch.empty(max(rsa.linformer_workspace_bytes(desc, Kp), 16), dtype=torch.uint8, device="cuda")

    def buffers():
        kp = lambda: torch.empty((B, Z, Kp, A), dtype=torch.bfloat16, device="cuda")
        return dict(Kp=kp(), Vp=kp(), O=torch.empty_like(Q), LSE=torch.empty((B, Z, L), dtype=torch.float32, device="cuda"),
                    dQ=torch.empty_like(Q), dKp=kp(), dVp=kp(), dK=torch.empty_like(K), dV=torch.empty_like(V),
                    dE=torch.empty((L, Kp), dtype=torch.float32, device="cuda"),
                    dF=torch.empty((L, Kp), dtype=torch.float32, device="cuda"))

    def run(b):
        rsa.linformer_project(desc, K, E, b["Kp"], ws)
        rsa.linformer_project(desc, V, F, b["Vp"], ws)
        rsa.linformer_forward(desc, Q, b["Kp"], b["Vp"], b["O"], b["LSE"])
        rsa.linformer_backward(desc, dO, Q, b["Kp"], b["Vp"], b["O"], b["LSE"], b["dQ"], b["dKp"], b["dVp"], ws)
        rsa.linformer_project_bwd(desc, b["dKp"], K, E, b["dK"], b["dE"])
        rsa.linformer_project_bwd(desc, b["dVp"], V, F, b["dV"], b["dF"])

    eager = buffers()
    run(eager)
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in eager.items()}
    gb = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(gb)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(gb)
    for replay in range(3):
        for v in gb.values():
            v.fill_(float("nan")) if v.dtype != torch.float32 else v.fill_(-1.0)
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(gb[k], ref[k]), f"replay {replay}: {k} differs from the eager result"
