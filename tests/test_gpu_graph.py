"""The hot path under HIP graph capture: no call of the path allocates, synchronises or copies, so quantize ->
select -> sparse attention can be captured once and replayed.  Every replay (with eager work and synchronisations
in between) must reproduce the eager results bit for bit."""
import pytest
import torch

from paper_2505_24179_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


@pytest.mark.parametrize("name", ["gqa4-2k", "gqa2-36k-long-rows"])
def test_captured_step_replays_bit_exact(sale, name):
    if name == "gqa4-2k":
        w = inputs.scaled(inputs.LLAMA_32K, 2048 + 64, 4, 1, name)
    else:      # long rows: the window launches, parking slots and balance tables are part of the captured work
        w = inputs.Workload(name, 36864, 4, 2, seed=0x5A1E0010, tau=0.0005)
    q, k, v = inputs.make_inputs(w)
    dev = torch.device("cuda:0")
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    tau = torch.tensor([w.tau], dtype=torch.float32, device=dev)

    def buffers():
        return dict(
            q4=torch.empty(1, w.n_q_heads, w.seq_len, 64, dtype=torch.uint8, device=dev),
            k4=torch.empty(1, w.n_kv_heads, w.seq_len, 64, dtype=torch.uint8, device=dev),
            qs=torch.empty(1, w.n_q_heads, p.n_q, dtype=torch.float32, device=dev),
            ks=torch.empty(1, w.n_kv_heads, p.n_k, dtype=torch.float32, device=dev),
            mask=torch.zeros(1, w.n_q_heads, p.n_q, p.words, dtype=torch.int64, device=dev),
            counts=torch.zeros(1, w.n_q_heads, p.n_q, dtype=torch.int32, device=dev),
            o=torch.full_like(qd, float("nan")),
            ws_sel=torch.empty(sale.workspace_bytes(p, sale.WS_SELECT), dtype=torch.uint8, device=dev),
            ws_att=torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev))

    def step(b):
        sale.quantize_qk(p, qd, kd, out=(b["q4"], b["k4"], b["qs"], b["ks"]))
        sale.select(p, qd, kd, b["q4"], b["k4"], b["qs"], b["ks"], tau, out=(b["mask"], b["counts"]), ws=b["ws_sel"])
        sale.sparse_attn(p, qd, kd, vd, b["mask"], b["counts"], out=b["o"], ws=b["ws_att"])

    eager = buffers()
    step(eager)
    torch.cuda.synchronize()
    assert not torch.isnan(eager["o"]).any()

    cap = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # warm-up on the capture stream (first-call initialisations happen outside capture)
        step(cap)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(cap)
    for replay in range(3):
        for name_ in ("mask", "counts"):
            cap[name_].zero_()
        cap["o"].fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=dev).sum()      # the program's own eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name_ in ("q4", "k4", "qs", "ks", "mask", "counts", "o"):
            assert torch.equal(cap[name_], eager[name_]), (replay, name_)
        assert float(scratch) == float(scratch)
