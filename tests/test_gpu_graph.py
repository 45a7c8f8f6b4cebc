"""The decode step recorded into a HIP graph and replayed: every replay, with new queries copied into the graph's input
buffer and unrelated eager work and synchronisations between the replays, must give what the same calls give when they
are launched directly.  The single-launch form keeps state in device memory between launches (epochs, tagged words), the
two-launch forms keep arrival counters: a replay must leave them as a direct launch does.  Both entry points: the
context's step and the allocation-free step (whose first call on a device, a symbol lookup, is made outside the capture)."""
import pytest
import torch

import paper_2504_00970_amd as skv
from workload import gen

pytestmark = pytest.mark.gpu

LAYERS = 3
N_QUERY_SETS = 3


@pytest.fixture(scope="module")
def U():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


@pytest.mark.parametrize("noalloc", [False, True], ids=["context", "noalloc"])
@pytest.mark.parametrize("B,budget,exact", [(1, 1024, True), (3, 700, True), (9, 1500, False)],
                         ids=["single-launch", "single-launch-256", "two-launch-stream"])
def test_decode_step_graph_replays_equal_direct_launches(U, B, budget, exact, noalloc):
    # (16 query heads for the batch of nine: the allocation-free step's split-K partials must fit its static scratch)
    wl = gen.CFG1.scaled(n_layers=LAYERS, batch=B, t_range=(2500, 6000), budgets=(budget,), n_q_heads=32 if B < 9 else 16)
    inp = gen.ragged_inputs(wl, seed=31 + B, device=U.DEV, resident_layers=LAYERS)
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T, S = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    desc = skv.Desc(n_layers=LAYERS, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype), max_tokens=T,
                    max_sentences=S, max_budget=budget, max_batch=B)
    ctx = skv.Context(desc)
    sv = torch.zeros(LAYERS, H, S, D, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S, sv)
    qsets = [torch.randn(LAYERS, B, Hq, D, device=U.DEV).to(inp.q.dtype) for _ in range(N_QUERY_SETS)]
    q = torch.empty_like(qsets[0])                                # the graph's input
    out = torch.zeros(LAYERS, B, Hq, D, device=U.DEV)
    lse = torch.zeros(LAYERS, B, Hq, device=U.DEV)
    n_tok = U.empty_i32(LAYERS, B, H, fill=-1)

    def layers(stream=None):
        for l in range(LAYERS):
            if noalloc:
                skv.decode_step_noalloc(desc, l, B, q[l], q[l], inp.K, inp.V, T, sv, S, *d, out[l], lse[l], None, n_tok[l],
                                        stream=stream)
            else:
                ctx.decode_step(l, B, q[l], q[l], inp.K, inp.V, T, sv, S, *d, out[l], lse[l], None, n_tok[l])

    refs = []
    for qs in qsets:                                              # direct launches (also the allocation-free step's first call)
        q.copy_(qs)
        layers()
        torch.cuda.synchronize()
        refs.append((out.clone(), lse.clone(), n_tok.clone()))

    print("capturing", LAYERS, "layers, B", B, "noalloc" if noalloc else "context", flush=True)
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        s = torch.cuda.current_stream().cuda_stream
        ctx.set_stream(s)
        layers(stream=s)
    ctx.set_stream(torch.cuda.current_stream().cuda_stream)

    scratch = torch.randn(512, 512, device=U.DEV)
    for rep in range(2 * N_QUERY_SETS):
        i = rep % N_QUERY_SETS
        q.copy_(qsets[i])
        out.fill_(7.0)
        g.replay()
        scratch = (scratch @ scratch).clamp_(-1, 1)               # the program's own eager work between replays
        torch.cuda.synchronize()
        r_out, r_lse, r_n = refs[i]
        assert torch.equal(n_tok, r_n), (rep, "n_tok")
        if exact:
            assert torch.equal(out, r_out) and torch.equal(lse, r_lse), (rep, "out / lse")
        else:                                                     # streaming kernel: tiles in arrival order
            assert float((out - r_out).abs().max()) <= 2e-2 / 4, rep
            fin = torch.isfinite(r_lse)
            assert torch.equal(fin, torch.isfinite(lse)) and float((lse[fin] - r_lse[fin]).abs().max()) <= 2e-2 / 4, rep
