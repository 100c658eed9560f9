"""Decode steps recorded into a HIP graph and replayed: the serving-loop use the allocation-free entry point is for.
The graph holds library launches only (the library clears with fill kernels, never with memset nodes); every replay is
checked against the eager result, with eager work and synchronisations between the replays."""
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.parametrize("path", [1, 2], ids=["head-path", "split-path"])
def test_decode_in_a_hip_graph_replays_bit_identically(path):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import akv_testlib as T
    from paper_2409_16546_amd import workloads, binding as A
    print(f"graph: static-scratch decode captured and replayed, path {path}", flush=True)
    w = workloads.make(2, B=3, Hq=8, Hkv=4, N=2500)
    lens = [2500, 1301, 0]
    gc = T.gpu_cache(w.k, w.v, lens, w.Hq, w.Ncap)
    q = w.q.to(DEV)
    q2 = (w.q * 0.5).to(DEV)
    eager = torch.empty(3, 8, 128, dtype=torch.float32, device=DEV)
    A.akv_decode_attention_static(gc, q, eager, path=path)            # first call on the device: looks up the scratch array
    eager2 = A.akv_decode_attention(gc, q2, path=path).clone()
    torch.cuda.synchronize()
    q_in = q.clone()
    out = torch.zeros_like(eager)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        A.akv_decode_attention_static(gc, q_in, out, path=path)       # warm-up on the side stream
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            A.akv_decode_attention_static(gc, q_in, out, path=path)
    torch.cuda.current_stream().wait_stream(s)
    for rep in range(4):
        src = q if rep % 2 == 0 else q2
        q_in.copy_(src)
        out.fill_(float("nan"))
        A.akv_decode_attention(gc, q2 if rep % 2 == 0 else q, path=3 - path)   # the program's own eager work in between, other kernels
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager if rep % 2 == 0 else eager2), f"replay {rep} differs from the eager result"
    assert not gc.flags.cpu()[:A.AKV_NFLAGS].any()
