"""The entry point that allocates nothing (akv_decode_attention_static: scratch in a static device array of the
library) against akv_decode_attention with a caller's workspace, through the C ABI: same decisions bit for bit, same
output bits, on two calls in a row, the second with a smaller input -- and with the token-split kernels, whose
control words live in that array."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_static_scratch_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import akv_testlib as T
    from paper_2409_16546_amd import workloads, binding as A

    def both(cfg, over, lens, path):
        w = workloads.make(cfg, **over)
        print(f"static scratch: cfg{cfg} {over} lens {lens} path {path}", flush=True)
        gc = T.gpu_cache(w.k, w.v, lens, w.Hq, w.Ncap)
        q = w.q.to(DEV)
        d_ws, d_st = A.DebugBuffers.allocate(gc), A.DebugBuffers.allocate(gc)
        s_ws, s_st = A.new_stats(DEV), A.new_stats(DEV)
        out_ws = A.akv_decode_attention(gc, q, dbg=d_ws, path=path, stats=s_ws)
        out_st = torch.empty_like(out_ws)
        plain_st = torch.empty_like(out_ws)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        A.akv_decode_attention_static(gc, q, out_st, dbg=d_st, path=path, stats=s_st)
        A.akv_decode_attention_static(gc, q, plain_st, path=path)       # and the variant without exports
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() <= before                    # nothing was allocated through torch either
        assert torch.equal(out_ws, out_st) and torch.equal(out_ws, plain_st)
        for name in ("lvlK", "logits", "a", "sel", "oest", "Ehat", "needV", "appliedV"):
            x, y = getattr(d_ws, name), getattr(d_st, name)
            assert torch.equal(x, y), f"{name} differs between the two entry points"
        assert torch.equal(s_ws, s_st)
        return w, lens, out_st, d_st

    from oracle import akv_oracle as O
    O.build()
    for path in (1, 2):
        # first call: several blocks per wave / several chunks; second call: a smaller shape, ragged, one empty sequence
        w, lens, out, dbg = both(2, dict(B=3, Hq=8, Hkv=4, N=3000), [3000, 2049, 700], path)
        w2, lens2, out2, dbg2 = both(4, dict(B=2, Hq=8, Hkv=2, N=600), [600, 0], path)
        # and the smaller call is right, not merely equal: against the oracle
        oc = T.oracle_cache(w2.k, w2.v, lens2, w2.Ncap)
        r = O.decode_attention(oc, T.bits(w2.q))
        T.assert_decode_equal(out2, dbg2, r, lens2, 4, f"static scratch, second call, path {path}")
    # a shape beyond the array is refused with a clear text and nothing runs
    big = A.Cache(4, 32, 8, 128, 131072)
    big._struct = A.akv_cache(A.akv_shape(4, 32, 8, 128, 131072), *[gcp for gcp in [0x1000] * 9])
    with pytest.raises(A.AkvError) as e:
        A.akv_decode_attention_static(big, torch.empty(4, 32, 128, dtype=torch.float16, device=DEV),
                                      torch.empty(4, 32, 128, dtype=torch.float32, device=DEV))
    assert e.value.status == A.AKV_EWORKSPACE and "static" in str(e.value)
