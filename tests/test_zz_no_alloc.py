"""The allocation-free small-M entry point (built-in scratch buffer) against the workspace
form it shares its kernels with."""
import numpy as np
import pytest

from paper_2605_11582_amd import binding as B, synth
import gpu_common as G

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_equals_the_workspace_form():
    # two calls in a row through the C ABI, the second with a smaller input: the buffer keeps
    # the first call's contents and the second result must not depend on them
    torch = G.torch_mod()
    outs = []
    for rows, cols, M in ((4096, 11008, 64), (2000, 8192, 33), (4096, 11008, 24)):
        print(f"case static scratch {rows}x{cols} M={M}", flush=True)
        w = synth.weights(rows, cols, 6100 + rows)
        p = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 128, 0).to("cuda")
        X = G.to_dev(synth.activation_rows(M, cols, 6100 + M).view(np.uint16)).view(torch.float16)
        need = B.smallm_ws_bytes(p, M)
        assert 0 < need <= (16 << 20)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        Y_ws = torch.zeros((M, rows), dtype=torch.float16, device="cuda")
        Ybuf = torch.full((M + 2, rows), G.CANARY, dtype=torch.int16, device="cuda")
        Y_st = Ybuf[1:M + 1].view(torch.float16)
        B.sparse_gemm_smallm_ws(p, X, Y_ws, ws)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        B.sparse_gemm_smallm_static(p, X, Y_st)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        host = Ybuf.cpu().numpy().view(np.uint16)
        assert np.all(host[0] == G.CANARY) and np.all(host[M + 1] == G.CANARY)
        assert np.array_equal(host[1:M + 1], Y_ws.cpu().numpy().view(np.uint16)), (rows, cols, M)
        outs.append(host[1:M + 1].copy())
    assert all(np.isfinite(o.view(np.float16)).all() for o in outs)
    # a request beyond the built-in buffer is refused on the host, before anything is launched
    big = B.Packed(4096, 32768, 2, 128, 0, None, None, None, None)
    assert B.smallm_ws_bytes(big, 64) > 16 << 20
    v = B.View(4096, 32768, 2, 128, 0, 16, 16, 16, 16)    # fake aligned pointers: never used
    assert B.lib().egt_sparse_gemm_smallm_static(__import__("ctypes").byref(v), 16, 32768, 16, 4096, 64, None) == 6
