"""enec_compress_static (the entry point that allocates nothing) against enec_compress, through the C ABI.

Two calls in a row share the library's per-GPU scratch array, the second with a smaller input; both must
write exactly the stream enec_compress writes for the same input (and that stream is the oracle's).
"""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_compress_equals_enec_compress_twice_in_a_row(oracle):
    import torch
    from paper_2604_03298_amd import enec
    assert torch.cuda.is_available(), "needs the MI355X"
    enec.lib()
    size = torch.zeros(1, dtype=torch.int64).pin_memory()
    cases = [(W.gaussian(37 * 16384 + 5001, 0.02, 71), 0), (W.gaussian(5 * 16384 + 123, 0.01, 72), 0),
             (W.gaussian(9 * 4096 + 17, 0.02, 73), 4096)]
    for i, (w, B) in enumerate(cases):
        prm = oracle.tune(w)
        src = torch.from_numpy(w.view(np.int16)).cuda()
        cap = enec.compress_bound(w.size, block_size=B)
        # the entry point under test first: its scratch array is in whatever state the last call left
        got = torch.full((cap,), 0xA5, dtype=torch.uint8, device="cuda")
        size.fill_(-1)
        rc = enec.compress_static(src, prm, got, block_size=B, out_bytes=size)
        assert rc == enec.OK, enec.strerror(rc)
        torch.cuda.synchronize()
        n_static = int(size.item())
        ws = enec.new_workspace(w.size, B)
        want = torch.full((cap,), 0xA5, dtype=torch.uint8, device="cuda")
        size.fill_(-1)
        rc = enec.compress(src, prm, want, ws, block_size=B, out_bytes=size)
        assert rc == enec.OK, enec.strerror(rc)
        torch.cuda.synchronize()
        n_ws = int(size.item())
        assert n_static == n_ws > 0, (i, n_static, n_ws)
        assert torch.equal(got[:n_ws], want[:n_ws]), f"call {i}: stream differs from enec_compress's"
        rc_o, ref = oracle.compress(w, prm, B if B else oracle.default_block(w.size))
        assert rc_o == 0 and np.array_equal(got[:n_ws].cpu().numpy(), ref), f"call {i}: stream differs from the oracle's"
        back = torch.zeros_like(src)
        assert enec.decompress(got, back) == enec.OK
        torch.cuda.synchronize()
        assert torch.equal(back, src)


def test_static_scratch_rejects_what_it_cannot_hold():
    import torch
    from paper_2604_03298_amd import enec
    src = torch.zeros(16384, dtype=torch.int16, device="cuda")
    out = torch.zeros(enec.compress_bound(16384), dtype=torch.uint8, device="cuda")
    assert enec.compress_static(src, None, out) == enec.E_ARG                 # no tuple: tuning waits for the stream
    # more scan state than the array holds: rejected on the host, nothing enqueued (the pointers are never used)
    n_big = 1 << 31
    assert enec.workspace_bytes(n_big, 2048) > enec.STATIC_SCRATCH_BYTES
    assert enec.compress_static(src, (122, 6, 3, 16), out, block_size=2048, n_elems=n_big) == enec.E_CAPACITY
