"""tgnn_memory_writeback_noalloc (the entry point that allocates nothing; its scratch is a static device array)
against tgnn_memory_writeback: winners and every written row bit for bit, on two calls in a row, the second with a
smaller input; plus the size limit."""
import numpy as np
import pytest
import torch

from gpu_common import custom_problem, batch_np

pytestmark = pytest.mark.gpu


def dev(a, dt=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.to("cuda", dtype=dt) if dt else t.to("cuda")


def test_noalloc_writeback_matches_the_context_entry_point():
    from paper_2307_07649_amd import tgnn
    P = custom_problem(n_nodes=300, E=2000, d_mem=100, d_time=8, d_edge=4, d_static=0, n_heads=2, k=5, batch=1200)
    d = P["d"]
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch)
    st_ref = tgnn.State(d.n_nodes, d.d_mem, 1)
    st_new = tgnn.State(d.n_nodes, d.d_mem, 1)
    rng = np.random.default_rng(3)
    for lo, hi in ((0, 1200), (1200, 1500), (1500, 1501)):          # the later calls are smaller than the first
        b = batch_np(P, lo, hi); n = hi - lo
        s_src = dev(rng.standard_normal((n, d.d_mem)).astype(np.float32))
        s_dst = dev(rng.standard_normal((n, d.d_mem)).astype(np.float32))
        tau_s = dev(rng.uniform(0, 50, n)); tau_d = dev(rng.uniform(0, 50, n))
        args = (dev(b["src"]), dev(b["dst"]), dev(b["eid"]), dev(b["t"]), s_src, s_dst, tau_s, tau_d)
        win_ref = ctx.tgnn_memory_writeback(st_ref, 0, *args)
        win_new = torch.full((2 * n,), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        tgnn.tgnn_memory_writeback_noalloc(st_new, *args, win_new)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(win_new, win_ref) and int(win_ref.sum().item()) == len(np.unique(np.concatenate([b["src"], b["dst"]])))
        for name in ("mem", "mail", "mem_ts", "mail_ts", "mail_eid"):
            assert torch.equal(getattr(st_new, name), getattr(st_ref, name)), (lo, name)
    assert (st_new.mail_eid >= 0).sum().item() > 100


def test_noalloc_writeback_rejects_sizes_beyond_its_scratch():
    import ctypes as C
    from paper_2307_07649_amd import tgnn
    st = tgnn.State(8, 4, 1)
    z = torch.zeros(16, dtype=torch.int32, device="cuda"); f = torch.zeros(64, device="cuda"); t = torch.zeros(16, dtype=torch.float64, device="cuda")
    lib = tgnn._lib
    rc = lib.tgnn_memory_writeback_noalloc(262145, 4, C.byref(st.c), z.data_ptr(), z.data_ptr(), z.data_ptr(), t.data_ptr(), 4,
                                           f.data_ptr(), f.data_ptr(), t.data_ptr(), t.data_ptr(), None, None)
    assert rc == -4 and b"scratch" in lib.tgnn_last_error()
    rc = lib.tgnn_memory_writeback_noalloc(8, 4, C.byref(st.c), z.data_ptr(), z.data_ptr(), z.data_ptr(), t.data_ptr(), 1 << 21,
                                           f.data_ptr(), f.data_ptr(), t.data_ptr(), t.data_ptr(), None, None)
    assert rc == -4
    rc = lib.tgnn_memory_writeback_noalloc(8, 4, C.byref(st.c), None, z.data_ptr(), z.data_ptr(), t.data_ptr(), 4,
                                           f.data_ptr(), f.data_ptr(), t.data_ptr(), t.data_ptr(), None, None)
    assert rc == -2
