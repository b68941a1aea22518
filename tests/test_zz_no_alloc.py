"""The sampler entry point that allocates nothing (pl_sample_static: slice partials in the library's own
device array) against pl_sample with a caller-provided workspace, through the C ABI: same kernels, so
tokens and log-probs must be identical bit for bit; two calls in a row, the second smaller, so stale
partials of the first call would show."""
import numpy as np
import pytest
import torch

import paper_2509_19128_amd as pl

pytestmark = pytest.mark.gpu


def _inputs(n, V, seed):
    rng = np.random.default_rng(seed)
    logits = torch.from_numpy((rng.standard_normal((n, V)) * 2.0).astype(np.float32)).cuda()
    sid = torch.from_numpy(rng.integers(0, 1 << 62, n, dtype=np.int64)).cuda()
    pos = torch.from_numpy(rng.integers(0, 16384, n).astype(np.int32)).cuda()
    inv_t = torch.from_numpy((1.0 / rng.uniform(0.5, 1.5, n)).astype(np.float32)).cuda()
    forced = np.full(n, -1, np.int32)
    forced[::3] = rng.integers(0, V, len(forced[::3]))
    return logits, sid, pos, inv_t, torch.from_numpy(forced).cuda()


def _both(n, V, seed):
    logits, sid, pos, inv_t, forced = _inputs(n, V, seed)
    res = []
    for static in (False, True):
        tok = torch.full((n,), -7, device="cuda", dtype=torch.int32)
        lp = torch.full((n,), 7.0, device="cuda", dtype=torch.float32)
        args = (logits.data_ptr(), n, V, sid.data_ptr(), pos.data_ptr(), inv_t.data_ptr(), forced.data_ptr(), 4242,
                tok.data_ptr(), lp.data_ptr())
        if static:
            pl.pl_sample_static(*args, 0)
        else:
            ws = torch.empty(pl.pl_sample_workspace_bytes(n, V), device="cuda", dtype=torch.uint8)
            pl.pl_sample(*args, ws.data_ptr(), 0)
        torch.cuda.synchronize()
        res.append((tok.cpu().numpy(), lp.cpu().numpy()))
    return res


def test_static_scratch_sampler_equals_the_workspace_sampler_on_two_calls_in_a_row():
    for n, V, seed in [(37, 152064, 1), (5, 4096, 2)]:      # the second call is smaller than the first
        (t0, l0), (t1, l1) = _both(n, V, seed)
        assert (t0 >= 0).all() and (t0 < V).all() and np.isfinite(l0).all() and (l0 <= 0).all()
        assert np.array_equal(t0, t1)
        assert np.array_equal(l0.view(np.uint32), l1.view(np.uint32))


def test_static_scratch_sampler_rejects_sizes_beyond_its_array():
    z = torch.zeros(8, device="cuda")
    for n, V in [(513, 4096), (4, 262144 + 4), (0, 4096)]:
        with pytest.raises(pl.PlError) as ex:
            pl.pl_sample_static(z.data_ptr(), n, V, z.data_ptr(), z.data_ptr(), z.data_ptr(), 0, 1, z.data_ptr(), z.data_ptr(), 0)
        assert ex.value.code == pl.PL_E_INVAL
