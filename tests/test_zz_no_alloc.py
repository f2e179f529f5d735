"""The entry point that allocates nothing (sd_accept_static) against the one it is a variant of (sd_accept):
identical outputs on two calls in a row, the second with a smaller input, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2505_08600_amd import api
from test_gpu_accept import check_against_oracle, synthetic_case

pytestmark = pytest.mark.gpu


def _both(L, logits, q, cand, u, gamma, T):
    B, rows, V = logits.shape
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d_l, d_q, d_c, d_u = dev(logits), dev(q), dev(cand), dev(u)
    ws = torch.zeros(3 * B * rows, device="cuda")
    out = [torch.full((B,), -7, dtype=torch.int32, device="cuda") for _ in range(4)]
    p = lambda t: C.c_void_p(t.data_ptr())
    s = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.sd_accept_static(p(d_l), B, gamma, V, T, p(d_c), p(d_q), p(d_u), p(out[2]), p(out[3]), s)
    assert rc == api.SD_OK, L.sd_last_error()
    rc = L.sd_accept(p(d_l), B, gamma, V, T, p(d_c), p(d_q), p(d_u), p(out[0]), p(out[1]), p(ws), s)
    assert rc == api.SD_OK, L.sd_last_error()
    torch.cuda.synchronize()
    na, nx, na_s, nx_s = (t.cpu().numpy() for t in out)
    return na, nx, na_s, nx_s


def test_static_scratch_variant_equals_workspace_variant_on_two_calls():
    L = api.lib()
    V, T = 32000, 1.0
    # first call: 12 sequences x 9 rows; second call, smaller: 5 sequences x 4 rows (stale statistics of the
    # first call sit behind the part of the array the second call uses)
    for seed, B, gamma in ((93, 12, 8), (94, 5, 3)):
        print(f"sd_accept_static B={B} gamma={gamma}", flush=True)
        logits, q, cand, u = synthetic_case(seed, B, gamma, V, 0.9, T)
        na, nx, na_s, nx_s = _both(L, logits, q, cand, u, gamma, T)
        assert np.array_equal(na, na_s) and np.array_equal(nx, nx_s), (na, na_s, nx, nx_s)
        assert check_against_oracle(logits, q, cand, u, T, na_s, nx_s) <= 1
        assert B < 12 or len(set(na_s.tolist())) >= 2


def test_static_scratch_variant_rejects_sizes_beyond_its_array():
    L = api.lib()
    x = torch.zeros(8, device="cuda")
    i = torch.zeros(8, dtype=torch.int32, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    assert L.sd_accept_static(p(x), 4097, 0, 8, 0.0, None, None, None, p(i), p(i), None) == api.SD_ECAP
    assert b"4096" in L.sd_last_error()
    assert L.sd_accept_static(p(x), 257, 15, 8, 0.0, p(i), None, None, p(i), p(i), None) == api.SD_ECAP
    assert L.sd_accept_static(None, 1, 0, 8, 0.0, None, None, None, p(i), p(i), None) == api.SD_EINVAL
