"""The cache lookup that allocates nothing (taser_cache_lookup_static), through the
C ABI, against taser_cache_lookup on the same requests: two calls in a row, the second
with fewer requests, so that whatever the first left in the shared scratch array
would show. Bit-exact, like every other comparison on this path (bytes and counts)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2402_05396_amd as T

pytestmark = pytest.mark.gpu


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def test_static_lookup_equals_the_allocating_lookup_on_two_calls_in_a_row():
    lib = T.lib()
    rng = np.random.default_rng(2024)
    rows, dim = 6000, 413                                     # 1652-byte rows, as the largest workload's node table
    host = torch.from_numpy(rng.standard_normal((rows, dim)).astype(np.float32)).pin_memory()
    cap = 1200
    residents = torch.from_numpy(rng.permutation(rows)[:cap].astype(np.int32))
    c_static = T.cache_init(host, cap, residents, staging_rows=3000)
    c_plain = T.cache_init(host, cap, residents, staging_rows=3000)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for n in (400_000, 33_333):                               # the second call is the smaller one
        ids_np = np.minimum(rng.zipf(1.15, n) - 1, rows - 1).astype(np.int32)
        ids_np[::53] = -1                                     # zero rows
        ids_np[7::1001] = rows + 5                            # out of range: served like a negative id
        ids = torch.from_numpy(ids_np).cuda()
        out_static = torch.full((n, dim), float("nan"), dtype=torch.float32, device="cuda")
        out_plain = torch.full((n, dim), float("nan"), dtype=torch.float32, device="cuda")
        hm_static = torch.zeros(2, dtype=torch.int64, device="cuda")
        hm_plain = torch.zeros(2, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        print(f"static lookup: n = {n}", flush=True)
        rc = lib.taser_cache_lookup_static(c_static.handle, _ptr(ids), n, _ptr(out_static), _ptr(hm_static), stream)
        assert rc == 0, T.last_error()
        rc = lib.taser_cache_lookup(c_plain.handle, _ptr(ids), n, _ptr(out_plain), _ptr(hm_plain), stream)
        assert rc == 0, T.last_error()
        torch.cuda.synchronize()
        assert out_static.cpu().numpy().tobytes() == out_plain.cpu().numpy().tobytes()
        assert hm_static.tolist() == hm_plain.tolist() and sum(hm_static.tolist()) > 0
    # beyond the fixed scratch: refused before anything is launched
    too_many = T.lib().taser_cache_lookup_static(c_static.handle, _ptr(ids), (1 << 21) + 1, _ptr(out_static), None, stream)
    assert too_many == -2 and "exceeds" in T.last_error()
    T.cache_free(c_static)
    T.cache_free(c_plain)
