"""moe_permute_static, the entry point that allocates nothing (for callers that cannot call hipMalloc:
graph capture, serving loops), against moe_permute through the C ABI and against the oracle.

Integer and byte work: everything must match bit for bit.  Two calls in a row on one stream, the
second with a smaller batch, so that what the first call left in the library's buffer is still there.
"""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _ids(T, E, K, seed):
    rng = np.random.default_rng(seed)
    pop = rng.random(E) ** 3 + 1e-3               # skewed: some experts large, some empty
    keys = rng.random((T, E)) ** (1.0 / pop)
    return np.argsort(-keys, axis=1)[:, :K].astype(np.int32)


def test_permute_without_allocation_equals_permute_on_two_calls_in_a_row(oracle64):
    import paper_2604_26881_amd as moe
    assert torch.cuda.is_available(), "this test needs the GPU"
    lib = moe.load()
    H = 128
    # (T, E, K, with the permuted copy): a large batch first, then smaller ones that reuse the buffer
    for T, E, K, copy in [(9000, 60, 4, True), (700, 60, 4, True), (3000, 200, 8, False), (40, 200, 8, False),
                          (4096, 60, 4, False), (1, 3, 2, True)]:
        print(f"[case] permute without allocation T={T} E={E} K={K} copy={copy}", flush=True)
        ids_np = _ids(T, E, K, T + E)
        ids = torch.from_numpy(ids_np).cuda()
        x = torch.randn((T, H), generator=torch.Generator().manual_seed(T)).to(torch.bfloat16).cuda()
        P = T * K
        mk = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
        off_a, src_a, rowp_a = mk(E + 1), mk(P), mk(P)
        off_b, src_b, rowp_b = mk(E + 1), mk(P), mk(P)
        Xa = torch.zeros((P, H), dtype=torch.bfloat16, device="cuda") if copy else None
        Xb = torch.zeros((P, H), dtype=torch.bfloat16, device="cuda") if copy else None
        ws = torch.empty(max(int(lib.moe_permute_workspace_bytes(T, K, E)), 256), dtype=torch.uint8, device="cuda")
        moe.moe_permute(ids, x, E, off_a, src_a, rowp_a, Xa, ws, materialize=copy)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        moe.moe_permute_static(ids, x, E, off_b, src_b, rowp_b, Xb)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(off_a, off_b) and torch.equal(src_a, src_b) and torch.equal(rowp_a, rowp_b)
        if copy:
            assert torch.equal(Xa.view(torch.int16), Xb.view(torch.int16))
        off_r, src_r, rowp_r = oracle64.permute(ids_np, E)
        assert np.array_equal(off_b.cpu().numpy(), off_r)
        assert np.array_equal(src_b.cpu().numpy(), src_r)
        assert np.array_equal(rowp_b.cpu().numpy(), rowp_r)


def test_permute_without_allocation_rejects_what_its_buffer_cannot_hold():
    import paper_2604_26881_amd as moe
    lib = moe.load()
    p = ctypes.c_void_p(0x1000)      # never dereferenced: the call is refused before anything is enqueued
    limit = 1 << 20
    T, K, E = 16385, 4, 256          # (T*K + 63) / 64 chunks * E * 4 bytes = 1 049 600 > 1 MiB
    assert ((T * K + 63) // 64) * E * 4 > limit
    assert lib.moe_permute_static(p, p, T, 64, E, K, p, p, p, None, None) == -3
    assert lib.moe_permute_static(p, p, 4, 60, 8, 2, p, p, p, None, None) == -2
    assert lib.moe_permute_static(p, p, 4, 64, 8, 2, None, p, p, None, None) == -1
    assert lib.moe_permute_static(None, None, 0, 64, 8, 2, None, None, None, None, None) == -1   # offsets are written even for T = 0
