"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes its workspaces as documented and rejects bad arguments before any launch."""
import ctypes

import numpy as np
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2604_26881_amd as moe
    return moe.load()


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", n)).read() for n in ("moe.h", "moe_tuning.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"moe_route", "moe_permute", "moe_expert_group_forward", "moe_combine"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n
    from paper_2604_26881_amd import binding
    assert sorted(binding.SYMBOLS) == names


def test_library_carries_the_id_of_the_sources_beside_it(lib):
    from paper_2604_26881_amd import binding, build
    assert binding.build_id() == build.source_id() and len(build.source_id()) == 64


def test_status_strings(lib):
    for code in (0, -1, -2, -3, -4, -99):
        s = lib.moe_status_string(code)
        assert isinstance(s, bytes) and len(s) > 0


def test_workspace_sizes(lib):
    P, I, T, Is = 16384, 1408, 4096, 5632
    assert lib.moe_expert_workspace_bytes(P, I) == P * I * 2
    assert lib.moe_shared_workspace_bytes(T, 2048, Is) == T * Is * 2
    # small batches: room for the fp32 partial sums of a down projection cut into 8 parts along K
    assert lib.moe_shared_workspace_bytes(128, 2048, Is) == 128 * Is * 2 + 8 * 128 * 2048 * 4
    assert lib.moe_expert_workspace_bytes(3, 64) % 256 == 0 and lib.moe_expert_workspace_bytes(3, 64) >= 3 * 64 * 2
    assert lib.moe_workspace_bytes(T, 2048, 60, 4, I, Is) == max(P * I * 2, T * Is * 2)
    assert lib.moe_permute_workspace_bytes(T, 4, 60) == (P // 64) * 60 * 4
    assert lib.moe_expert_workspace_bytes(0, 64) == 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    p = ctypes.c_void_p(0x1000)   # never dereferenced on the host; no launch happens on these paths
    SHAPE, NULL, WS = -2, -1, -3
    # route
    assert lib.moe_route(p, p, None, 4, 63, 8, 2, 0, p, p, None) == SHAPE     # H not a multiple of 64
    assert lib.moe_route(p, p, None, 4, 64, 8, 9, 0, p, p, None) == SHAPE     # K > E
    assert lib.moe_route(p, p, None, 4, 64, 300, 2, 0, p, p, None) == SHAPE   # E > 256
    assert lib.moe_route(p, p, None, -1, 64, 8, 2, 0, p, p, None) == SHAPE
    assert lib.moe_route(None, p, None, 4, 64, 8, 2, 0, p, p, None) == NULL
    assert lib.moe_route(None, None, None, 0, 64, 8, 2, 0, None, None, None) == 0   # T = 0: no-op
    # route, one bias row per segment
    assert lib.moe_route_segments(p, p, p, p, 0, 4, 64, 8, 2, 0, p, p, None) == SHAPE       # no segment
    assert lib.moe_route_segments(p, p, p, p, 5000, 4, 64, 8, 2, 0, p, p, None) == SHAPE
    assert lib.moe_route_segments(p, p, p, p, 2, 4, 64, 8, 9, 0, p, p, None) == SHAPE       # K > E
    assert lib.moe_route_segments(p, p, None, p, 2, 4, 64, 8, 2, 0, p, p, None) == NULL     # bias rows are required
    assert lib.moe_route_segments(p, p, p, None, 2, 4, 64, 8, 2, 0, p, p, None) == NULL
    assert lib.moe_route_segments(None, None, None, None, 1, 0, 64, 8, 2, 0, None, None, None) == 0
    # permute
    assert lib.moe_permute(p, p, 4, 64, 8, 2, None, p, p, p, p, 1 << 20, None) == NULL
    assert lib.moe_permute(p, p, 4, 64, 8, 2, p, p, p, p, p, 8, None) == WS
    assert lib.moe_permute(p, p, 4, 64, 8, 2, p, p, p, p, None, 0, None) == NULL
    assert lib.moe_permute(p, p, 4, 60, 8, 2, p, p, p, p, None, 0, None) == SHAPE
    # expert block: range checks
    args = (p, p, p, p, p, 32, 64, 8, 128, p, p, 32 * 128 * 2, None)
    assert lib.moe_expert_group_forward(3, 3, *args) == SHAPE      # empty range
    assert lib.moe_expert_group_forward(-1, 3, *args) == SHAPE
    assert lib.moe_expert_group_forward(0, 9, *args) == SHAPE      # hi > E
    assert lib.moe_expert_group_forward(0, 8, p, p, p, p, p, 32, 64, 8, 100, p, p, 1 << 20, None) == SHAPE
    assert lib.moe_expert_group_forward(0, 8, p, None, p, p, p, 32, 64, 8, 128, p, p, 1 << 20, None) == NULL
    assert lib.moe_expert_group_forward(0, 8, p, p, p, p, p, 32, 64, 8, 128, p, p, 100, None) == WS
    assert lib.moe_expert_group_forward(0, 8, None, None, None, None, None, 0, 64, 8, 128, None, None, 0, None) == 0
    # expert block reading x through src_of_row
    ga = lambda src, K, P: lib.moe_expert_group_forward_gather(0, 8, p, src, K, p, p, p, p, P, 64, 8, 128, p, p, 1 << 20,
                                                               0, None)
    assert ga(None, 2, 32) == NULL        # no gather list
    assert ga(p, 3, 32) == SHAPE          # P is not a multiple of K
    assert ga(p, 0, 32) == SHAPE
    assert ga(None, 2, 0) == 0            # P = 0: no-op
    # expert block as an id list
    li = lambda ids, n, src, K, P: lib.moe_expert_list_forward(ids, n, p, src, K, p, p, p, p, P, 64, 8, 128, p, p, 1 << 20,
                                                               0, None)
    assert li(None, 3, None, 1, 32) == NULL
    assert li(p, 0, None, 1, 32) == SHAPE        # empty list
    assert li(p, 9, None, 1, 32) == SHAPE        # more ids than experts
    assert li(p, 3, p, 5, 32) == SHAPE           # gather form: P not a multiple of K
    assert li(p, 3, None, 1, 0) == 0             # P = 0: no-op
    # shared expert
    assert lib.moe_shared_forward(p, p, p, p, p, 4, 64, 96, p, p, p, 1 << 20, None) == SHAPE
    assert lib.moe_shared_forward(p, p, p, p, p, 4, 64, 128, p, None, p, 1 << 20, None) == NULL
    assert lib.moe_shared_forward(p, p, p, p, p, 4, 64, 128, p, p, p, 8, None) == WS
    # kernel policies that do not exist (1, 2, 6 and 7 named kernels that have been removed) and stray bits
    ex = lambda pol: lib.moe_expert_group_forward_ex(0, 8, p, p, p, p, p, 32, 64, 8, 128, p, p, 1 << 20, pol, None)
    shx = lambda pol: lib.moe_shared_forward_ex(p, p, p, p, p, 4, 64, 128, p, p, p, 1 << 20, pol, None)
    for pol in (1, 2, 6, 7, 12, 255, 0x800, 0x1003):
        assert ex(pol) == SHAPE and shx(pol) == SHAPE, pol
    # gating and the inter-layer step keep a token row in registers: H <= 8192
    assert lib.moe_route(p, p, None, 4, 8256, 8, 2, 0, p, p, None) == SHAPE
    assert lib.moe_route_segments(p, p, p, p, 2, 4, 8256, 8, 2, 0, p, p, None) == SHAPE
    assert lib.moe_residual_norm(p, p, 4, 8256, ctypes.c_float(1e-6), p, None) == SHAPE
    # block call that hosts the shared experts
    fu = lambda T, I, Is, ws, pol=0, x=p, E=8: lib.moe_expert_group_forward_fused(0, 8, x, p, 2, p, p, p, p, p, p, p, p, T, 64,
                                                                                  E, I, Is, p, p, p, p, ws, pol, None)
    assert lib.moe_fused_shared_sets(512, 64, 8, 2, 128, 512) == 4
    assert lib.moe_fused_shared_sets(512, 64, 8, 2, 128, 448) == 0          # Is is not a multiple of I
    assert lib.moe_fused_shared_sets(512, 64, 8, 2, 128, 128 * 9) == 0      # more than 8 sets
    assert lib.moe_fused_shared_sets(64, 64, 60, 2, 128, 512) == 0          # a batch for the weight-streaming kernels
    assert lib.moe_fused_shared_sets(512, 64, 254, 2, 128, 512) == 0        # E + sets > 256
    assert lib.moe_fused_workspace_bytes(512, 2, 128, 512) == (1024 + 4 * 512) * 128 * 2
    assert fu(512, 128, 448, 1 << 24) == SHAPE
    assert fu(64, 128, 512, 1 << 24, E=60) == SHAPE
    assert fu(512, 128, 512, 1 << 24, 9) == SHAPE                           # streaming kernels cannot host them
    assert fu(512, 128, 512, 1 << 24, 8) == SHAPE
    assert fu(512, 128, 512, 1000) == WS
    assert fu(512, 128, 512, 1 << 24, 0, None) == NULL
    assert fu(0, 128, 512, 0) == 0
    assert lib.moe_combine_parts(p, p, p, p, 0, p, 4, 64, 2, p, None) == SHAPE
    assert lib.moe_combine_parts(p, p, p, p, 9, p, 4, 64, 2, p, None) == SHAPE
    assert lib.moe_combine_parts(p, p, p, None, 2, p, 4, 64, 2, p, None) == NULL
    assert lib.moe_combine_parts(p, p, p, p, 2, None, 4, 64, 2, p, None) == NULL
    # combine
    assert lib.moe_combine(p, p, p, p, None, 4, 64, 2, p, None) == NULL      # S without sg
    assert lib.moe_combine(p, p, p, None, None, 4, 64, 17, p, None) == SHAPE
    assert lib.moe_combine(None, p, p, None, None, 4, 64, 2, p, None) == NULL
    # the clock record of the tile kernels (a per-thread setting, no GPU call)
    assert lib.moe_tile_clock_buffer(p, 0) == SHAPE
    assert lib.moe_tile_clock_buffer(p, -3) == SHAPE
    assert lib.moe_tile_clock_buffer(None, 0) == 0
    assert lib.moe_tile_clock_buffer(None, 7) == 0                          # off, whatever the count
    # the MFMA rate probe
    assert lib.moe_probe_mfma(None, 32768, 10, 1, p, None) == NULL
    assert lib.moe_probe_mfma(p, 32768, 10, 1, None, None) == NULL
    assert lib.moe_probe_mfma(p, 32767, 10, 1, p, None) == SHAPE            # operand buffer too small
    assert lib.moe_probe_mfma(p, 32768, 0, 1, p, None) == SHAPE
    assert lib.moe_probe_mfma(p, 32768, 10, 0, p, None) == SHAPE
    assert lib.moe_probe_mfma(p, 32768, 10, 65536, p, None) == SHAPE


def test_balanced_blocks_partition_and_balance():
    from paper_2604_26881_amd.binding import balanced_blocks
    rng = np.random.default_rng(3)
    for E, nb in ((60, 3), (60, 4), (60, 7), (8, 8), (5, 9), (1, 1)):
        rows = (rng.zipf(1.3, size=E) % 500).tolist()
        blocks = balanced_blocks(rows, nb)
        assert len(blocks) == min(nb, E)
        flat = sorted(e for b in blocks for e in b)
        assert flat == list(range(E))                        # every expert exactly once
        assert all(b == sorted(b) for b in blocks)
        loads = [sum(rows[e] for e in b) for b in blocks]
        assert max(loads) - min(loads) <= max(rows)          # greedy bound: spread at most one item
    assert balanced_blocks([5, 5, 5, 5], 2) == [[0, 2], [1, 3]]


def test_segment_offsets_accepts_only_consecutive_slices():
    from paper_2604_26881_amd import segment_offsets
    assert segment_offsets([(0, 3), (3, 3), (3, 10)], 10, "cpu").tolist() == [0, 3, 3, 10]
    assert segment_offsets([(0, 3), (4, 10)], 10, "cpu") is None      # a gap
    assert segment_offsets([(3, 10), (0, 3)], 10, "cpu") is None      # out of order
    assert segment_offsets([(0, 3), (3, 9)], 10, "cpu") is None       # does not cover the batch


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout
