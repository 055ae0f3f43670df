"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

``tests/sanitize_driver.c`` is linked with ``oracle/moe_oracle.c`` under
``-fsanitize=address,undefined`` (sanitizer runtimes linked statically, so the program needs no
preloaded library), runs every exported function on small layers (top-k = all experts, experts
without rows, bias, shared expert, an empty batch) and dumps its outputs.  The test requires a clean
exit with no sanitizer report, and every dumped array to equal, bit for bit, what the ordinary build
of the oracle returns for the same inputs: an out-of-bounds read that happened to land on mapped
memory, or arithmetic that relies on undefined behaviour, would show in one of the two.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CASES = [  # T, H, E, K, I, Is, renorm, bias, cut  (the same table as in sanitize_driver.c)
    (16, 64, 8, 2, 128, 0, 0, 0, 3), (33, 128, 12, 4, 64, 192, 1, 1, 5), (5, 8, 3, 3, 16, 8, 0, 1, 1),
    (40, 72, 20, 1, 24, 0, 1, 0, 19), (0, 64, 4, 2, 64, 64, 0, 1, 2),
]


def draw(stream: int, n: int, scale: float) -> np.ndarray:
    """The driver's input formula: value i of stream s (uint32 arithmetic, wrapping)."""
    i = np.arange(n, dtype=np.uint64)
    v = ((i + 1) * 2654435761 + stream * 40503) & 0xFFFFFFFF
    v ^= v >> 15
    v = (v * 2246822519) & 0xFFFFFFFF
    v ^= v >> 13
    return ((v & 511).astype(np.float32) - np.float32(256.0)) * np.float32(1.0 / 256.0) * np.float32(scale)


@pytest.fixture(scope="module")
def dump(tmp_path_factory):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    d = tmp_path_factory.mktemp("san")
    exe, out = str(d / "oracle_san"), str(d / "out.bin")
    cmd = [gcc, "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-mfma", "-ffp-contract=off", "-fopenmp", "-DREAL=double",
           os.path.join(ROOT, "oracle", "moe_oracle.c"), os.path.join(ROOT, "tests", "sanitize_driver.c"), "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, out], capture_output=True, text=True, timeout=300, env=env)
    report = r.stdout + r.stderr
    assert r.returncode == 0, report
    assert "runtime error" not in report and "AddressSanitizer" not in report and "LeakSanitizer" not in report, report
    assert "5 cases done" in r.stdout
    return np.fromfile(out, dtype=np.uint8)


def test_sanitized_oracle_runs_clean_and_matches_the_ordinary_build(dump, oracle64):
    pos = 0

    def take(dtype, shape):
        nonlocal pos
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        a = dump[pos:pos + n].view(dtype).reshape(shape)
        pos += n
        return a

    def same(a, b, what):
        assert a.shape == b.shape and a.dtype == b.dtype, what
        assert a.tobytes() == b.tobytes(), what

    for c, (T, H, E, K, I, Is, renorm, with_bias, cut) in enumerate(CASES):
        s = c * 16
        x = draw(s + 0, T * H, 1.0).reshape(T, H)
        Wr = draw(s + 1, E * H, 0.125).reshape(E, H)
        bias = draw(s + 2, E, 2.0) if with_bias else None
        Wg = draw(s + 3, E * I * H, 0.125).reshape(E, I, H)
        Wu = draw(s + 4, E * I * H, 0.125).reshape(E, I, H)
        Wd = draw(s + 5, E * H * I, 0.125).reshape(E, H, I)
        shared = None
        if Is:
            shared = (draw(s + 6, Is * H, 0.125).reshape(Is, H), draw(s + 7, Is * H, 0.125).reshape(Is, H),
                      draw(s + 8, H * Is, 0.125).reshape(H, Is), draw(s + 9, H, 0.125))
        P = T * K
        what = f"case {c}"
        ids, w, logits = oracle64.route(x, Wr, bias, K, renorm, want_logits=True)
        same(take(np.int32, (T, K)), ids, what + " ids")
        same(take(np.float32, (T, K)), w, what + " w")
        same(take(np.float32, (T, E)), logits, what + " logits")
        off, src, rowp = oracle64.permute(ids, E)
        same(take(np.int32, (E + 1,)), off, what + " offsets")
        same(take(np.int32, (P,)), src, what + " src_of_row")
        same(take(np.int32, (P,)), rowp, what + " row_of_pair")
        Xp = oracle64.gather(x, src, K)
        same(take(np.float32, (P, H)), Xp, what + " Xp")
        Yp = np.zeros((P, H), np.float64)
        oracle64.expert_group_forward(cut, E, Xp, off, Wg, Wu, Wd, Yp)
        oracle64.expert_group_forward(0, cut, Xp, off, Wg, Wu, Wd, Yp)
        same(take(np.float64, (P, H)), Yp, what + " Yp")
        S = sg = None
        if Is:
            S, sg = oracle64.shared_forward(x, *shared)
            same(take(np.float64, (T, H)), S, what + " S")
            same(take(np.float64, (T,)), sg, what + " sg")
        out = oracle64.combine(Yp, rowp, w, S, sg, K) if T > 0 else np.empty((0, H))
        same(take(np.float64, (T, H)), out, what + " out")
        tok = np.arange(T - 1, -1, -1, dtype=np.int32)
        tout, tids, tw = oracle64.token_forward(tok, x, Wr, bias, Wg, Wu, Wd, shared, K, renorm)
        same(take(np.float64, (T, H)), tout, what + " token_forward out")
        same(take(np.int32, (T, K)), tids, what + " token_forward ids")
        same(take(np.float32, (T, K)), tw, what + " token_forward w")
        same(take(np.float32, (T, H)), oracle64.residual_norm(x, out, 1e-6), what + " residual_norm")
    assert pos == dump.size
