"""Pins for the CPU oracle (no GPU needed).

The paper prints no number for the MoE-layer path (no worked example, no table of values), so
the oracle is pinned by what the mathematics fixes: hand-worked cases, closed forms, library
routines on special cases, a dense brute force written separately in numpy, and invariants the
paper states (block size does not change the result, Sec. 3; micro-batching keeps routing
correct, Sec. 4.1).
"""
import numpy as np
import pytest
import torch

import workloads
from tests import bruteforce as bf


def _np(w):
    return w.f32_numpy()


def _shared(d):
    return None if d["Wsg"] is None else (d["Wsg"], d["Wsu"], d["Wsd"], d["wgate"])


# ------------------------------------------------------------------ router dot product

def test_router_dot_exact_on_integers(oracle64):
    # small integers: every partial sum is exact in fp32, so any summation order must give the
    # exact integer dot product; a dropped or doubled term, or a wrong index, changes it.
    rng = np.random.default_rng(0)
    for H in (8, 64, 72, 512, 520, 2048):
        x = rng.integers(-8, 9, size=(5, H)).astype(np.float32)
        Wr = rng.integers(-8, 9, size=(7, H)).astype(np.float32)
        _, _, logits = oracle64.route(x, Wr, None, K=1, renorm=False, want_logits=True)
        exact = x.astype(np.int64) @ Wr.astype(np.int64).T
        assert np.array_equal(logits.astype(np.int64), exact)
        assert np.array_equal(logits, exact.astype(np.float32))


def test_router_dot_order_hand_worked(oracle64):
    # Hand-worked cases where the summation order changes the fp32 result (w = 1 everywhere, so the
    # products are the x values).  Element h goes to partial (h/8) mod 64; the partials are folded
    # by a[j] += a[j xor s] for s = 1, 2, 4, ...
    H = 64
    Wr = np.ones((1, H), np.float32)

    def logit(values):
        x = np.zeros((1, H), np.float32)
        for h, v in values.items():
            x[0, h] = v
        return oracle64.route(x, Wr, None, K=1, renorm=False, want_logits=True)[2][0, 0]

    B = 2.0 ** 24
    # partials p0 = 2^24 (h=0), p1 = 1 (h=8), p2 = -2^24 (h=16), p3 = 1 (h=24).
    # stride 1: p0+p1 = 2^24+1 -> rounds to 2^24 (tie to even); p2+p3 = -2^24+1 = -16777215 (exact).
    # stride 2: 2^24 - 16777215 = 1.   Strides 4..32 add zeros.
    # (Folding stride 2 first would give (p0+p2) + (p1+p3) = 0 + 2 = 2; one left-to-right sum gives
    #  2^24+1 -> 2^24, -2^24 -> 0, +1 -> 1 as well, which the next case separates.)
    assert logit({0: B, 8: 1.0, 16: -B, 24: 1.0}) == 1.0
    # partials p0 = 2^24, p1 = -2^24, p2 = 1, p3 = 1: stride 1: 0 and 2; stride 2: 2.
    # and p0 = 2^24, p1 = 1, p2 = 1, p3 = -2^24: stride 1: 2^24 and -16777215; stride 2: 1
    # (a left-to-right sum gives 2^24+1 -> 2^24, +1 -> 2^24, -2^24 -> 0).
    assert logit({0: B, 8: -B, 16: 1.0, 24: 1.0}) == 2.0
    assert logit({0: B, 8: 1.0, 16: 1.0, 24: -B}) == 1.0

    # Same partial, sequential: x[0] = 2^24, x[1] = 1, x[2] = 1 all fall in partial 0:
    # 2^24 + 1 rounds back to 2^24 twice; a pairwise order would give 2^24 + 2.
    assert logit({0: B, 1: 1.0, 2: 1.0}) == B

    # Wrap-around and the widest stride, H = 1024: h = 0 and h = 512 share partial 0
    # ((512/8) mod 64 = 0) and are taken in ascending h: 2^24 + 1 -> 2^24, then h = 513: again 2^24.
    H = 1024
    Wr = np.ones((1, H), np.float32)
    assert logit({0: B, 512: 1.0, 513: 1.0}) == B
    # ... while h = 8 and h = 9 sit in partial 1 and survive: 2^24 + (1 + 1).
    assert logit({0: B, 8: 1.0, 9: 1.0}) == B + 2.0
    # partials p0 = 2^24 (h=0), p32 = 1 (h=256), p33 = 1 (h=264), p1 = -2^24 (h=8):
    # stride 1: (p0+p1) = 0 in partials 0,1; (p32+p33) = 2 in partials 32,33; stride 32: 0 + 2 = 2.
    # With the widest stride first: (p0+p32) = 2^24+1 -> 2^24, (p1+p33) = -2^24+1 = -16777215, sum 1.
    assert logit({0: B, 256: 1.0, 264: 1.0, 8: -B}) == 2.0


def test_router_dot_fused_multiply_add(oracle64):
    # One product that is not representable in fp32: (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24.
    # With a fused multiply-add, -1 + that product = 2^-11 + 2^-24 exactly; an unfused
    # multiply rounds the product to 1 + 2^-11 first and gives 2^-11.
    H = 8
    a = np.float32(1.0 + 2.0 ** -12)
    x = np.zeros((1, H), np.float32)
    Wr = np.zeros((1, H), np.float32)
    x[0, 0], Wr[0, 0] = -1.0, 1.0
    x[0, 1], Wr[0, 1] = a, a
    _, _, logits = oracle64.route(x, Wr, None, K=1, renorm=False, want_logits=True)
    assert logits[0, 0] == np.float32(2.0 ** -11 + 2.0 ** -24)


def test_router_logits_close_to_float64_matmul(oracle64):
    d = _np(workloads.tiny(seed=0, with_bias=True))
    _, _, logits = oracle64.route(d["x"], d["Wr"], d["bias"], K=2, renorm=False, want_logits=True)
    ref = d["x"].astype(np.float64) @ d["Wr"].astype(np.float64).T + d["bias"].astype(np.float64)
    assert np.abs(logits - ref).max() < 5e-6


def test_router_dot_order_in_numpy(oracle64):
    # the fixed order written a second time with numpy vector operations (bf16-valued inputs,
    # so every product is exact in fp32 and a*b+c rounds once either way): bit-equal logits.
    w = workloads.decode(seed=11, T=9, E=12, I=64, Is=0)
    d = _np(w)
    x, Wr = d["x"], d["Wr"]
    H = x.shape[1]
    a = np.zeros((x.shape[0], Wr.shape[0], 64), np.float32)
    for c in range(0, H, 512):
        for i in range(8):
            cols = c + 8 * np.arange(64) + i
            ok = cols < H
            prod = x[:, None, cols[ok]] * Wr[None, :, cols[ok]]
            a[:, :, ok] = a[:, :, ok] + prod
    for s in (1, 2, 4, 8, 16, 32):
        a = a + a[:, :, np.arange(64) ^ s]
    _, _, logits = oracle64.route(x, Wr, None, K=4, renorm=False, want_logits=True)
    assert np.array_equal(logits, a[:, :, 0])


# ------------------------------------------------------------------ selection and weights

def test_zero_router_ties_to_lowest_ids(oracle64):
    T, H, E = 5, 64, 8
    x = np.random.default_rng(1).standard_normal((T, H)).astype(np.float32)
    Wr = np.zeros((E, H), np.float32)
    for K in (1, 3, 8):
        ids, w = oracle64.route(x, Wr, None, K=K, renorm=False)
        assert np.array_equal(ids, np.tile(np.arange(K, dtype=np.int32), (T, 1)))
        assert np.allclose(w, 1.0 / E, rtol=1e-6)
        ids, w = oracle64.route(x, Wr, None, K=K, renorm=True)
        assert np.allclose(w, 1.0 / K, rtol=1e-6)


def test_negative_zero_ties_with_positive_zero(oracle64):
    # logits -0.0 (expert 0) and +0.0 (expert 1) compare equal, so expert 0 comes first
    x = np.zeros((1, 8), np.float32)
    x[0, 0] = 1.0
    Wr = np.zeros((3, 8), np.float32)
    Wr[0, 0] = -0.0
    Wr[2, 0] = -1.0
    ids, _ = oracle64.route(x, Wr, None, K=3, renorm=False)
    assert ids.tolist() == [[0, 1, 2]]


def test_unit_vectors_known_order(oracle64):
    # x = e_i, Wr[e] = c_e * e_i  =>  logit[e] = c_e; the order of c is the answer
    H, E = 64, 6
    c = np.array([0.5, -1.0, 3.0, 2.0, 3.0, 0.25], np.float32)     # experts 2 and 4 tie at 3
    for i in (0, 9, 63):
        x = np.zeros((1, H), np.float32)
        x[0, i] = 1.0
        Wr = np.zeros((E, H), np.float32)
        Wr[:, i] = c
        ids, w = oracle64.route(x, Wr, None, K=E, renorm=False)
        assert ids.tolist() == [[2, 4, 3, 0, 5, 1]]
        p = np.exp(c.astype(np.float64))
        p /= p.sum()
        assert np.allclose(w[0], p[ids[0]], rtol=1e-6)
        assert abs(w.sum() - 1.0) < 1e-6


def test_duplicate_router_rows_lower_id_wins(oracle64):
    d = _np(workloads.tiny(seed=3))
    Wr = d["Wr"].copy()
    Wr[5] = Wr[1]
    Wr[6] = Wr[1]
    ids, _, logits = oracle64.route(d["x"], Wr, None, K=8, renorm=False, want_logits=True)
    for t in range(ids.shape[0]):
        pos = {int(e): j for j, e in enumerate(ids[t])}
        assert pos[1] + 1 == pos[5] and pos[5] + 1 == pos[6]
        assert logits[t, 1] == logits[t, 5] == logits[t, 6]


def test_bias_is_added_after_the_reduction(oracle64):
    d = _np(workloads.tiny(seed=4))
    b = np.linspace(-1, 1, 8).astype(np.float32)
    _, _, l0 = oracle64.route(d["x"], d["Wr"], None, K=2, renorm=False, want_logits=True)
    _, _, l1 = oracle64.route(d["x"], d["Wr"], b, K=2, renorm=False, want_logits=True)
    assert np.array_equal(l1, l0 + b[None, :])


@pytest.mark.parametrize("K", [1, 2, 8])
@pytest.mark.parametrize("renorm", [False, True])
def test_selection_equals_full_sort_and_softmax_library(oracle64, K, renorm):
    d = _np(workloads.tiny(seed=0, with_bias=True))
    ids, w, logits = oracle64.route(d["x"], d["Wr"], d["bias"], K=K, renorm=renorm, want_logits=True)
    assert np.array_equal(ids, bf.select(logits, K))
    p = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    wref = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if renorm:
        wref = wref / wref.sum(axis=1, keepdims=True)
    assert np.abs(w - wref).max() < 1e-6
    # invariants: K distinct experts, descending logits, weights sum to 1 when renormalised
    for t in range(ids.shape[0]):
        assert len(set(ids[t].tolist())) == K
        lt = logits[t, ids[t]]
        assert np.all(lt[:-1] >= lt[1:])
    s = w.sum(axis=1)
    assert np.all(s <= 1 + 1e-6)
    if renorm or K == 8:
        assert np.allclose(s, 1.0, atol=1e-6)


def test_selection_on_random_shapes_with_many_ties(oracle64):
    # logits from a tiny integer alphabet: ties everywhere, the full sort decides
    rng = np.random.default_rng(5)
    for (T, E, K) in [(33, 60, 4), (7, 5, 5), (64, 17, 1), (20, 64, 8)]:
        H = 8
        x = np.zeros((T, H), np.float32)
        x[:, 0] = 1.0
        Wr = np.zeros((E, H), np.float32)
        Wr[:, 0] = rng.integers(-2, 3, size=E)
        bias = rng.integers(-1, 2, size=E).astype(np.float32)
        ids, _, logits = oracle64.route(x, Wr, bias, K=K, renorm=False, want_logits=True)
        assert np.array_equal(ids, bf.select(logits, K))


def test_route_is_row_independent(oracle64):
    d = _np(workloads.tiny(seed=6, T=40))
    ids, w = oracle64.route(d["x"], d["Wr"], None, K=2, renorm=True)
    ids2, w2 = oracle64.route(d["x"][13:29], d["Wr"], None, K=2, renorm=True)
    assert np.array_equal(ids[13:29], ids2) and np.array_equal(w[13:29], w2)


# ------------------------------------------------------------------ permutation

@pytest.mark.parametrize("T,E,K", [(16, 8, 2), (128, 60, 4), (1, 4, 4), (300, 7, 3), (0, 5, 2)])
def test_permute_equals_stable_argsort(oracle64, T, E, K):
    rng = np.random.default_rng(T + E)
    ids = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32) if T else \
        np.zeros((0, K), np.int32)
    offsets, src, rowp = oracle64.permute(ids, E)
    flat = ids.ravel()
    P = T * K
    assert np.array_equal(src, np.argsort(flat, kind="stable").astype(np.int32))
    counts = np.bincount(flat, minlength=E)
    assert np.array_equal(np.diff(offsets), counts)
    assert offsets[0] == 0 and offsets[E] == P
    assert np.array_equal(src[rowp], np.arange(P))            # inverse of each other
    assert np.array_equal(rowp[src], np.arange(P))
    assert np.all(np.diff(flat[src]) >= 0)                    # rows grouped by expert
    for e in range(E):                                        # ascending pair order inside
        seg = src[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0) and np.all(flat[seg] == e)


def test_gather_copies_the_tokens_rows(oracle64):
    d = _np(workloads.tiny(seed=7))
    ids, _ = oracle64.route(d["x"], d["Wr"], None, K=2, renorm=False)
    _, src, rowp = oracle64.permute(ids, 8)
    Xp = oracle64.gather(d["x"], src, 2)
    for p in range(32):
        assert np.array_equal(Xp[rowp[p]], d["x"][p // 2])


def test_permute_then_unpermute_is_identity(oracle64):
    # one-hot gate weights on slot 0 and experts that copy nothing: combine of the gathered rows
    # themselves (Yp := Xp) with w = (1, 0) gives x back
    d = _np(workloads.tiny(seed=8))
    ids, _ = oracle64.route(d["x"], d["Wr"], None, K=2, renorm=False)
    _, src, rowp = oracle64.permute(ids, 8)
    Xp = oracle64.gather(d["x"], src, 2)
    w = np.zeros((16, 2), np.float32)
    w[:, 0] = 1.0
    out = oracle64.combine(Xp.astype(np.float64), rowp, w, None, None, 2)
    assert np.array_equal(out, d["x"].astype(np.float64))


# ------------------------------------------------------------------ expert FFN

def test_single_expert_is_a_dense_swiglu_mlp(oracle64):
    # E = 1, K = 1: the gate weight is exactly 1 and the layer is one SwiGLU MLP; compare with
    # torch's CPU matmul and F.silu in float64.
    w = workloads.tiny(seed=9, T=24, E=1, K=1, I=96)
    d = _np(w)
    res = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], None, 1, False)
    assert np.all(res["w"] == 1.0) and np.all(res["ids"] == 0)
    x = w.x.double()
    ref = (torch.nn.functional.silu(x @ w.Wg[0].double().T) * (x @ w.Wu[0].double().T)) @ w.Wd[0].double().T
    assert np.abs(res["out"] - ref.numpy()).max() <= 1e-12 * np.abs(ref.numpy()).max() + 1e-15


def test_ffn_linear_in_down_projection_and_zero_up(oracle64):
    d = _np(workloads.tiny(seed=10))
    a = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], None, 2, False)["out"]
    b = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], 2 * d["Wd"], None, 2, False)["out"]
    assert np.array_equal(b, 2 * a)                  # scaling by 2 is exact in binary floating point
    z = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], 0 * d["Wu"], d["Wd"], None, 2, False)["out"]
    assert np.all(z == 0)


def test_gate_and_up_are_not_swapped(oracle64):
    # silu acts on the gate branch only: with Wu = row-selector of ones and Wg large positive,
    # silu(g) ~ g, with Wg large negative silu(g) ~ 0.
    H, I = 8, 8
    x = np.ones((1, H), np.float32)
    Wr = np.zeros((1, H), np.float32)
    Wg = np.full((1, I, H), -10.0, np.float32)       # g = -80 -> silu ~ 0
    Wu = np.full((1, I, H), 1.0, np.float32)         # u = 8
    Wd = np.full((1, H, I), 1.0, np.float32)
    out = oracle64.layer(x, Wr, None, Wg, Wu, Wd, None, 1, False)["out"]
    assert np.all(np.abs(out) < 1e-30)
    out = oracle64.layer(x, Wr, None, Wu, Wg, Wd, None, 1, False)["out"]   # swapped roles
    g = 8.0
    expect = I * (g / (1 + np.exp(-g))) * (-80.0)
    assert np.allclose(out, expect, rtol=1e-12)


# ------------------------------------------------------------------ whole layer

@pytest.mark.parametrize("renorm", [False, True])
@pytest.mark.parametrize("shared", [False, True])
def test_layer_equals_dense_brute_force(oracle64, renorm, shared):
    w = workloads.tiny(seed=0, renorm=renorm, Is=(64 if shared else 0), with_bias=True)
    d = _np(w)
    res = oracle64.layer(d["x"], d["Wr"], d["bias"], d["Wg"], d["Wu"], d["Wd"], _shared(d), 2, renorm)
    _, _, logits = oracle64.route(d["x"], d["Wr"], d["bias"], 2, renorm, want_logits=True)
    ref, ids, wref = bf.dense_layer(d["x"], d["Wr"], d["bias"], d["Wg"], d["Wu"], d["Wd"], _shared(d), 2,
                                    renorm, logits=logits)
    assert np.array_equal(res["ids"], ids)
    assert np.abs(res["w"] - wref).max() < 1e-6
    scale = np.abs(ref).max()
    # the fp32 gate weights are the only fp32 quantity left in the output: 1e-6 relative
    assert np.abs(res["out"] - ref).max() <= 2e-6 * scale
    # and with the oracle's own fp32 weights put into the brute force, only summation order is left
    full = np.zeros((16, 8))
    np.put_along_axis(full, ids.astype(np.int64), res["w"].astype(np.float64), axis=1)
    ref2 = sum(full[:, e:e + 1] * bf.swiglu_ffn(d["x"], d["Wg"][e], d["Wu"][e], d["Wd"][e]) for e in range(8))
    if shared:
        gate = 1 / (1 + np.exp(-(d["x"].astype(np.float64) @ d["wgate"].astype(np.float64))))
        ref2 = ref2 + gate[:, None] * bf.swiglu_ffn(d["x"], d["Wsg"], d["Wsu"], d["Wsd"])
    assert np.abs(res["out"] - ref2).max() <= 1e-12 * scale


def test_layer_equals_dense_brute_force_qwen_proportions(oracle64):
    # a scaled-down Qwen-shaped layer (60 experts top-4, shared expert with sigmoid gate, bf16 values)
    w = workloads.prefill(seed=2, T=48, H=128, I=64, Is=256)
    d = _np(w)
    res = oracle64.layer(d["x"], d["Wr"], d["bias"], d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False)
    _, _, logits = oracle64.route(d["x"], d["Wr"], d["bias"], 4, False, want_logits=True)
    ref, ids, _ = bf.dense_layer(d["x"], d["Wr"], d["bias"], d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False,
                                 logits=logits)
    assert np.array_equal(res["ids"], ids)
    assert np.abs(res["out"] - ref).max() <= 2e-6 * np.abs(ref).max()


def test_token_definition_equals_path_form(oracle64):
    w = workloads.decode(seed=12, T=40, H=128, E=12, I=64, Is=128)
    d = _np(w)
    res = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False,
                         groups=workloads.partition(12, 5))
    tok = np.array([0, 7, 39, 7, 20], np.int32)
    out, ids, wt = oracle64.token_forward(tok, d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4,
                                          False)
    assert np.array_equal(ids, res["ids"][tok]) and np.array_equal(wt, res["w"][tok])
    assert np.abs(out - res["out"][tok]).max() <= 1e-13 * np.abs(res["out"]).max()


def test_identical_experts_with_renorm_give_the_plain_ffn(oracle64):
    w = workloads.tiny(seed=13, renorm=True)
    d = _np(w)
    for name in ("Wg", "Wu", "Wd"):
        d[name] = np.repeat(d[name][:1], 8, axis=0)
    out = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], None, 2, True)["out"]
    ref = bf.swiglu_ffn(d["x"], d["Wg"][0], d["Wu"][0], d["Wd"][0])
    assert np.abs(out - ref).max() <= 1e-6 * np.abs(ref).max()


def test_token_permutation_equivariance(oracle64):
    d = _np(workloads.tiny(seed=14, Is=64))
    perm = np.random.default_rng(14).permutation(16)
    a = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 2, False)["out"]
    b = oracle64.layer(d["x"][perm], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 2, False)["out"]
    assert np.array_equal(a[perm], b)


def test_block_size_does_not_change_the_result(oracle64):
    # Sec. 3: changing the expert-block size must not change model semantics
    w = workloads.tenants(seed=3, n_tenants=2, T_per=12, H=64, I=64, Is=64)
    d = _np(w)
    bias = d["bias"][0]
    outs = []
    for g in (1, 4, 15, 60, 6, 20, 30, 7):
        groups = workloads.partition(60, g)
        outs.append(oracle64.layer(d["x"], d["Wr"], bias, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False,
                                   groups=groups)["out"])
    groups = workloads.partition(60, 4)[::-1]                           # any order of the blocks
    outs.append(oracle64.layer(d["x"], d["Wr"], bias, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False,
                               groups=groups)["out"])
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


def test_group_call_writes_only_its_rows(oracle64):
    d = _np(workloads.tiny(seed=15))
    ids, _ = oracle64.route(d["x"], d["Wr"], None, 2, False)
    offsets, src, _ = oracle64.permute(ids, 8)
    Xp = oracle64.gather(d["x"], src, 2)
    Yp = np.full((32, 64), 777.0)
    oracle64.expert_group_forward(2, 5, Xp, offsets, d["Wg"], d["Wu"], d["Wd"], Yp)
    assert np.all(Yp[:offsets[2]] == 777.0) and np.all(Yp[offsets[5]:] == 777.0)
    assert not np.any(Yp[offsets[2]:offsets[5]] == 777.0)


def test_shared_expert_with_zero_gate_vector_counts_half(oracle64):
    d = _np(workloads.tiny(seed=16, Is=64))
    d["wgate"] = np.zeros_like(d["wgate"])
    for name in ("Wg", "Wu", "Wd"):
        d[name] = np.zeros_like(d[name])
    out = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 2, False)["out"]
    ref = 0.5 * bf.swiglu_ffn(d["x"], d["Wsg"], d["Wsu"], d["Wsd"])
    assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()


def test_tenant_slices_route_like_the_concatenation(oracle64):
    # Sec. 3 (orchestrator shared or per tenant): routing each tenant's slice with its own bias
    # equals routing the whole batch with the per-token bias
    w = workloads.tenants(seed=3, n_tenants=3, T_per=10, H=64, I=64, Is=0)
    d = _np(w)
    ids_all = []
    for i, (a, b) in enumerate(w.tenant_rows):
        ids, _ = oracle64.route(d["x"][a:b], d["Wr"], d["bias"][i], 4, False)
        ids_all.append(ids)
    ids_all = np.concatenate(ids_all)
    l = d["x"].astype(np.float64) @ d["Wr"].astype(np.float64).T + np.repeat(d["bias"], 10, axis=0)
    assert np.array_equal(ids_all, bf.select(l.astype(np.float32), 4))


# ------------------------------------------------------------------ precision of the reference

def test_float_build_agrees_with_double_build(oracle64, oracle32):
    w = workloads.decode(seed=1, T=24, H=256, E=12, I=192, Is=384)
    d = _np(w)
    a = oracle64.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False)
    b = oracle32.layer(d["x"], d["Wr"], None, d["Wg"], d["Wu"], d["Wd"], _shared(d), 4, False)
    assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["w"], b["w"])
    assert np.array_equal(a["row_of_pair"], b["row_of_pair"])
    err = np.abs(a["out"] - b["out"]).max() / np.abs(a["out"]).max()
    assert err < 1e-5          # three orders of magnitude under the 2e-2 parity bound


# ------------------------------------------------------------------ chaining layers

def test_residual_norm_closed_forms_and_library_rounding(oracle64):
    H = 64
    # constant rows: u = c everywhere, mean(u^2) = c^2, out = c / sqrt(c^2 + eps), rounded to bf16
    for c, d in ((1.0, 0.0), (0.5, 0.25), (-3.0, 1.0)):
        x = np.full((2, H), c, np.float32)
        y = np.full((2, H), d, np.float64)
        u = c + d
        expect = torch.tensor(u / np.sqrt(u * u + 1e-6), dtype=torch.float32).to(torch.bfloat16).float().item()
        out = oracle64.residual_norm(x, y, 1e-6)
        assert np.all(out == np.float32(expect))
    # random rows against the formula in numpy float64, rounded by torch's bf16 conversion
    rng = np.random.default_rng(3)
    x = torch.from_numpy(rng.standard_normal((9, 256)).astype(np.float32)).to(torch.bfloat16).float().numpy()
    y = rng.standard_normal((9, 256)) * 0.3
    u = x.astype(np.float64) + y
    ref = u / np.sqrt((u * u).mean(axis=1, keepdims=True) + 1e-6)
    ref_bf16 = torch.from_numpy(ref.astype(np.float32)).to(torch.bfloat16).float().numpy()
    out = oracle64.residual_norm(x, y, 1e-6)
    # double rounding (float64 -> float32 -> bf16) can move a value by one bf16 step in rare ties only
    assert np.mean(out != ref_bf16) < 1e-3
    assert np.abs(out - ref).max() <= 2.0 ** -8 * np.abs(ref).max()
    # rows come out with unit mean square (up to bf16 rounding)
    assert np.allclose((out.astype(np.float64) ** 2).mean(axis=1), 1.0, atol=5e-3)
    # a zero row stays zero (eps keeps the divisor finite)
    assert np.all(oracle64.residual_norm(np.zeros((1, H), np.float32), np.zeros((1, H)), 1e-6) == 0)
