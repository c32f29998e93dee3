"""Pins for the CPU oracle: facts fixed by the paper's definitions and by mathematics.

None of these retype the oracle's own formulae; each checks the oracle against a
closed form, a hand-derived example, an invariant, a special case that reduces to
something simpler, or an independently written brute force.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def random_layer(seed, T=7, E=5, H=4, F=6):
    g = rng(seed)
    return (g.standard_normal((T, H)), g.standard_normal((E, H)),
            g.standard_normal((E, F, H)), g.standard_normal((E, F, H)),
            g.standard_normal((E, H, F)))


# ----------------------------------------------------------------------------- O1
def test_expert_scalar_closed_form():
    # H = F = 1: gate = ln 3 -> sigmoid = 3/4; up = 2 ln 3; Y = 5 * (3/4 ln 3) * (2 ln 3)
    x = np.array([[math.log(3.0)]])
    logits, Y = oracle.expert_outputs(x, np.array([[7.0]]), np.array([[[1.0]]]),
                                      np.array([[[2.0]]]), np.array([[[5.0]]]))
    assert Y.shape == (1, 1, 1)
    assert Y[0, 0, 0] == pytest.approx(7.5 * math.log(3.0) ** 2, rel=1e-14)
    assert logits[0, 0] == pytest.approx(7.0 * math.log(3.0), rel=1e-14)


def test_expert_one_hot_indexing():
    # A single non-zero entry in each operand: catches any transposed or mis-indexed operand.
    T, E, H, F = 3, 2, 4, 5
    x = np.zeros((T, H)); x[1, 2] = 2.0
    Wg = np.zeros((E, H)); Wg[1, 2] = 3.0
    W1 = np.zeros((E, F, H)); W3 = np.zeros((E, F, H)); W2 = np.zeros((E, H, F))
    W1[1, 4, 2] = 0.5      # gate pre-activation 1.0 at f = 4
    W3[1, 4, 2] = -1.5     # up value -3.0
    W2[1, 3, 4] = 2.0      # lands in hidden unit 3
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    want = (1.0 / (1.0 + math.exp(-1.0))) * (-3.0) * 2.0
    expect = np.zeros((E, T, H)); expect[1, 1, 3] = want
    np.testing.assert_allclose(Y, expect, rtol=1e-14, atol=0)
    el = np.zeros((T, E)); el[1, 1] = 6.0
    np.testing.assert_array_equal(logits, el)


def test_expert_zero_branches_and_linearity():
    x, Wg, W1, W3, W2 = random_layer(1)
    _, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    _, Y0 = oracle.expert_outputs(x, Wg, W1, np.zeros_like(W3), W2)
    assert np.all(Y0 == 0.0)                                   # linear branch zero
    _, Yg = oracle.expert_outputs(x, Wg, np.zeros_like(W1), W3, W2)
    assert np.all(Yg == 0.0)                                   # silu(0) = 0
    _, Y2 = oracle.expert_outputs(x, Wg, W1, W3, 2.5 * W2)     # linear in W2
    np.testing.assert_allclose(Y2, 2.5 * Y, rtol=1e-13)
    _, Y3 = oracle.expert_outputs(x, Wg, W1, -W3, W2)          # odd in W3
    np.testing.assert_allclose(Y3, -Y, rtol=1e-13)
    # silu is not odd: silu(a) - silu(-a) = a  =>  Y(W1) - Y(-W1) = (x W1^T * x W3^T) W2^T
    _, Ym = oracle.expert_outputs(x, Wg, -W1, W3, W2)
    for e in range(len(W1)):
        lin = ((x @ W1[e].T) * (x @ W3[e].T)) @ W2[e].T
        np.testing.assert_allclose(Y[e] - Ym[e], lin, rtol=1e-11, atol=1e-11)


def test_silu_large_arguments():
    assert oracle.silu(np.array([50.0]))[0] == pytest.approx(50.0, rel=1e-15)
    assert abs(oracle.silu(np.array([-50.0]))[0]) < 1e-19
    assert oracle.silu(np.array([0.0]))[0] == 0.0


# ------------------------------------------------------------------------- Eq. 1
def test_routing_order_ties_go_to_lower_index():
    logits = np.array([[0.5, 2.0, 2.0, -1.0, 2.0], [1.0, 1.0, 1.0, 1.0, 1.0]])
    order = oracle.routing_order(logits)
    assert order[0].tolist() == [1, 2, 4, 0, 3]
    assert order[1].tolist() == [0, 1, 2, 3, 4]


def test_eq1_weights_sum_to_one_and_match_full_softmax():
    g = rng(2)
    logits = g.standard_normal((50, 8)) * 3.0
    order = oracle.routing_order(logits)
    k = 3
    sel = np.zeros_like(logits, dtype=bool)
    np.put_along_axis(sel, order[:, :k], True, axis=1)
    w = oracle.renormalised_weights(logits, sel)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-15)
    assert np.all(w[~sel] == 0.0)
    # The paper's route: softmax over ALL n logits, keep the top-k, divide by their sum.
    full = np.exp(logits) / np.exp(logits).sum(1, keepdims=True)
    topk = np.where(sel, full, 0.0)
    np.testing.assert_allclose(w, topk / topk.sum(1, keepdims=True), rtol=1e-12, atol=0)
    # shift invariance
    w2 = oracle.renormalised_weights(logits + 123.25, sel)
    np.testing.assert_allclose(w2, w, rtol=1e-12)


def test_layer_output_two_experts_closed_form():
    # weights (2/3, 1/3) from logits (ln 4, ln 2, ln 1), see tests/golden/hand_example_eq3.txt
    logits = np.log(np.array([[4.0, 2.0, 1.0]]))
    Y = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[1.0, 1.0]]])
    z = oracle.layer_output(logits, Y, 2)
    np.testing.assert_allclose(z, [[2.0 / 3.0, 1.0 / 3.0]], rtol=1e-15)


# ------------------------------------------------------------------ subset index
@pytest.mark.parametrize("E,r", [(4, 2), (8, 6), (8, 4), (16, 8), (16, 12), (5, 5), (6, 1)])
def test_subsets_each_once_in_lexicographic_order(E, r):
    subs = oracle.kept_subsets(E, r)
    assert len(subs) == math.comb(E, r) == math.comb(E, E - r)
    assert len(set(subs)) == len(subs)
    assert all(len(s) == r and list(s) == sorted(set(s)) for s in subs)
    assert all(a < b for a, b in zip(subs, subs[1:]))          # strictly increasing tuples
    assert subs[0] == tuple(range(r))
    masks = [oracle.subset_mask(s) for s in subs]
    assert all(bin(m).count("1") == r for m in masks)
    assert all(m < (1 << E) for m in masks)


# ------------------------------------------------------------------------- Eq. 3
def test_hand_example_golden():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "hand_example_eq3.txt"))
            if ln.strip() and not ln.startswith("#")]
    logits = np.log(np.array([[4.0, 2.0, 1.0]]))
    Y = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[1.0, 1.0]]])
    loss, amin, masks = oracle.prune_enumerate(logits, Y, k=2, r=2)
    assert len(rows) == len(loss) == 3
    for idx, mask, num, den in rows:
        assert masks[int(idx)] == int(mask)
        assert loss[int(idx)] == pytest.approx(float(Fraction(int(num), int(den))), rel=1e-14, abs=1e-300)
    assert amin == 0 and loss[0] == 0.0
    z_kept02 = oracle.pruned_layer_output(logits, Y, (0, 2), 2)
    np.testing.assert_allclose(z_kept02, [[1.0, 0.2]], rtol=1e-15)


def enumeration_case(seed, T=40, E=6, H=5):
    g = rng(seed)
    return g.standard_normal((T, E)), g.standard_normal((E, T, H))


def test_keep_all_experts_gives_exactly_zero():
    logits, Y = enumeration_case(3)
    for k in (1, 2, 3):
        loss, amin, masks = oracle.prune_enumerate(logits, Y, k, r=6)
        assert loss.tolist() == [0.0] and amin == 0 and masks.tolist() == [63]


@pytest.mark.parametrize("E,k,r,T", [(4, 2, 2, 64), (8, 2, 6, 33), (6, 3, 4, 50)])
def test_unaffected_pairs_are_exactly_zero_and_counted(E, k, r, T):
    # A token whose full top-k all survive in C contributes exactly 0; with generic
    # (tie-free) inputs those are the only zero pairs: T * C(E-k, r-k) of them.
    g = rng(4)
    logits, Y = g.standard_normal((T, E)), g.standard_normal((E, T, 3))
    subs = oracle.kept_subsets(E, r)
    zero_pairs = 0
    for t in range(T):
        lt, Yt = logits[t:t + 1], Y[:, t:t + 1, :]
        loss_t, _, _ = oracle.prune_enumerate(lt, Yt, k, r)
        top = set(np.argsort(-lt[0], kind="stable")[:k].tolist())
        for i, c in enumerate(subs):
            if top <= set(c):
                assert loss_t[i] == 0.0
            else:
                assert loss_t[i] > 0.0
        zero_pairs += int(np.sum(loss_t == 0.0))
    assert zero_pairs == T * math.comb(E - k, r - k)


def test_top1_special_case():
    # k = 1: the layer output is the arg-max expert's output; the pruned layer's is the
    # arg-max expert among the kept ones.
    logits, Y = enumeration_case(5, T=30, E=5, H=4)
    loss, _, _ = oracle.prune_enumerate(logits, Y, k=1, r=3)
    for i, c in enumerate(itertools.combinations(range(5), 3)):
        want = 0.0
        for t in range(30):
            e_full = int(np.argmax(logits[t]))
            e_kept = max(c, key=lambda e: logits[t, e])
            want += float(np.sum((Y[e_kept, t] - Y[e_full, t]) ** 2))
        assert loss[i] == pytest.approx(want, rel=1e-12, abs=1e-300)


def test_scale_law_shift_invariance_and_token_additivity():
    logits, Y = enumeration_case(6)
    loss, _, _ = oracle.prune_enumerate(logits, Y, 2, 4)
    loss_scaled, _, _ = oracle.prune_enumerate(logits, -3.0 * Y, 2, 4)
    np.testing.assert_allclose(loss_scaled, 9.0 * loss, rtol=1e-12)
    loss_shift, _, _ = oracle.prune_enumerate(logits + 2.0, Y, 2, 4)   # exact in binary for +2
    np.testing.assert_allclose(loss_shift, loss, rtol=1e-10)
    la, _, _ = oracle.prune_enumerate(logits[:17], Y[:, :17], 2, 4)
    lb, _, _ = oracle.prune_enumerate(logits[17:], Y[:, 17:], 2, 4)
    np.testing.assert_allclose(la + lb, loss, rtol=1e-12)
    ls, amin, _ = oracle.prune_enumerate_streamed(logits, Y, 2, 4, chunk=9)
    np.testing.assert_allclose(ls, loss, rtol=1e-12)
    assert amin == int(np.argmin(loss))


def test_expert_relabelling_permutes_subsets():
    logits, Y = enumeration_case(7, E=6)
    perm = rng(70).permutation(6)                 # new label p -> old expert perm[p]
    loss, _, _ = oracle.prune_enumerate(logits, Y, 2, 4)
    loss_p, _, _ = oracle.prune_enumerate(logits[:, perm], Y[perm], 2, 4)
    subs = oracle.kept_subsets(6, 4)
    index = {s: i for i, s in enumerate(subs)}
    for j, kept_new in enumerate(subs):
        kept_old = tuple(sorted(int(perm[p]) for p in kept_new))
        assert loss_p[j] == pytest.approx(loss[index[kept_old]], rel=1e-9)
    np.testing.assert_allclose(np.sort(loss_p), np.sort(loss), rtol=1e-9)


def test_quadratic_form_identity():
    # ||sum_e d_e Y_e||^2 = d^T (Y_t Y_t^T) d with d = pruned weights - full weights: the
    # identity the GPU path relies on, evaluated here with independently built d.
    logits, Y = enumeration_case(8, T=25, E=6, H=7)
    k, r = 2, 3
    loss, _, _ = oracle.prune_enumerate(logits, Y, k, r)
    for i, c in enumerate(itertools.combinations(range(6), r)):
        total = 0.0
        for t in range(25):
            l = logits[t]
            full = sorted(range(6), key=lambda e: (-l[e], e))[:k]
            kept = sorted(c, key=lambda e: (-l[e], e))[:k]
            d = np.zeros(6)
            d[kept] += np.exp(l[kept]) / np.exp(l[kept]).sum()
            d[full] -= np.exp(l[full]) / np.exp(l[full]).sum()
            G = Y[:, t, :] @ Y[:, t, :].T
            total += d @ G @ d
        assert loss[i] == pytest.approx(total, rel=1e-10)


@pytest.mark.parametrize("E,k,r,T,H", [(6, 2, 3, 40, 9), (8, 3, 5, 30, 5), (5, 1, 2, 25, 4), (7, 4, 2, 20, 6), (6, 2, 6, 10, 3)])
def test_gram_form_oracle_is_pinned_to_the_direct_definition(E, k, r, T, H):
    # the second oracle (per-token Gram matrix, fp64) against the direct definition, with ties and a
    # never-selected expert thrown in; identical argmin and masks, losses to 1e-10
    logits, Y = enumeration_case(23 + E + r, T=T, E=E, H=H)
    logits[::4, 1] = logits[::4, 0]
    logits[:, E - 1] = -1e9
    direct, amin, masks = oracle.prune_enumerate(logits, Y, k, r)
    gram, amin_g, masks_g = oracle.prune_enumerate_gram_form(logits, Y, k, r)
    np.testing.assert_allclose(gram, direct, rtol=1e-10, atol=1e-12 * max(direct.max(), 1.0))
    assert np.array_equal(masks, masks_g)
    assert amin_g == amin or direct[amin_g] == pytest.approx(direct[amin], rel=1e-10)
    if r == E:
        assert gram.tolist() == [0.0]


def test_planted_argmin():
    # Experts 1 and 4 get logits of -1e9 on every token: they are never routed to, so the
    # subset that drops exactly those two reproduces the layer and is the argmin with loss 0.
    logits, Y = enumeration_case(9, T=64, E=6, H=4)
    logits[:, [1, 4]] = -1e9
    loss, amin, masks = oracle.prune_enumerate(logits, Y, 2, 4)
    want = oracle.kept_subsets(6, 4).index((0, 2, 3, 5))
    assert amin == want and loss[want] == 0.0
    assert masks[want] == 0b101101
    assert np.all(np.delete(loss, want) > 0.0)
    # Both survivors of a subset at -1e9: Eq. 1 must still give finite (1/2, 1/2) weights.
    l2, _, _ = oracle.prune_enumerate(logits, Y, 2, 2)
    assert np.all(np.isfinite(l2))
    i14 = oracle.kept_subsets(6, 2).index((1, 4))
    z = oracle.pruned_layer_output(logits, Y, (1, 4), 2)
    np.testing.assert_allclose(z, 0.5 * (Y[1] + Y[4]), rtol=1e-14)
    assert l2[i14] > 0.0


def test_argmin_is_the_lowest_index_among_equal_losses():
    # Keeping five experts of six when two are never routed to: the two subsets that drop one of those two both
    # reproduce the layer exactly; the one that comes first in lexicographic order is the argmin.
    logits, Y = enumeration_case(11, T=40, E=6, H=4)
    logits[:, [1, 4]] = -1e9
    loss, amin, _ = oracle.prune_enumerate(logits, Y, 2, 5)
    subsets = oracle.kept_subsets(6, 5)
    first, second = subsets.index((0, 1, 2, 3, 5)), subsets.index((0, 2, 3, 4, 5))
    assert first < second and loss[first] == 0.0 and loss[second] == 0.0
    assert np.all(np.delete(loss, [first, second]) > 0.0)
    assert amin == first
    # expert outputs that are all zero: every loss is exactly 0 and the argmin is subset 0
    loss0, amin0, _ = oracle.prune_enumerate(logits, np.zeros_like(Y), 2, 3)
    assert not loss0.any() and amin0 == 0
    gram, gram_amin, _ = oracle.prune_enumerate_gram_form(logits, Y, 2, 5)
    assert gram_amin == first and gram[first] == 0.0 and gram[second] == 0.0


def test_r_smaller_than_k_uses_all_kept():
    logits, Y = enumeration_case(10, T=12, E=4, H=3)
    loss, _, _ = oracle.prune_enumerate(logits, Y, k=3, r=1)
    full = oracle.layer_output(logits, Y, 3)
    for e in range(4):
        assert loss[e] == pytest.approx(float(np.sum((Y[e] - full) ** 2)), rel=1e-12)


@pytest.mark.parametrize("E,k,r", [(3, 2, 2), (4, 2, 2), (5, 2, 3), (5, 3, 4), (4, 1, 2), (5, 4, 2)])
def test_against_pure_python_brute_force(E, k, r):
    g = rng(100 + 10 * E + r)
    T, H = 6, 3
    logits = g.standard_normal((T, E))
    logits[2, 0] = logits[2, E - 1]            # an exact tie inside one token
    Y = g.standard_normal((E, T, H))
    loss, amin, masks = oracle.prune_enumerate(logits, Y, k, r)
    bf, kept_sets = oracle.brute_force_enumerate(logits.tolist(), Y.tolist(), k, r)
    np.testing.assert_allclose(loss, bf, rtol=1e-11, atol=1e-14)
    assert kept_sets == oracle.kept_subsets(E, r)
    assert [oracle.subset_mask(c) for c in kept_sets] == masks.tolist()
    assert amin == min(range(len(bf)), key=lambda i: (loss[i], i))


# ---------------------------------------------------------------- Sec. 3.3 / A.2
def skip_case(seed, T=60, E=5, H=6, F=8):
    return random_layer(seed, T=T, E=E, H=H, F=F)


def test_skip_beta_zero_is_eq2_and_beta_large_is_top1():
    x, Wg, W1, W3, W2 = skip_case(11)
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    out0, skip0, e0, e1 = oracle.forward_skip(x, Wg, W1, W3, W2, beta=0.0)
    assert not skip0.any()
    np.testing.assert_allclose(out0, oracle.layer_output(logits, Y, 2), rtol=1e-11, atol=1e-13)
    out1, skip1, e0b, _ = oracle.forward_skip(x, Wg, W1, W3, W2, beta=1.5)
    assert skip1.all()
    t = np.arange(x.shape[0])
    np.testing.assert_allclose(out1, Y[e0b, t], rtol=1e-11, atol=1e-13)
    assert np.array_equal(e0, np.argmax(logits, 1))
    assert np.all(logits[t, e0] >= logits[t, e1])


def test_skip_error_closed_form_and_bound():
    # App. A.2 with k = 2, i = 1: z_hat - z = w~_e1 (f_e0 - f_e1), so the error norm is
    # w~_e1 ||f_e0 - f_e1|| exactly, and <= (w_e1 / (w_e0 + w_e1)) D for any D >= the distance.
    x, Wg, W1, W3, W2 = skip_case(12)
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    beta = 0.6
    out_s, skip, e0, e1 = oracle.forward_skip(x, Wg, W1, W3, W2, beta)
    out_f, _, _, _ = oracle.forward_skip(x, Wg, W1, W3, W2, 0.0)
    assert 0 < skip.sum() < len(skip)
    t = np.arange(x.shape[0])
    w = np.exp(logits) / np.exp(logits).sum(1, keepdims=True)      # full softmax, as in the paper
    w0, w1 = w[t, e0], w[t, e1]
    assert np.array_equal(skip, w1 < beta * w0)                      # the rule as printed (no near-ties here)
    dist = np.linalg.norm(Y[e0, t] - Y[e1, t], axis=1)
    err = np.linalg.norm(out_s - out_f, axis=1)
    np.testing.assert_allclose(err[skip], (w1 / (w0 + w1) * dist)[skip], rtol=1e-10)
    assert np.all(err[~skip] == 0.0)
    D = dist.max()
    assert np.all(err <= w1 / (w0 + w1) * D * (1 + 1e-12))


def test_skip_set_monotone_in_beta_and_median_halves():
    g = rng(13)
    logits = g.standard_normal((1000, 8)).astype(np.float32)
    prev = None
    for beta in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.0, 1.1):
        _, _, skip, delta = oracle.skip_decision(logits, beta)
        assert np.all(delta <= 0)
        if prev is not None:
            assert np.all(skip | ~prev)          # once skipped, skipped for any larger beta
        prev = skip
    assert prev.all()
    beta = oracle.median_skip_ratio(logits)
    _, _, skip, _ = oracle.skip_decision(logits, beta)
    assert abs(skip.mean() - 0.5) <= 1.0 / len(logits) + 1e-12
    # median convention: mean of the two middle order statistics
    l = np.asarray(logits, dtype=np.float64)
    srt = np.sort(l, axis=1)
    rho = np.sort(np.exp(srt[:, -2] - srt[:, -1]))
    assert beta == pytest.approx(0.5 * (rho[499] + rho[500]), rel=1e-15)


def test_skip_uses_given_logits():
    x, Wg, W1, W3, W2 = skip_case(14, T=20)
    forced = np.zeros((20, 5), dtype=np.float32)
    forced[:, 3] = 2.0
    forced[:, 1] = 1.0
    out, skip, e0, e1 = oracle.forward_skip(x, Wg, W1, W3, W2, beta=0.5, logits=forced)
    assert np.all(e0 == 3) and np.all(e1 == 1)
    assert skip.all()                      # exp(-1) = 0.37 < 0.5
    np.testing.assert_allclose(out, oracle.expert_ffn(x, W1[3], W3[3], W2[3]), rtol=1e-12)


def test_pruned_skip_forward_reduces_to_known_cases():
    # kept = everything is the unpruned forward; with beta = 0 the pruned forward is F'(x, C) of
    # Sec. 3.2 (computed by the enumeration code path), so its distance to the full layer is Eq. 3.
    x, Wg, W1, W3, W2 = skip_case(15, T=40, E=6)
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    a = oracle.forward_skip(x, Wg, W1, W3, W2, 0.55)
    b = oracle.forward_skip(x, Wg, W1, W3, W2, 0.55, kept=range(6))
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    kept = (0, 2, 3, 5)
    out, skip, e0, e1 = oracle.forward_skip(x, Wg, W1, W3, W2, 0.0, kept=kept)
    assert not skip.any() and set(e0) | set(e1) <= set(kept)
    np.testing.assert_allclose(out, oracle.pruned_layer_output(logits, Y, kept, 2), rtol=1e-11, atol=1e-13)
    loss, _, _ = oracle.prune_enumerate(logits, Y, 2, 4)
    idx = oracle.kept_subsets(6, 4).index(kept)
    full, _, _, _ = oracle.forward_skip(x, Wg, W1, W3, W2, 0.0)
    assert float(np.sum((out - full) ** 2)) == pytest.approx(loss[idx], rel=1e-10)
    # ties and order: the two best KEPT experts, lower index first on equal logits
    forced = np.tile(np.array([[3.0, 1.0, 3.0, 2.0, 2.0, 0.0]], dtype=np.float32), (40, 1))
    _, _, e0, e1 = oracle.forward_skip(x, Wg, W1, W3, W2, 0.0, logits=forced, kept=(1, 3, 4, 5))
    assert np.all(e0 == 3) and np.all(e1 == 4)
    with pytest.raises(ValueError):
        oracle.skip_decision(forced, 0.5, kept=(2,))


# ---- generalised top-k skipping (theory appendix) -------------------------------------------

def test_topk_skip_reduces_to_known_cases():
    x, Wg, W1, W3, W2 = skip_case(21, T=60, E=6)
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    # beta = 0: nothing is skipped, the output is Eq. 2 with k experts
    for k in (1, 2, 3, 4):
        out, i_star, experts = oracle.forward_skip_topk(x, Wg, W1, W3, W2, k, 0.0)
        assert np.all(i_star == k)
        np.testing.assert_allclose(out, oracle.layer_output(logits, Y, k), rtol=1e-11, atol=1e-13)
        assert np.array_equal(experts, oracle.routing_order(logits)[:, :k])
    # beta >= 1: sum_{m>1} w_m <= sum_m w_m always, so only the best expert stays
    out, i_star, experts = oracle.forward_skip_topk(x, Wg, W1, W3, W2, 4, 1.0)
    assert np.all(i_star == 1)
    t = np.arange(60)
    np.testing.assert_allclose(out, Y[experts[:, 0], t], rtol=1e-11, atol=1e-13)
    # k = 2: w_2 <= b (w_1 + w_2)  <=>  w_2 <= b / (1 - b) w_1, the rule of Sec. 3.3 with
    # beta = b / (1 - b) (the appendix's "abuse of notation"); compare with the top-2 code path
    b = 0.3
    out_g, i_star, _ = oracle.forward_skip_topk(x, Wg, W1, W3, W2, 2, b)
    out_2, skip, _, _ = oracle.forward_skip(x, Wg, W1, W3, W2, b / (1 - b))
    assert 0 < skip.sum() < 60
    assert np.array_equal(i_star == 1, skip)
    np.testing.assert_allclose(out_g, out_2, rtol=1e-11, atol=1e-13)


def test_topk_skip_rule_by_hand_and_monotone():
    # weights proportional to 8 : 4 : 2 : 1 (logits ln 8, ln 4, ln 2, 0): tails 7/15, 3/15, 1/15, 0
    logits = np.log(np.array([[4.0, 1.0, 8.0, 2.0, 1e-3]], dtype=np.float64)).astype(np.float32)
    want = {0.0: 4, 0.05: 4, 0.07: 3, 0.19: 3, 0.21: 2, 0.45: 2, 0.47: 1, 1.0: 1}
    for beta, i_want in want.items():
        experts, i_star, w = oracle.skip_topk_decision(logits, 4, beta)
        assert list(experts[0]) == [2, 0, 3, 1]
        assert i_star[0] == i_want, beta
    g = rng(22)
    lg = g.standard_normal((500, 8)).astype(np.float32)
    prev = None
    for beta in (0.0, 0.02, 0.1, 0.2, 0.4, 0.8, 1.0):
        _, i_star, _ = oracle.skip_topk_decision(lg, 4, beta)
        assert np.all((1 <= i_star) & (i_star <= 4))
        if prev is not None:
            assert np.all(i_star <= prev)            # a larger budget never keeps more experts
        prev = i_star
    # kept set: experts outside it never appear
    experts, _, _ = oracle.skip_topk_decision(lg, 3, 0.1, kept=(0, 2, 5, 7))
    assert set(np.unique(experts)) <= {0, 2, 5, 7}


def test_topk_skip_error_bound():
    # Theory appendix: ||z_hat - z|| <= (sum_{m>i} w_m / sum_{m<=k} w_m) D whenever D bounds every
    # pairwise distance ||f_m - f_n|| of the token's top-k expert outputs; and the chosen i*
    # therefore keeps the error below beta * D.
    x, Wg, W1, W3, W2 = skip_case(23, T=80, E=8)
    logits, Y = oracle.expert_outputs(x, Wg, W1, W3, W2)
    k, beta = 4, 0.15
    out_s, i_star, experts = oracle.forward_skip_topk(x, Wg, W1, W3, W2, k, beta)
    full = oracle.layer_output(logits, Y, k)
    assert len(np.unique(i_star)) > 1
    for t in range(80):
        f = Y[experts[t], t]                                   # [k, H]
        D = max(np.linalg.norm(f[m] - f[n]) for m in range(k) for n in range(m))
        w = np.exp(logits[t, experts[t]])
        frac = w[i_star[t]:].sum() / w.sum()
        err = np.linalg.norm(out_s[t] - full[t])
        assert err <= frac * D * (1 + 1e-9) + 1e-12     # rounding of two summation orders when nothing is skipped
        assert frac <= beta + 1e-12
        if i_star[t] > 1:                                      # i* is minimal
            assert w[i_star[t] - 1:].sum() / w.sum() > beta


def test_median_skip_ratio_with_kept_set():
    g = rng(24)
    lg = g.standard_normal((301, 8)).astype(np.float32)
    kept = (1, 2, 4, 7)
    beta = oracle.median_skip_ratio(lg, kept=kept)
    sub = np.sort(lg[:, list(kept)].astype(np.float64), axis=1)
    rho = np.sort(np.exp(sub[:, -2] - sub[:, -1]))
    assert beta == pytest.approx(rho[150], rel=1e-15)          # odd count: the middle one
    assert oracle.median_skip_ratio(lg, kept=range(8)) == oracle.median_skip_ratio(lg)


# ---- selection statistics and the frequency baseline ------------------------------------------

def test_selection_stats_hand_example_and_invariants():
    # three tokens, four experts, k = 2: selections {2,0}, {2,3}, {1,0} (second token ties 3 with 1? no: 3 wins by value)
    logits = np.array([[2.0, 0.0, 3.0, 1.0],
                       [0.0, 1.0, 5.0, 4.0],
                       [3.0, 7.0, 0.0, 3.0]], dtype=np.float32)    # last row: experts 0 and 3 tie, lower index wins
    count, co = oracle.expert_selection_stats(logits, 2)
    assert count.tolist() == [2, 1, 2, 1]
    want = np.zeros((4, 4), dtype=np.int64)
    for pair in ((2, 0), (2, 3), (1, 0)):
        for i in pair:
            for j in pair:
                want[i, j] += 1
    assert np.array_equal(co, want)
    g = rng(31)
    lg = g.standard_normal((400, 8)).astype(np.float32)
    for k in (1, 2, 4, 8):
        count, co = oracle.expert_selection_stats(lg, k)
        assert count.sum() == 400 * k
        assert np.array_equal(np.diag(co), count)
        assert np.array_equal(co, co.T)
        assert np.array_equal(co.sum(axis=1), k * count)
        if k == 1:
            assert np.array_equal(count, np.bincount(np.argmax(lg, axis=1), minlength=8))
        if k == 8:
            assert np.all(co == 400)
    # k = 2 co-selection against the top-2 pairs the skipping code path reports
    e0, e1, _, _ = oracle.skip_decision(lg, 0.0)
    _, co = oracle.expert_selection_stats(lg, 2)
    pairs = np.zeros((8, 8), dtype=np.int64)
    np.add.at(pairs, (e0, e1), 1)
    off = co - np.diag(np.diag(co))
    assert np.array_equal(off, pairs + pairs.T)


def test_frequency_baseline_keeps_most_selected():
    assert oracle.frequency_kept(np.array([5, 9, 1, 7]), 2) == (1, 3)
    assert oracle.frequency_kept(np.array([5, 9, 1, 7]), 3) == (0, 1, 3)
    assert oracle.frequency_kept(np.array([4, 4, 4, 4]), 2) == (0, 1)          # ties: lower index kept
    assert oracle.frequency_kept(np.array([3, 8, 3, 8, 3]), 3) == (0, 1, 3)
    assert oracle.frequency_kept(np.array([1, 2, 3]), 3) == (0, 1, 2)
