"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Tolerances (from the benchmark spec): subset indices, masks, argmin, top-2 ids and
skip masks bit-exact; losses within 1e-3 relative; logits within 1e-3 * max|logits|
absolute; expert outputs / layer outputs within 2e-2 relative (per-row L2, and max-abs
against the largest reference magnitude).
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2402_14800_amd as pkg
from paper_2402_14800_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LOSS_RTOL = 1e-3
OUT_RTOL = 2e-2


def check_outputs(got: np.ndarray, ref: np.ndarray, what: str):
    """Rows along the last axis: relative L2 error per row and max-abs error vs max|ref|."""
    err = np.linalg.norm(got - ref, axis=-1)
    nrm = np.linalg.norm(ref, axis=-1)
    floor = 1e-6 * max(float(nrm.max()), 1e-30)       # rows that are (nearly) zero in the reference
    rel = err / np.maximum(nrm, floor)
    assert rel.max() <= OUT_RTOL, f"{what}: worst row relative L2 error {rel.max():.3e}"
    assert np.abs(got - ref).max() <= OUT_RTOL * np.abs(ref).max(), f"{what}: max-abs error"


def check_losses(got: np.ndarray, ref: np.ndarray):
    assert got.shape == ref.shape
    bad = np.abs(got - ref) > LOSS_RTOL * np.abs(ref)
    assert not bad.any(), f"loss mismatch at {np.nonzero(bad)[0][:5]}: {got[bad][:5]} vs {ref[bad][:5]}"


def check_argmin(amin_gpu: int, loss_ref: np.ndarray, loss_gpu: np.ndarray):
    """The GPU argmin must be the oracle's, or a subset whose oracle loss ties the minimum within
    the loss tolerance; and it must be the lowest index attaining the GPU's own minimum."""
    amin_ref = int(np.argmin(loss_ref))
    assert amin_gpu == int(np.argmin(loss_gpu))
    if amin_gpu != amin_ref:
        assert abs(loss_ref[amin_gpu] - loss_ref[amin_ref]) <= LOSS_RTOL * abs(loss_ref[amin_ref])


def run_enumerate(logits_t, Y_t, k, r):
    loss, amin, amask, unaff = pkg.prune_enumerate(logits_t, Y_t, k, r)
    torch.cuda.synchronize()
    return (loss.cpu().numpy().astype(np.float64), int(amin.item()),
            int(amask.item()) & 0xFFFFFFFF, int(unaff.item()))


def tie_free(logits: np.ndarray) -> bool:
    s = np.sort(logits, axis=1)
    return bool(np.all(s[:, 1:] != s[:, :-1]))


# ------------------------------------------------------------------ prune_enumerate
ENUM_CASES = [
    # E, k, r, T, H, dtype
    (4, 2, 2, 512, 64, "f32"),
    (4, 2, 2, 512, 64, "bf16"),
    (4, 2, 4, 100, 64, "bf16"),       # r = E
    (4, 3, 2, 77, 128, "bf16"),       # r < k
    (5, 1, 3, 301, 64, "bf16"),       # k = 1, odd E
    (8, 2, 6, 1000, 256, "bf16"),     # ragged token count (token pairs, scoring tiles)
    (8, 2, 4, 1001, 192, "bf16"),     # odd T: last Gram tile holds one token
    (8, 2, 7, 333, 64, "f32"),
    (8, 2, 1, 129, 64, "bf16"),
    (8, 8, 8, 64, 64, "bf16"),        # k = r = E
    (16, 4, 12, 300, 128, "bf16"),
    (16, 4, 8, 130, 64, "bf16"),      # 12870 subsets
    (12, 3, 6, 90, 64, "bf16"),
    (20, 2, 18, 70, 64, "bf16"),      # E > 16: 32-row Gram tiles
    (6, 2, 4, 1, 64, "bf16"),         # a single token
    (16, 4, 4, 100, 64, "bf16"),      # every one of 16 rank positions can be selected (n_act = 16)
    (16, 2, 5, 90, 64, "bf16"),       # n_act = 13: the 16-position scorer with unused positions
    (24, 2, 3, 60, 64, "bf16"),       # n_act = 23: the 32-position scorer, 32-row Gram tiles
    (32, 2, 31, 50, 128, "bf16"),     # the largest E
    (8, 2, 6, 200, 576, "bf16"),      # H = 512 + 64: a second, partly filled block of hidden units in the Gram pass
    (16, 4, 12, 77, 1088, "bf16"),    # the same with 16 rows per token
    # many subsets, few possible selections per token: scored through per-token selection tables
    (32, 2, 29, 40, 64, "bf16"),      # 4960 subsets, 5 active ranks, 8 nibbles of kept mask
    (20, 2, 17, 60, 64, "bf16"),      # 1140 subsets, 5 nibbles
    (12, 1, 6, 70, 64, "bf16"),       # top-1: 924 subsets, 7 selections per token
    (12, 3, 6, 300, 64, "f32"),       # 924 subsets, 84 selections, several token groups and a ragged last one
    (16, 4, 8, 517, 64, "bf16"),      # 12870 subsets over several token tiles, 17 subsets per lane
    (16, 3, 7, 39, 64, "bf16"),       # 11440 subsets, 8 per lane; the last token group holds 7 tokens
    (15, 2, 11, 2049, 64, "bf16"),    # 1365 subsets, tiles of 32 tokens, the last one a single token
]


@pytest.mark.parametrize("E,k,r,T,H,dtype", ENUM_CASES)
def test_prune_enumerate_matches_oracle(E, k, r, T, H, dtype):
    bias = 0.5 if E == 16 else 0.0
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, dtype, seed=1000 + 31 * E + r, bias_var=bias, device=DEV)
    loss, amin, amask, unaff = run_enumerate(logits_t, Y_t, k, r)
    logits, Y = wl.to_f64(logits_t), wl.to_f64(Y_t)
    ref, ref_amin, ref_masks = oracle.prune_enumerate(logits, Y, k, r)
    assert len(loss) == math.comb(E, r)
    check_losses(loss, ref)
    check_argmin(amin, ref, loss)
    assert amask == int(ref_masks[amin]) == pkg.subset_unrank(E, r, amin)
    if r == E:
        assert loss.tolist() == [0.0] and amin == 0
    assert tie_free(logits)
    assert unaff == (T * math.comb(E - k, r - k) if r >= k else 0)


@pytest.mark.parametrize("E,k,rs,T,H,dtype", [(8, 2, (6, 4, 8, 1), 1000, 128, "bf16"), (4, 2, (2, 3), 300, 36, "f32"),
                                              (16, 4, (12, 14), 500, 64, "bf16")])
def test_prune_enumerate_multi_equals_separate_calls(E, k, rs, T, H, dtype):
    """One Gram pass shared by several r: every part bit-identical to prune_enumerate for that r."""
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, dtype, seed=321, device=DEV)
    parts = pkg.prune_enumerate_multi(logits_t, Y_t, k, rs)
    torch.cuda.synchronize()
    for r, (loss, amin, amask, unaff) in zip(rs, parts):
        l1, a1, m1, u1 = pkg.prune_enumerate(logits_t, Y_t, k, r)
        torch.cuda.synchronize()
        assert torch.equal(loss.view(torch.int32), l1.view(torch.int32))
        assert torch.equal(amin, a1) and torch.equal(amask, m1) and torch.equal(unaff, u1)


def test_prune_enumerate_is_deterministic_and_handles_empty_batch():
    logits_t, Y_t = wl.make_enumeration_inputs(8, 4096, 256, "bf16", seed=5, device=DEV)
    a = pkg.prune_enumerate(logits_t, Y_t, 2, 4)
    b = pkg.prune_enumerate(logits_t, Y_t, 2, 4)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[3], b[3])
    loss, amin, amask, unaff = pkg.prune_enumerate(logits_t[:0].contiguous(), Y_t[:, :0].contiguous(), 2, 6)
    torch.cuda.synchronize()
    assert loss.tolist() == [0.0] * 28 and amin.item() == 0 and amask.item() == 0b111111 and unaff.item() == 0


def test_prune_enumerate_ties_and_planted_argmin():
    E, T, H = 6, 200, 64
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, "bf16", seed=9, device=DEV)
    logits_t[:, [1, 4]] = -1e9                 # never routed to: dropping exactly these costs nothing
    logits_t[::7, 2] = logits_t[::7, 0]        # exact ties between experts 0 and 2
    loss, amin, amask, _ = run_enumerate(logits_t, Y_t, 2, 4)
    ref, ref_amin, masks = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), 2, 4)
    check_losses(loss, ref)
    assert amin == ref_amin == oracle.kept_subsets(E, 4).index((0, 2, 3, 5)) and loss[amin] == 0.0
    assert amask == 0b101101
    # Subsets whose survivors all sit at -1e9 still need finite Eq. 1 weights.
    loss2, _, _, _ = run_enumerate(logits_t, Y_t, 2, 2)
    ref2, _, _ = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), 2, 2)
    assert np.all(np.isfinite(loss2))
    check_losses(loss2, ref2)


def test_prune_enumerate_tables_with_ties_and_logits_far_below_the_maximum():
    """The table scorer (924 subsets, 28 selections per token) on logits with exact ties and with six experts at
    -1e9: the subset that keeps exactly those six has every survivor far below the token's maximum and needs Eq. 1
    redone relative to the largest selected logit; the subset that keeps the other six loses nothing."""
    E, T, H = 12, 150, 64
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, "bf16", seed=19, device=DEV)
    low = [1, 4, 7, 9, 10, 11]
    logits_t[:, low] = -1e9
    logits_t[::5, 2] = logits_t[::5, 0]        # exact ties between experts 0 and 2
    loss, amin, amask, _ = run_enumerate(logits_t, Y_t, 2, 6)
    ref, ref_amin, masks = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), 2, 6)
    assert len(loss) == 924 and np.all(np.isfinite(loss))
    check_losses(loss, ref)
    keep_high = oracle.kept_subsets(E, 6).index((0, 2, 3, 5, 6, 8))
    assert amin == ref_amin == keep_high and loss[amin] == 0.0
    assert loss[oracle.kept_subsets(E, 6).index(tuple(low))] > 0.0


DIRECT_CASES = [
    # E, k, r, T, H, dtype -- Eq. 3 as written (no Gram matrices): at most 128 subsets, k <= 4
    (4, 2, 2, 512, 64, "f32"),
    (4, 2, 4, 100, 64, "bf16"),       # r = E: nothing changes, every pair counted
    (4, 3, 2, 77, 128, "bf16"),       # r < k
    (5, 1, 3, 301, 64, "bf16"),       # top-1
    (8, 2, 6, 1000, 256, "bf16"),     # more tokens than workgroups: two tokens per workgroup, ragged
    (8, 2, 4, 1001, 192, "bf16"),     # 70 subsets; 24 chunks of hidden units for 256 threads
    (8, 2, 7, 333, 100, "f32"),       # H = 100: 25 chunks of 4
    (8, 4, 5, 130, 4096, "bf16"),     # top-4 (d has up to 8 entries), 64 KB of rows per token, two chunks per thread
    (9, 3, 7, 50, 320, "bf16"),       # odd E, 40 chunks of hidden units
    (6, 2, 4, 1, 64, "bf16"),         # a single token
    (16, 4, 15, 90, 2048, "bf16"),    # 16 experts
    (32, 2, 31, 40, 128, "f32"),      # 32 experts
]


@pytest.mark.parametrize("E,k,r,T,H,dtype", DIRECT_CASES)
def test_direct_enumeration_matches_oracle_and_gram_path(E, k, r, T, H, dtype):
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, dtype, seed=2000 + 31 * E + r, device=DEV)
    loss_t, amin_t, amask_t, unaff_t = pkg.prune_enumerate_direct(logits_t, Y_t, k, r)
    torch.cuda.synchronize()
    loss, amin, amask = loss_t.cpu().numpy().astype(np.float64), int(amin_t.item()), int(amask_t.item()) & 0xFFFFFFFF
    logits, Y = wl.to_f64(logits_t), wl.to_f64(Y_t)
    ref, _, ref_masks = oracle.prune_enumerate(logits, Y, k, r)
    check_losses(loss, ref)
    check_argmin(amin, ref, loss)
    assert amask == int(ref_masks[amin])
    assert tie_free(logits)
    assert int(unaff_t.item()) == (T * math.comb(E - k, r - k) if r >= k else 0)
    if r == E:
        assert loss.tolist() == [0.0]
    # the Gram path on the same inputs: different arithmetic, the same numbers to fp32 rounding
    gram, gram_amin, _, gram_unaff = run_enumerate(logits_t, Y_t, k, r)
    np.testing.assert_allclose(loss, gram, rtol=2e-4, atol=0.0)
    assert gram_unaff == int(unaff_t.item())
    # reproducible bit for bit
    again = pkg.prune_enumerate_direct(logits_t, Y_t, k, r)
    torch.cuda.synchronize()
    assert torch.equal(again[0], loss_t) and torch.equal(again[1], amin_t)


def test_direct_enumeration_limits_empty_batch_and_never_routed_experts():
    logits_t, Y_t = wl.make_enumeration_inputs(16, 64, 64, "bf16", seed=77, device=DEV)
    with pytest.raises(pkg.MoepError, match="subsets"):
        pkg.prune_enumerate_direct(logits_t, Y_t, 4, 8)            # 12870 subsets
    with pytest.raises(pkg.MoepError, match="k=5"):
        pkg.prune_enumerate_direct(logits_t, Y_t, 5, 15)
    big_t = torch.zeros((8, 4, 16384), dtype=torch.bfloat16, device=DEV)      # 256 KB of rows per token
    with pytest.raises(pkg.MoepError, match="LDS"):
        pkg.prune_enumerate_direct(torch.zeros((4, 8), device=DEV), big_t, 2, 6)
    logits_t, Y_t = wl.make_enumeration_inputs(8, 50, 72, "f32", seed=78, device=DEV)
    with pytest.raises(pkg.MoepError):
        pkg.prune_enumerate_direct(logits_t, Y_t[:, :, :70].contiguous(), 2, 6)   # H = 70 is no multiple of 4
    loss, amin, amask, unaff = pkg.prune_enumerate_direct(logits_t[:0].contiguous(), Y_t[:, :0].contiguous(), 2, 6)
    torch.cuda.synchronize()
    assert loss.tolist() == [0.0] * 28 and amin.item() == 0 and amask.item() == 0b111111 and unaff.item() == 0
    # experts 1 and 4 never routed to (Eq. 1 on logits of -1e9): the subset without them costs exactly nothing
    E, T, H = 6, 200, 64
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, "bf16", seed=9, device=DEV)
    logits_t[:, [1, 4]] = -1e9
    loss, amin, amask, _ = pkg.prune_enumerate_direct(logits_t, Y_t, 2, 4)
    ref, ref_amin, _ = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), 2, 4)
    assert amin.item() == ref_amin and amask.item() == 0b101101 and loss[ref_amin].item() == 0.0
    check_losses(loss.cpu().numpy().astype(np.float64), ref)
    l2, _, _, _ = pkg.prune_enumerate_direct(logits_t, Y_t, 2, 2)   # both survivors at -1e9: weights (1/2, 1/2)
    ref2, _, _ = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), 2, 2)
    check_losses(l2.cpu().numpy().astype(np.float64), ref2)


def test_prune_enumerate_relabelling_and_scale():
    E, T, H = 8, 512, 128
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, "bf16", seed=11, device=DEV)
    loss, _, _, _ = run_enumerate(logits_t, Y_t, 2, 5)
    perm = torch.tensor(np.random.default_rng(3).permutation(E), device=DEV)
    loss_p, _, _, _ = run_enumerate(logits_t[:, perm].contiguous(), Y_t[perm].contiguous(), 2, 5)
    np.testing.assert_allclose(np.sort(loss_p), np.sort(loss), rtol=1e-4)
    loss_s, _, _, _ = run_enumerate(logits_t, (Y_t * 4).contiguous(), 2, 5)     # exact scaling in bf16
    np.testing.assert_allclose(loss_s, 16.0 * loss, rtol=1e-6)


# ------------------------------------------------------------------ moe_expert_outputs
def small_layer(dtype, E, k, H, F, T, index=7):
    cfg = wl.LayerConfig(f"t-{dtype}-{E}-{H}-{F}-{T}", index, dtype, E=E, k=k, H=H, F=F, T=T, rs=())
    return cfg, wl.make_layer(cfg, device="cpu")


def to_dev(layer):
    return {n: (v.to(DEV) if isinstance(v, torch.Tensor) else v) for n, v in layer.items()}


EXPERT_CASES = [
    ("f32", 4, 64, 128, 512),        # config 1
    ("f32", 3, 36, 52, 70),          # ragged everything (multiples of 4)
    ("bf16", 4, 64, 128, 512),
    ("bf16", 2, 128, 192, 300),      # ragged M tile, N tail in both GEMMs
    ("bf16", 3, 256, 320, 257),      # one row into a second M tile
    ("bf16", 2, 512, 1024, 1000),
    ("bf16", 1, 64, 64, 76837),      # more tiles than compute units, K shorter than the load-ahead distance
    ("bf16", 2, 192, 448, 66000),    # several tiles per workgroup in both GEMMs, ragged last tile
    ("bf16", 1, 128, 320, 66000),    # several tiles per workgroup with K = 4 and 10 slices (the load-ahead distance and twice the ring)
    ("bf16", 20, 64, 64, 300),       # more than 16 experts: the router's second MFMA, batched launches over 20 experts
    ("bf16", 32, 128, 64, 77),       # the largest E
]


@pytest.mark.parametrize("dtype,E,H,F,T", EXPERT_CASES)
def test_moe_expert_outputs_matches_oracle(dtype, E, H, F, T):
    cfg, layer = small_layer(dtype, E, 2, H, F, T)
    d = to_dev(layer)
    logits_t, Y_t = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    ref_logits, ref_Y = oracle.expert_outputs(*(wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")))
    got_logits = logits_t.cpu().numpy().astype(np.float64)
    assert np.abs(got_logits - ref_logits).max() <= 1e-3 * np.abs(ref_logits).max()
    check_outputs(wl.to_f64(Y_t), ref_Y, "Y")
    # and again: bitwise reproducible
    logits2, Y2 = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    assert torch.equal(logits2, logits_t) and torch.equal(Y2.view(torch.int16 if dtype == "bf16" else torch.int32),
                                                         Y_t.view(torch.int16 if dtype == "bf16" else torch.int32))


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        E = int(rng.integers(1, 4))
        H = 64 * int(rng.integers(1, 9))
        F = 64 * int(rng.integers(1, 13))
        T = int(rng.choice([1, 15, 17, 255, 257, 511, 1025, int(rng.integers(1, 2500))]))
        shapes.append((E, H, F, T))
    return shapes


@pytest.mark.parametrize("E,H,F,T", _random_shapes(8, 20240214))
def test_moe_expert_outputs_random_shapes(E, H, F, T):
    """Seeded random layer shapes (every multiple of 64 up to 512 x 768, ragged token counts) against the oracle."""
    cfg, layer = small_layer("bf16", E, min(2, E), H, F, T, index=31)
    d = to_dev(layer)
    logits_t, Y_t = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    ref_logits, ref_Y = oracle.expert_outputs(*(wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")))
    assert np.abs(logits_t.cpu().numpy().astype(np.float64) - ref_logits).max() <= 1e-3 * np.abs(ref_logits).max()
    check_outputs(wl.to_f64(Y_t), ref_Y, "Y")


def test_expert_pass_in_batches_of_experts_and_on_prepacked_weights():
    """A layer whose intermediate activations exceed what one launch may hold (12 GiB): the 8 experts go through
    the projections in batches of 3, 3 and 2.  One token of every M tile against the oracle, and the same call on
    weights packed once gives the same bits."""
    E, H, F, T = 8, 64, 14336, 131072 + 300
    cfg, layer = small_layer("bf16", E, 2, H, F, 1, index=23)
    cfg = cfg.with_tokens(T)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cfg.seed)
    d = to_dev(layer)
    d["x"] = torch.randn((T, H), generator=gen, device=DEV).to(torch.bfloat16)
    need = pkg.binding.moe_expert_outputs_workspace(T, E, H, F, 1)
    per_expert_h = -(-T // 256) * 256 * F * 2
    assert 3 * per_expert_h <= (12 << 30) < 4 * per_expert_h and need > 3 * per_expert_h
    logits_t, Y_t = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    layer_x = dict(layer, x=d["x"])
    sampled_expert_check(layer_x, logits_t, Y_t, torch.tensor(one_token_per_tile(T), device=DEV), weights_f64(layer))
    packed = pkg.moe_pack_weights(d["W1"], d["W3"], d["W2"])
    logits_p, Y_p = pkg.moe_expert_outputs_packed(d["x"], d["Wgate"], packed, F)
    torch.cuda.synchronize()
    assert torch.equal(logits_p, logits_t) and torch.equal(Y_p.view(torch.int16), Y_t.view(torch.int16))


def test_config1_end_to_end():
    cfg = wl.CONFIGS["C1"]
    layer = wl.make_layer(cfg, device="cpu")
    d = to_dev(layer)
    logits_t, Y_t = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    loss, amin, amask, unaff = run_enumerate(logits_t, Y_t, cfg.k, 2)
    ref, ref_amin, masks = oracle.prune_enumerate(wl.to_f64(logits_t), wl.to_f64(Y_t), cfg.k, 2)
    check_losses(loss, ref)
    check_argmin(amin, ref, loss)
    assert unaff == 512 * math.comb(2, 0)
    # the whole pipeline against the oracle's own expert outputs (fp32 storage: tight)
    l64, Y64 = oracle.expert_outputs(*(wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")))
    ref_full, _, _ = oracle.prune_enumerate(l64, Y64, cfg.k, 2)
    np.testing.assert_allclose(loss, ref_full, rtol=1e-3)


# ------------------------------------------------------------------ moe_forward_skip
SKIP_CASES = [
    ("f32", 4, 64, 128, 512, None),
    ("bf16", 4, 64, 128, 300, None),
    ("bf16", 8, 256, 512, 1000, None),
    ("bf16", 8, 128, 256, 700, 0.0),     # never skip: Eq. 2
    ("bf16", 8, 128, 256, 700, 1.5),     # always skip: top-1
    ("bf16", 5, 128, 192, 3, None),      # fewer tokens than experts: empty expert segments
    ("bf16", 4, 128, 320, 70000, None),  # grouped GEMMs with several tiles per workgroup and short K
    ("bf16", 3, 192, 448, 1839, None),   # odd sizes all round
    ("bf16", 16, 64, 704, 513, 0.3),
    ("bf16", 2, 448, 64, 257, None),
]


@pytest.mark.parametrize("dtype,E,H,F,T,beta", SKIP_CASES)
def test_moe_forward_skip_matches_oracle(dtype, E, H, F, T, beta):
    cfg, layer = small_layer(dtype, E, 2, H, F, T, index=9)
    d = to_dev(layer)
    logits_full, _ = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    median = beta is None
    if median:
        beta = oracle.median_skip_ratio(logits_full.cpu().numpy())
    beta = float(np.float32(beta))
    out_t, skip_t, logits_t, top2_t = pkg.moe_forward_skip(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"], beta)
    torch.cuda.synchronize()
    assert torch.equal(logits_t, logits_full)                     # same router, same bits
    args = [wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")]
    ref_out, ref_skip, e0, e1 = oracle.forward_skip(*args, beta, logits=logits_t.cpu().numpy())
    assert np.array_equal(skip_t.cpu().numpy().astype(bool), ref_skip)
    top2 = top2_t.cpu().numpy()
    assert np.array_equal(top2[:, 0], e0) and np.array_equal(top2[:, 1], e1)
    check_outputs(wl.to_f64(out_t), ref_out, "out")
    if beta == 0.0:
        assert not ref_skip.any()
    elif beta > 1.0:
        assert ref_skip.all()
    elif median and T >= 100:
        assert abs(ref_skip.mean() - 0.5) <= 1.0 / T + 1e-9


@pytest.mark.parametrize("dtype,E,H", [("bf16", 8, 256), ("bf16", 16, 128), ("bf16", 20, 64), ("f32", 4, 64)])
def test_router_logits_do_not_depend_on_the_batch(dtype, E, H):
    """A token's logits are the same bits whatever batch it is in and wherever it sits in it."""
    cfg, layer = small_layer(dtype, E, 2, H, 64, 1000, index=17)
    d = to_dev(layer)
    ws = [d[n] for n in ("Wgate", "W1", "W3", "W2")]
    full, _ = pkg.moe_expert_outputs(d["x"], *ws)
    for lo, hi in ((0, 333), (5, 905), (999, 1000), (37, 53)):
        part, _ = pkg.moe_expert_outputs(d["x"][lo:hi].contiguous(), *ws)
        torch.cuda.synchronize()
        assert torch.equal(part, full[lo:hi])


def test_skip_empty_batch_and_bad_k():
    cfg, layer = small_layer("bf16", 4, 2, 64, 128, 16, index=9)
    d = to_dev(layer)
    out, skip, logits, top2 = pkg.moe_forward_skip(d["x"][:0].contiguous(), d["Wgate"], d["W1"], d["W3"], d["W2"], 0.5)
    torch.cuda.synchronize()
    assert out.shape == (0, 64) and skip.numel() == 0
    with pytest.raises(pkg.MoepError) as ei:
        pkg.moe_forward_skip(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"], 0.5, k=3)
    assert ei.value.status == 2


# ================================================================== full-size configurations
# The launch shapes bench.py times.  The oracle cannot redo these sizes in seconds, so outputs are
# checked on sampled tokens (each expert output row is computable on its own) and the summed losses
# through a token prefix plus properties that hold at any size (additivity over token ranges, the
# count of unaffected pairs, reproducibility).

def sampled_expert_check(layer, logits_t, Y_t, tokens, W64):
    x64 = wl.to_f64(layer["x"][tokens])
    ref_logits, ref_Y = oracle.expert_outputs(x64, wl.to_f64(layer["Wgate"]), W64["W1"], W64["W3"], W64["W2"])
    got_logits = logits_t[tokens].cpu().numpy().astype(np.float64)
    assert np.abs(got_logits - ref_logits).max() <= 1e-3 * np.abs(ref_logits).max()
    check_outputs(wl.to_f64(Y_t[:, tokens]), ref_Y, "Y (sampled tokens)")


def weights_f64(layer):
    return {n: [wl.to_f64(layer[n][e]) for e in range(layer[n].shape[0])] for n in ("W1", "W3", "W2")}


def test_config2_full_size():
    cfg = wl.CONFIGS["C2"]
    layer = wl.make_layer(cfg, device=DEV)
    x, Wg, W1, W3, W2 = (layer[n] for n in ("x", "Wgate", "W1", "W3", "W2"))
    logits_t, Y_t = pkg.moe_expert_outputs(x, Wg, W1, W3, W2)
    torch.cuda.synchronize()
    tokens = torch.tensor(np.random.default_rng(2).choice(cfg.T, 256, replace=False), device=DEV).sort().values
    sampled_expert_check(layer, logits_t, Y_t, tokens, weights_f64(layer))
    for r in cfg.rs:
        loss, amin, amask, unaff = run_enumerate(logits_t, Y_t, cfg.k, r)
        ref, _, masks = oracle.prune_enumerate_streamed(logits_t, Y_t, cfg.k, r, chunk=4096, to_f64=wl.to_f64)
        check_losses(loss, ref)
        check_argmin(amin, ref, loss)
        assert amask == int(masks[amin])
        assert unaff == cfg.T * math.comb(cfg.E - cfg.k, r - cfg.k)


@pytest.fixture(scope="module")
def config3():
    cfg = wl.CONFIGS["C3"]
    layer = wl.make_layer(cfg, device=DEV)
    x, Wg, W1, W3, W2 = (layer[n] for n in ("x", "Wgate", "W1", "W3", "W2"))
    logits_t, Y_t = pkg.moe_expert_outputs(x, Wg, W1, W3, W2)
    torch.cuda.synchronize()
    yield cfg, layer, logits_t, Y_t, weights_f64(layer)
    del layer, logits_t, Y_t
    torch.cuda.empty_cache()


def one_token_per_tile(T, tile=256):
    """One token of every 256-row M tile of the expert GEMMs, the row inside the tile varying from tile to tile
    (first and last rows included), so that every (M tile, N tile) of both projections is compared with the oracle."""
    n_tiles = -(-T // tile)
    rows = (37 * np.arange(n_tiles) + 11) % tile
    rows[::7] = 0
    rows[3::7] = tile - 1
    tokens = np.minimum(tile * np.arange(n_tiles) + rows, T - 1)
    return np.unique(np.concatenate([tokens, [0, T - 1]]))


def test_config3_expert_outputs_one_row_per_tile(config3):
    cfg, layer, logits_t, Y_t, W64 = config3
    tokens = one_token_per_tile(cfg.T)
    assert len(np.unique(tokens // 256)) == cfg.T // 256 == 1024
    for part in np.array_split(tokens, 4):                   # fp64 intermediates of 256 tokens at a time
        sampled_expert_check(layer, logits_t, Y_t, torch.tensor(part, device=DEV), W64)


def enumeration_windows_check(logits_t, Y_t, k, r, windows, loss, unaff, gram_form_windows=()):
    """Cuts the tokens at the ends of `windows` (token ranges), enumerates every piece on its own and checks
    (a) the pieces inside `windows` against the oracle (Sec. 3.2, Eq. 3), and (b) that all pieces add up to
    the full call's losses and unaffected-pair count, which ties the oracle-checked windows to the full call.
    Pieces in `gram_form_windows` (longer ones) are checked against the SECOND oracle, the fp64 Gram form that a
    CPU test pins to the direct definition."""
    T = logits_t.shape[0]
    windows = list(windows) + list(gram_form_windows)
    cuts = sorted({0, T} | {a for a, _ in windows} | {b for _, b in windows})
    total = np.zeros_like(loss)
    total_unaff = 0
    for a, b in zip(cuts[:-1], cuts[1:]):
        lp, ap, _, up = run_enumerate(logits_t[a:b].contiguous(), Y_t[:, a:b].contiguous(), k, r)
        total += lp
        total_unaff += up
        if (a, b) in windows:
            enumerate_ref = oracle.prune_enumerate_gram_form if (a, b) in gram_form_windows else oracle.prune_enumerate
            ref, _, _ = enumerate_ref(wl.to_f64(logits_t[a:b]), wl.to_f64(Y_t[:, a:b]), k, r)
            check_losses(lp, ref)
            check_argmin(ap, ref, lp)
    np.testing.assert_allclose(total, loss, rtol=2e-5)
    assert total_unaff == unaff


def test_config3_enumeration(config3):
    cfg, layer, logits_t, Y_t, _ = config3
    T = cfg.T
    # head, an unaligned window in the middle, and the tail
    windows = [(0, 4096), (T // 2 + 1021, T // 2 + 1021 + 3003), (T - 4099, T)]
    for r in cfg.rs:
        loss, amin, amask, unaff = run_enumerate(logits_t, Y_t, cfg.k, r)
        assert unaff == T * math.comb(cfg.E - cfg.k, r - cfg.k)
        assert amin == int(np.argmin(loss)) and amask == pkg.subset_unrank(cfg.E, r, amin)
        enumeration_windows_check(logits_t, Y_t, cfg.k, r, windows, loss, unaff)
        # reproducible bit for bit
        loss2, amin2, _, _ = run_enumerate(logits_t, Y_t, cfg.k, r)
        assert np.array_equal(loss, loss2) and amin == amin2
        # Eq. 3 as written, over all 262144 tokens: the same losses from different arithmetic
        direct = pkg.prune_enumerate_direct(logits_t, Y_t, cfg.k, r)
        torch.cuda.synchronize()
        np.testing.assert_allclose(direct[0].cpu().numpy().astype(np.float64), loss, rtol=1e-4, atol=0.0)
        assert int(direct[1].item()) == amin and int(direct[3].item()) == unaff


def test_config5_skip_forward_sampled(config3):
    cfg, layer, _, _, W64 = config3
    Ts = wl.CONFIGS["C5"].T
    x = layer["x"][:Ts]
    Wg, W1, W3, W2 = (layer[n] for n in ("Wgate", "W1", "W3", "W2"))
    _, _, lg, _ = pkg.moe_forward_skip(x, Wg, W1, W3, W2, 0.0)
    torch.cuda.synchronize()
    beta = float(np.float32(oracle.median_skip_ratio(lg.cpu().numpy())))
    out_t, skip_t, logits_t, top2_t = pkg.moe_forward_skip(x, Wg, W1, W3, W2, beta)
    torch.cuda.synchronize()
    assert torch.equal(logits_t, lg)
    # decisions: every token, exactly
    e0, e1, ref_skip, _ = oracle.skip_decision(logits_t.cpu().numpy(), beta)
    assert np.array_equal(skip_t.cpu().numpy().astype(bool), ref_skip)
    top2 = top2_t.cpu().numpy()
    assert np.array_equal(top2[:, 0], e0) and np.array_equal(top2[:, 1], e1)
    assert abs(ref_skip.mean() - 0.5) <= 1.0 / Ts + 1e-9
    # outputs: sampled tokens through the fp64 experts
    tokens = np.unique(np.concatenate([[0, Ts - 1], np.random.default_rng(5).choice(Ts, 46, replace=False)]))
    tt = torch.tensor(tokens, device=DEV)
    ref_out, rs, _, _ = oracle.forward_skip(wl.to_f64(x[tt]), wl.to_f64(Wg), W64["W1"], W64["W3"], W64["W2"], beta,
                                            logits=logits_t[tt].cpu().numpy())
    assert np.array_equal(rs, ref_skip[tokens])
    check_outputs(wl.to_f64(out_t[tt]), ref_out, "skip out (sampled tokens)")
    # never skipping reproduces Eq. 2 on the dense expert outputs
    out0, skip0, _, _ = pkg.moe_forward_skip(x, Wg, W1, W3, W2, 0.0)
    torch.cuda.synchronize()
    assert int(skip0.sum().item()) == 0


@pytest.fixture(scope="module")
def config4():
    cfg = wl.CONFIGS["C4"]
    layer = wl.make_layer(cfg, device=DEV)
    x, Wg, W1, W3, W2 = (layer[n] for n in ("x", "Wgate", "W1", "W3", "W2"))
    logits_t, Y_t = pkg.moe_expert_outputs(x, Wg, W1, W3, W2)
    torch.cuda.synchronize()
    yield cfg, layer, logits_t, Y_t
    del layer, logits_t, Y_t
    torch.cuda.empty_cache()


def test_config4_expert_outputs_one_row_per_tile(config4):
    """The expert pass at the stress configuration's shape (16 experts, H = 2048, F = 5632, 65536 tokens: 44 and 8
    N tiles, 64 and 176 K slices) against the oracle, one token from every M tile."""
    cfg, layer, logits_t, Y_t = config4
    tokens = one_token_per_tile(cfg.T)
    assert len(np.unique(tokens // 256)) == 256
    sampled_expert_check(layer, logits_t, Y_t, torch.tensor(tokens, device=DEV), weights_f64(layer))


# windows sized so that the CPU oracle needs about two minutes per r at most (a GPU run that prints nothing for three
# minutes is taken to be hung): head, unaligned middle and tail against the direct definition, and a longer unaligned
# one in the second half against the Gram-form oracle
@pytest.mark.parametrize("r,w_head,w_mid,w_tail,w_gram", [(12, 768, 517, 700, 8197), (8, 128, 67, 96, 2051)])
def test_config4_enumeration_stress(config4, r, w_head, w_mid, w_tail, w_gram):
    """Both r of the stress configuration on the GPU's own expert outputs, the per-expert logit bias added by the
    harness between the two calls as the configuration says."""
    cfg, layer, logits_t, Y_t = config4
    E, k, T = cfg.E, cfg.k, cfg.T
    logits_b = (logits_t + layer["bias"].to(DEV)).contiguous()
    load = torch.bincount(torch.topk(logits_b, k, dim=1).indices.flatten(), minlength=E).float()
    assert load.max() > 1.5 * load.min()                     # experts are unequally used
    assert tie_free(logits_b.cpu().numpy())
    loss, amin, amask, unaff = run_enumerate(logits_b, Y_t, k, r)
    assert len(loss) == math.comb(E, r)
    assert unaff == T * math.comb(E - k, r - k)
    assert amin == int(np.argmin(loss)) and amask == pkg.subset_unrank(E, r, amin)
    mid = T // 3 + 7
    windows = [(0, w_head), (mid, mid + w_mid), (T - w_tail, T)]
    enumeration_windows_check(logits_b, Y_t, k, r, windows, loss, unaff,
                              gram_form_windows=[(2 * T // 3 + 5, 2 * T // 3 + 5 + w_gram)])


# ------------------------------------------------------------------ pruned + skipping forward
@pytest.mark.parametrize("dtype,E,H,F,T,r", [("bf16", 8, 256, 512, 900, 6), ("f32", 6, 64, 128, 300, 3),
                                             ("bf16", 8, 128, 256, 500, 2)])
def test_pruned_skip_forward_matches_oracle_and_enumeration(dtype, E, H, F, T, r):
    cfg, layer = small_layer(dtype, E, 2, H, F, T, index=11)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    logits_t, Y_t = pkg.moe_expert_outputs(*ws)
    loss, amin, amask, _ = run_enumerate(logits_t, Y_t, 2, r)
    kept = [e for e in range(E) if (amask >> e) & 1]
    args = [wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")]
    for beta in (0.0, float(np.float32(0.5))):
        out_t, skip_t, lg, top2_t = pkg.moe_forward_pruned_skip(*ws, amask, beta)
        torch.cuda.synchronize()
        assert torch.equal(lg, logits_t)
        ref_out, ref_skip, e0, e1 = oracle.forward_skip(*args, beta, logits=lg.cpu().numpy(), kept=kept)
        assert np.array_equal(skip_t.cpu().numpy().astype(bool), ref_skip)
        top2 = top2_t.cpu().numpy()
        assert np.array_equal(top2[:, 0], e0) and np.array_equal(top2[:, 1], e1)
        assert set(np.unique(top2)) <= set(kept)
        check_outputs(wl.to_f64(out_t), ref_out, "pruned out")
    # beta = 0: the pruned forward is F'(x, C); its distance to the full forward is the Eq. 3 loss
    # the enumeration reported for that subset (different kernels: GEMMs on routed rows vs Gram).
    pruned, _, _, _ = pkg.moe_forward_pruned_skip(*ws, amask, 0.0)
    full, _, _, _ = pkg.moe_forward_skip(*ws, 0.0)
    torch.cuda.synchronize()
    dist = float(((pruned.double() - full.double()) ** 2).sum().item())
    assert dist == pytest.approx(loss[amin], rel=3e-2)
    allmask = (1 << E) - 1
    same, sk2, _, _ = pkg.moe_forward_pruned_skip(*ws, allmask, 0.5)
    ref2, sk1, _, _ = pkg.moe_forward_skip(*ws, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(same.view(torch.int16 if dtype == "bf16" else torch.int32),
                       ref2.view(torch.int16 if dtype == "bf16" else torch.int32)) and torch.equal(sk1, sk2)


@pytest.mark.parametrize("E,H,F,T,kept,beta", [(8, 256, 512, 900, 0b10110111, 0.5), (4, 128, 192, 300, 0b1111, 0.0),
                                               (8, 64, 64, 5, 0b11000011, 1.5)])
def test_forward_on_prepacked_weights_is_bit_identical(E, H, F, T, kept, beta):
    """moe_pack_weights once + moe_forward_pruned_skip_packed = moe_forward_pruned_skip, bit for bit, call after call."""
    cfg, layer = small_layer("bf16", E, 2, H, F, T, index=13)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    ref_out, ref_skip, ref_lg, ref_top2 = pkg.moe_forward_pruned_skip(*ws, kept, beta)
    packed = pkg.moe_pack_weights(d["W1"], d["W3"], d["W2"])
    for _ in range(2):
        out, skip, lg, top2 = pkg.moe_forward_pruned_skip_packed(d["x"], d["Wgate"], packed, F, beta, kept_mask=kept)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
        assert torch.equal(skip, ref_skip) and torch.equal(lg, ref_lg) and torch.equal(top2, ref_top2)
    with pytest.raises(pkg.MoepError):
        pkg.moe_pack_weights(d["W1"].float(), d["W3"].float(), d["W2"].float())


def test_overlapping_calls_on_two_streams_give_the_serial_results():
    """The bf16 GEMM kernels line their persistent workgroups up through counters that every launch on the GPU
    shares.  Two calls that overlap on different streams may make each other wait, for a bounded time; they must
    finish and must not change a bit of either result."""
    E, H, F, T = 2, 256, 2048, 24576         # 1536 gate/up tiles = 6 rounds of 256: the workgroups line up in between
    sets = []
    for index in (21, 22):
        _, layer = small_layer("bf16", E, 2, H, F, T, index=index)
        d = to_dev(layer)
        sets.append([d[n] for n in ("x", "Wgate", "W1", "W3", "W2")])
    serial = [pkg.moe_expert_outputs(*ws) for ws in sets]
    torch.cuda.synchronize()
    need = pkg.binding.moe_expert_outputs_workspace(T, E, H, F, 1)      # 1 = bf16
    spaces = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in sets]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for _ in range(3):
        got = []
        for ws, space, stream in zip(sets, spaces, streams):
            with torch.cuda.stream(stream):
                got.append(pkg.moe_expert_outputs(*ws, workspace=space))
        torch.cuda.synchronize()
        for (lg, Y), (lg0, Y0) in zip(got, serial):
            assert torch.equal(lg, lg0) and torch.equal(Y.view(torch.int16), Y0.view(torch.int16))


# ------------------------------------------------------------------ generalised top-k skipping, beta calibration
TOPK_CASES = [
    # dtype, E, H, F, T, k, beta, kept
    ("bf16", 8, 256, 512, 900, 4, 0.15, None),
    ("bf16", 16, 128, 256, 700, 4, 0.05, None),        # the E=16, k=4 shape of the stress configuration
    ("f32", 6, 64, 128, 300, 3, 0.2, (0, 2, 3, 5)),
    ("bf16", 8, 128, 256, 500, 2, 0.3, None),          # k = 2: equals the top-2 rule with beta / (1 - beta)
    ("bf16", 8, 128, 256, 400, 8, 0.1, None),          # every expert selected
    ("bf16", 8, 128, 256, 300, 1, 0.5, None),          # top-1: nothing to skip
    ("bf16", 8, 128, 256, 300, 4, 0.0, None),          # never skip: Eq. 2 with k = 4
    ("bf16", 8, 128, 256, 300, 4, 1.0, (1, 2, 4, 6, 7)),   # always down to the best kept expert
    ("bf16", 16, 128, 256, 400, 12, 0.02, None),       # wide top-k
]


@pytest.mark.parametrize("dtype,E,H,F,T,k,beta,kept", TOPK_CASES)
def test_moe_forward_skip_topk_matches_oracle(dtype, E, H, F, T, k, beta, kept):
    cfg, layer = small_layer(dtype, E, min(k, 2), H, F, T, index=12)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    mask = None if kept is None else sum(1 << e for e in kept)
    beta = float(np.float32(beta))
    out_t, n_used_t, logits_t, topk_t = pkg.moe_forward_skip_topk(*ws, k, beta, kept_mask=mask)
    torch.cuda.synchronize()
    logits_full, _ = pkg.moe_expert_outputs(*ws)
    torch.cuda.synchronize()
    assert torch.equal(logits_t, logits_full)
    args = [wl.to_f64(layer[n]) for n in ("x", "Wgate", "W1", "W3", "W2")]
    ref_out, i_star, experts = oracle.forward_skip_topk(*args, k, beta, logits=logits_t.cpu().numpy(), kept=kept)
    assert np.array_equal(topk_t.cpu().numpy(), experts)
    assert np.array_equal(n_used_t.cpu().numpy(), i_star)
    check_outputs(wl.to_f64(out_t), ref_out, "top-k skip out")
    if beta == 0.0:
        assert np.all(i_star == k)
    elif beta >= 1.0:
        assert np.all(i_star == 1)
    elif k > 2:
        assert len(np.unique(i_star)) > 1               # the case exercises more than one branch
    if k == 2 and kept is None:
        # same tokens skipped, same output bits as the top-2 entry point with the converted threshold
        # (a token sitting exactly on the threshold would differ: "<" there, "<=" here)
        out2, skip2, _, top2 = pkg.moe_forward_skip(*ws, float(np.float32(beta / (1 - beta))))
        torch.cuda.synchronize()
        assert torch.equal(top2, topk_t)
        agree = (skip2.cpu().numpy().astype(bool) == (i_star == 1))
        assert agree.mean() >= 1 - 2.0 / T
        check_outputs(wl.to_f64(out2)[agree], ref_out[agree], "top-2 entry point vs generalised rule")


def test_skip_topk_empty_batch_and_reuse_of_workspace():
    cfg, layer = small_layer("bf16", 8, 2, 128, 256, 64, index=12)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    out, n_used, _, _ = pkg.moe_forward_skip_topk(d["x"][:0].contiguous(), *ws[1:], 4, 0.1)
    torch.cuda.synchronize()
    assert out.shape == (0, 128) and n_used.numel() == 0
    a = pkg.moe_forward_skip_topk(*ws, 4, 0.1)
    b = pkg.moe_forward_skip_topk(*ws, 4, 0.1)
    torch.cuda.synchronize()
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("T,E,kept", [(1, 4, None), (2, 4, None), (1000, 8, None), (1001, 8, None),
                                      (70000, 8, None), (4097, 16, (0, 3, 5, 6, 9, 12)), (5000, 32, None)])
def test_skip_calibrate_beta_matches_oracle(T, E, kept):
    g = np.random.default_rng(1234 + T + E)
    logits = (g.standard_normal((T, E)) * 1.3).astype(np.float32)
    if T >= 1000:
        logits[5] = logits[7]                           # duplicated token: equal keys
        logits[9, :] = 0.25                              # all logits equal: ratio exactly 1
    mask = None if kept is None else sum(1 << e for e in kept)
    beta_t = pkg.skip_calibrate_beta(torch.from_numpy(logits).to(DEV), kept_mask=mask)
    torch.cuda.synchronize()
    beta = float(beta_t.item())
    ref = oracle.median_skip_ratio(logits, kept=kept)
    assert beta == pytest.approx(ref, rel=2e-6)          # fp32 differences, fp32 result
    if T >= 1000:
        _, _, skip, _ = oracle.skip_decision(logits, beta, kept=kept)
        assert abs(skip.mean() - 0.5) <= 2.0 / T


def test_calibrated_beta_feeds_the_skip_forward():
    cfg, layer = small_layer("bf16", 8, 2, 128, 256, 1024, index=13)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    logits_t, _ = pkg.moe_expert_outputs(*ws)
    beta = float(pkg.skip_calibrate_beta(logits_t).item())
    _, skip_t, _, _ = pkg.moe_forward_skip(*ws, beta)
    torch.cuda.synchronize()
    assert abs(float(skip_t.float().mean().item()) - 0.5) <= 2.0 / 1024


# ------------------------------------------------------------------ selection statistics, frequency baseline
@pytest.mark.parametrize("T,E,k,r", [(1000, 8, 2, 6), (70001, 8, 2, 4), (3000, 16, 4, 8), (500, 32, 8, 20),
                                     (300, 5, 5, 2), (257, 4, 1, 3), (0, 8, 2, 6)])
def test_expert_selection_stats_match_oracle(T, E, k, r):
    g = np.random.default_rng(77 + T + E)
    logits = (g.standard_normal((T, E)) + 0.3 * g.standard_normal((1, E))).astype(np.float32)
    if T >= 300:
        logits[3, :] = 1.0                               # all equal: the k lowest indices are selected
        logits[4, 1] = logits[4, 0]                      # a tie at the top
    count_t, co_t, fmask_t = pkg.expert_selection_stats(torch.from_numpy(logits).to(DEV), k, r)
    torch.cuda.synchronize()
    count, co = oracle.expert_selection_stats(logits, k)
    assert np.array_equal(count_t.cpu().numpy(), count)
    assert np.array_equal(co_t.cpu().numpy(), co)
    kept = oracle.frequency_kept(count, r)
    assert (int(fmask_t.item()) & 0xFFFFFFFF) == sum(1 << e for e in kept)


def test_frequency_baseline_is_scored_by_the_enumeration():
    # the baseline's kept set is one of the enumerated subsets: its Eq. 3 loss can be read off the
    # loss vector, and can be no smaller than the minimum the enumeration found
    E, r = 8, 6
    cfg, layer = small_layer("bf16", E, 2, 128, 256, 800, index=14)
    d = to_dev(layer)
    logits_t, Y_t = pkg.moe_expert_outputs(d["x"], d["Wgate"], d["W1"], d["W3"], d["W2"])
    loss, amin, amask, _ = run_enumerate(logits_t, Y_t, 2, r)
    _, _, fmask_t = pkg.expert_selection_stats(logits_t, 2, r)
    fmask = int(fmask_t.item()) & 0xFFFFFFFF
    idx = pkg.subset_rank(E, r, fmask)
    assert 0 <= idx < len(loss) and loss[idx] >= loss[amin]
    kept = [e for e in range(E) if (fmask >> e) & 1]
    l64 = logits_t.cpu().numpy().astype(np.float64)
    ref = oracle.pruned_layer_output(l64, wl.to_f64(Y_t), kept, 2) - oracle.layer_output(l64, wl.to_f64(Y_t), 2)
    assert loss[idx] == pytest.approx(float((ref ** 2).sum()), rel=LOSS_RTOL)


# ------------------------------------------------------------------ rank-limited expert pass
def densify(ranked, E, T):
    """Full [E,T,H] fp64 array from the ranked outputs, zeros where an expert was not run."""
    logits_t, experts_t, slot_t, Yr_t = ranked
    Yr = wl.to_f64(Yr_t)
    experts, slot = experts_t.cpu().numpy(), slot_t.cpu().numpy()
    Y = np.zeros((E, T, Yr.shape[1]))
    for j in range(experts.shape[1]):
        Y[experts[:, j], np.arange(T)] = Yr[slot[:, j]]
    return Y


@pytest.mark.parametrize("dtype,E,H,F,T,k,rs,n_rank", [
    ("bf16", 8, 256, 512, 1100, 2, (6, 4), 6),         # the benchmark's pair of r from one pass
    ("bf16", 8, 128, 256, 700, 2, (6,), 4),            # exactly n_act ranks
    ("bf16", 8, 128, 256, 300, 2, (7, 5, 3), 8),       # every expert: same work as the dense pass
    ("f32", 6, 64, 128, 400, 2, (4, 3), 5),
    ("bf16", 5, 128, 192, 3, 3, (4,), 4),              # fewer tokens than experts: empty segments
    ("bf16", 16, 128, 256, 600, 4, (14,), 6),          # 16 experts, top-4
    ("bf16", 16, 128, 256, 500, 4, (8, 12), 12),       # the stress configuration's E, k, r: 12 ranks reach every subset
])
def test_rank_limited_pass_matches_dense_pass_and_oracle(dtype, E, H, F, T, k, rs, n_rank):
    cfg, layer = small_layer(dtype, E, k, H, F, T, index=15)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    logits_d, Y_d = pkg.moe_expert_outputs(*ws)
    ranked = pkg.moe_expert_outputs_ranked(*ws, n_rank)
    torch.cuda.synchronize()
    logits_t, experts_t, slot_t, Yr_t = ranked
    assert torch.equal(logits_t, logits_d)
    lg = logits_t.cpu().numpy()
    experts, slot = experts_t.cpu().numpy(), slot_t.cpu().numpy()
    assert np.array_equal(experts, oracle.routing_order(lg)[:, :n_rank])
    # slots: a permutation of 0 .. T n_rank - 1, grouped by expert, ascending token inside an expert
    flat = slot.reshape(-1)
    assert np.array_equal(np.sort(flat), np.arange(T * n_rank))
    by_slot_expert = np.empty(T * n_rank, dtype=np.int64)
    by_slot_token = np.empty(T * n_rank, dtype=np.int64)
    by_slot_expert[flat] = experts.reshape(-1)
    by_slot_token[flat] = np.repeat(np.arange(T), n_rank)
    assert np.all(np.diff(by_slot_expert) >= 0)
    same = np.diff(by_slot_expert) == 0
    assert np.all(np.diff(by_slot_token)[same] > 0)
    # each stored row is the dense pass's row, bit for bit (same K loop, same epilogue)
    bits = torch.int16 if dtype == "bf16" else torch.int32
    tok = torch.arange(T, device=DEV)
    for j in range(n_rank):
        dense_rows = Y_d[experts_t[:, j].long(), tok]
        assert torch.equal(Yr_t[slot_t[:, j].long()].view(bits), dense_rows.view(bits))
    Yfull = densify(ranked, E, T)
    l64 = lg.astype(np.float64)
    for r in rs:
        loss_t, amin_t, amask_t, unaff_t = pkg.prune_enumerate_ranked(logits_t, experts_t, slot_t, Yr_t, k, r)
        dl, da, dm, du = pkg.prune_enumerate(logits_d, Y_d, k, r)
        torch.cuda.synchronize()
        loss = loss_t.cpu().numpy().astype(np.float64)
        ref, _, _ = oracle.prune_enumerate(l64, Yfull, k, r)
        check_losses(loss, ref)
        check_argmin(int(amin_t.item()), ref, loss)
        np.testing.assert_allclose(loss, dl.cpu().numpy().astype(np.float64), rtol=1e-5, atol=0)
        assert int(amin_t.item()) == int(da.item()) and int(amask_t.item()) == int(dm.item())
        assert int(unaff_t.item()) == int(du.item())


def test_rank_limited_enumeration_with_streaming_loads():
    """Above half a GB of expert outputs the Gram kernels read them with non-temporal loads (another instantiation).
    Ranked rows assembled from a dense random Y: the ranked enumeration has to return the dense one's losses, which
    the oracle checks at this size in the config 3 and config 4 tests (GPU against GPU here)."""
    E, T, H, k, r, n = 8, 70001, 1024, 2, 6, 4
    logits_t, Y_t = wl.make_enumeration_inputs(E, T, H, "bf16", seed=4242, device=DEV)
    assert Y_t.numel() * 2 >= 512 << 20 and T * n * H * 2 >= 512 << 20
    experts_t = torch.argsort(logits_t, dim=1, descending=True, stable=True)[:, :n].to(torch.int32).contiguous()
    perm = torch.randperm(T * n, device=DEV, generator=torch.Generator(device=DEV).manual_seed(7))
    slot_t = perm.view(T, n).to(torch.int32).contiguous()
    Yr_t = torch.empty((T * n, H), dtype=torch.bfloat16, device=DEV)
    tok = torch.arange(T, device=DEV)
    for j in range(n):
        Yr_t[slot_t[:, j].long()] = Y_t[experts_t[:, j].long(), tok]
    dense = pkg.prune_enumerate(logits_t, Y_t, k, r)
    ranked = pkg.prune_enumerate_ranked(logits_t, experts_t, slot_t, Yr_t, k, r)
    torch.cuda.synchronize()
    assert torch.equal(ranked[0].view(torch.int32), dense[0].view(torch.int32))      # the same dot products, bit for bit
    assert torch.equal(ranked[1], dense[1]) and torch.equal(ranked[3], dense[3])
    head = 3000                                       # and the oracle on a window of the same inputs
    ref, _, _ = oracle.prune_enumerate(wl.to_f64(logits_t[:head]), wl.to_f64(Y_t[:, :head]), k, r)
    part = pkg.prune_enumerate(logits_t[:head].contiguous(), Y_t[:, :head].contiguous(), k, r)
    rest = pkg.prune_enumerate(logits_t[head:].contiguous(), Y_t[:, head:].contiguous(), k, r)
    check_losses(part[0].cpu().numpy().astype(np.float64), ref)
    np.testing.assert_allclose((part[0].double() + rest[0].double()).cpu().numpy(), dense[0].double().cpu().numpy(), rtol=2e-5)


def test_rank_limited_pass_argument_checks():
    cfg, layer = small_layer("bf16", 8, 2, 128, 256, 64, index=15)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    ranked = pkg.moe_expert_outputs_ranked(*ws, 4)
    torch.cuda.synchronize()
    with pytest.raises(pkg.MoepError) as ei:               # r = 4 can reach rank 6 > n_rank = 4
        pkg.prune_enumerate_ranked(*ranked, 2, 4)
    assert ei.value.status == 1
    with pytest.raises(pkg.MoepError) as ei:
        pkg.moe_expert_outputs_ranked(*ws, 9)              # more ranks than experts
    assert ei.value.status == 1
    empty = pkg.moe_expert_outputs_ranked(d["x"][:0].contiguous(), *ws[1:], 4)
    torch.cuda.synchronize()
    assert empty[3].shape == (0, 128)


# ------------------------------------------------------------------ HIP graph replay
def test_enumeration_and_skip_forward_replay_in_a_hip_graph():
    """The entry points allocate nothing and enqueue only kernels, so a caller can capture them.
    Every replay (with the program's own eager work and synchronisations in between) must give
    the bits of the eager call on the same inputs."""
    E, k, r, T, H, F = 8, 2, 6, 700, 128, 256
    cfg, layer = small_layer("bf16", E, k, H, F, T, index=16)
    d = to_dev(layer)
    ws = [d[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    logits0, Y0 = pkg.moe_expert_outputs(*ws)
    torch.cuda.synchronize()
    from paper_2402_14800_amd import binding
    dt = binding.MOEP_BF16
    ws_enum = torch.empty(binding.prune_enumerate_workspace(T, E, H, k, r, dt), dtype=torch.uint8, device=DEV)
    ws_skip = torch.empty(binding.moe_forward_skip_workspace(T, E, H, F, dt), dtype=torch.uint8, device=DEV)
    ws_dir = torch.empty(binding._lib.prune_enumerate_direct_workspace(T, E, H, k, r, dt), dtype=torch.uint8, device=DEV)
    s_logits, s_Y, s_x = logits0.clone(), Y0.clone(), d["x"].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                    # warm-up on the side stream, as torch asks before capture
        pkg.prune_enumerate(s_logits, s_Y, k, r, workspace=ws_enum)
        pkg.moe_forward_skip(s_x, *ws[1:], 0.5, workspace=ws_skip)
        pkg.prune_enumerate_direct(s_logits, s_Y, k, r, workspace=ws_dir)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g_loss, g_amin, g_amask, g_unaff = pkg.prune_enumerate(s_logits, s_Y, k, r, workspace=ws_enum)
        g_out, g_skip, _, _ = pkg.moe_forward_skip(s_x, *ws[1:], 0.5, workspace=ws_skip,
                                                   want_logits=False, want_top2=False)
        g_direct = pkg.prune_enumerate_direct(s_logits, s_Y, k, r, workspace=ws_dir)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    for trial in range(3):
        new_logits = torch.randn((T, E), generator=gen, device=DEV)
        new_Y = torch.randn((E, T, H), generator=gen, device=DEV).to(torch.bfloat16)
        new_x = torch.randn((T, H), generator=gen, device=DEV).to(torch.bfloat16)
        s_logits.copy_(new_logits); s_Y.copy_(new_Y); s_x.copy_(new_x)
        graph.replay()
        torch.cuda.synchronize()
        e_loss, e_amin, e_amask, e_unaff = pkg.prune_enumerate(new_logits, new_Y, k, r)
        e_out, e_skip, _, _ = pkg.moe_forward_skip(new_x, *ws[1:], 0.5)
        torch.cuda.synchronize()
        assert torch.equal(g_loss.view(torch.int32), e_loss.view(torch.int32)), trial
        assert int(g_amin.item()) == int(e_amin.item()) and int(g_unaff.item()) == int(e_unaff.item())
        assert torch.equal(g_skip, e_skip) and torch.equal(g_out.view(torch.int16), e_out.view(torch.int16)), trial
        e_direct = pkg.prune_enumerate_direct(new_logits, new_Y, k, r)
        torch.cuda.synchronize()
        assert torch.equal(g_direct[0].view(torch.int32), e_direct[0].view(torch.int32)), trial
        assert torch.equal(g_direct[1], e_direct[1]) and torch.equal(g_direct[3], e_direct[3])


# ------------------------------------------------------------------ widened entry points at full size
def test_config2_rank_limited_and_topk_skip_full_size():
    """Mid layer (config 2) through the rank-limited pass (sampled rows against the oracle, losses against
    the dense pass and, on a token prefix, the oracle) and through the generalised skipping forward
    (sampled tokens against the oracle)."""
    cfg = wl.CONFIGS["C2"]
    layer = wl.make_layer(cfg, device=DEV)
    ws = [layer[n] for n in ("x", "Wgate", "W1", "W3", "W2")]
    E, k, T = cfg.E, cfg.k, cfg.T
    n_rank = max(min(E, min(k, r) + E - r) for r in cfg.rs)
    logits_d, Y_d = pkg.moe_expert_outputs(*ws)
    ranked = pkg.moe_expert_outputs_ranked(*ws, n_rank)
    torch.cuda.synchronize()
    logits_t, experts_t, slot_t, Yr_t = ranked
    assert torch.equal(logits_t, logits_d)
    W64 = weights_f64(layer)
    tokens = torch.tensor(np.random.default_rng(5).choice(T, 128, replace=False), device=DEV).sort().values
    x64 = wl.to_f64(layer["x"][tokens])
    _, ref_Y = oracle.expert_outputs(x64, wl.to_f64(layer["Wgate"]), W64["W1"], W64["W3"], W64["W2"])
    ex = experts_t[tokens].cpu().numpy()
    for j in range(n_rank):
        got = wl.to_f64(Yr_t[slot_t[tokens, j].long()])
        check_outputs(got, ref_Y[ex[:, j], np.arange(len(tokens))], f"ranked rows, rank {j}")
    prefix = 2048
    pre = pkg.moe_expert_outputs_ranked(*(w[:prefix].contiguous() if i == 0 else w for i, w in enumerate(ws)), n_rank)
    torch.cuda.synchronize()
    for r in cfg.rs:
        lr, ar, mr, ur = pkg.prune_enumerate_ranked(logits_t, experts_t, slot_t, Yr_t, k, r)
        ld, ad, md, ud = pkg.prune_enumerate(logits_d, Y_d, k, r)
        lp, ap, _, _ = pkg.prune_enumerate_ranked(*pre, k, r)
        torch.cuda.synchronize()
        np.testing.assert_allclose(lr.cpu().numpy(), ld.cpu().numpy(), rtol=1e-5)
        assert int(ar.item()) == int(ad.item()) and int(mr.item()) == int(md.item()) and int(ur.item()) == int(ud.item())
        ref, _, _ = oracle.prune_enumerate(pre[0].cpu().numpy().astype(np.float64), densify(pre, E, prefix), k, r)
        lp64 = lp.cpu().numpy().astype(np.float64)
        check_losses(lp64, ref)
        check_argmin(int(ap.item()), ref, lp64)
    # generalised skipping, k = 4 of 8, on the whole batch; the oracle redoes sampled tokens
    beta = float(np.float32(0.1))
    out_t, n_used_t, lg_t, topk_t = pkg.moe_forward_skip_topk(*ws, 4, beta)
    torch.cuda.synchronize()
    ref_out, i_star, experts = oracle.forward_skip_topk(x64, wl.to_f64(layer["Wgate"]), W64["W1"], W64["W3"], W64["W2"],
                                                        4, beta, logits=lg_t[tokens].cpu().numpy())
    assert np.array_equal(n_used_t[tokens].cpu().numpy(), i_star)
    assert np.array_equal(topk_t[tokens].cpu().numpy(), experts)
    check_outputs(wl.to_f64(out_t[tokens]), ref_out, "top-k skip out (sampled tokens)")
    hist = torch.bincount(n_used_t, minlength=5).cpu().numpy()
    assert hist[0] == 0 and hist[1:].sum() == T and (hist[1:] > 0).sum() >= 3
