"""Do the oracle's pins bite?  Each case plants one plausible mistake (a wrong sign, a dropped renormalisation, an
off-by-one, swapped operands, a wrong tie rule) in a COPY of the oracle's source and re-runs tests/test_oracle_pins.py
against that copy in a child process: at least one pin has to fail.  The unchanged copy has to pass, which shows that
the failures come from the planted mistake and not from the harness.  CPU only; nothing here touches the GPU path.
"""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# name -> (text in oracle/moe_reference.py, replacement); the text must occur exactly `count` times (default 1)
MUTANTS = {
    "silu_sign": ("return a / (1.0 + np.exp(-a))", "return a / (1.0 + np.exp(a))"),
    "swiglu_branches_swapped": ("return (silu(gate) * up) @", "return (silu(up) * gate) @"),
    "router_picks_smallest": ('return np.argsort(-logits, axis=1, kind="stable")',
                              'return np.argsort(logits, axis=1, kind="stable")'),
    "ties_to_higher_index": ('return np.argsort(-logits, axis=1, kind="stable")',
                             'return logits.shape[1] - 1 - np.argsort(-logits[:, ::-1], axis=1, kind="stable")'),
    "eq1_not_renormalised_over_selection": ("return ex / ex.sum(axis=1, keepdims=True)",
                                            "return ex / np.exp(logits - m).sum(axis=1, keepdims=True)"),
    "top_k_minus_one": ("taken = flags & (np.cumsum(flags, axis=1) <= count)",
                        "taken = flags & (np.cumsum(flags, axis=1) < count)"),
    "pruning_ignored_by_router": ("    allowed[list(kept)] = True\n    order = routing_order(logits)\n"
                                  "    sel = _first_in_order(order, allowed, min(k, len(kept)))\n"
                                  "    b = renormalised_weights(logits, sel)",
                                  "    allowed[:] = True\n    order = routing_order(logits)\n"
                                  "    sel = _first_in_order(order, allowed, min(k, len(kept)))\n"
                                  "    b = renormalised_weights(logits, sel)"),
    "pruned_experts_dropped_without_rerouting": (
        "    sel = _first_in_order(order, allowed, min(k, len(kept)))\n    b = renormalised_weights(logits, sel)",
        "    sel = _first_in_order(order, np.ones(E, dtype=bool), min(k, E)) & allowed[None, :]\n"
        "    b = np.nan_to_num(renormalised_weights(logits, sel))"),
    "pruned_weights_keep_full_normalisation": (
        "    sel = _first_in_order(order, allowed, min(k, len(kept)))\n    b = renormalised_weights(logits, sel)",
        "    sel = _first_in_order(order, allowed, min(k, len(kept)))\n"
        "    b = renormalised_weights(logits, sel | _first_in_order(order, np.ones(E, dtype=bool), min(k, E))) * sel"),
    "loss_not_squared": ("        loss[i] = np.sum(diff * diff)", "        loss[i] = np.sqrt(np.sum(diff * diff))"),
    "loss_is_mean_over_tokens": ("        loss[i] = np.sum(diff * diff)",
                                 "        loss[i] = np.sum(diff * diff) / diff.shape[0]"),
    "argmin_ties_to_highest_index": ("    return loss, int(np.argmin(loss)), masks\n\n\ndef prune_enumerate_gram_form",
                                     "    return loss, int(len(loss) - 1 - np.argmin(loss[::-1])), masks\n\n\n"
                                     "def prune_enumerate_gram_form"),
    "mask_bit_off_by_one": ("m |= 1 << int(e)", "m |= 1 << (int(e) + 1)"),
    "subsets_in_reverse_order": ("return list(itertools.combinations(range(E), r))",
                                 "return list(itertools.combinations(range(E), r))[::-1]"),
    "full_layer_takes_k_plus_one": ("    sel = _first_in_order(order, np.ones(E, dtype=bool), min(k, E))\n"
                                    "    a = renormalised_weights(logits, sel)\n    return np.einsum",
                                    "    sel = _first_in_order(order, np.ones(E, dtype=bool), min(k + 1, E))\n"
                                    "    a = renormalised_weights(logits, sel)\n    return np.einsum"),
    "gram_form_sign": ("d = renormalised_weights(logits, sel) - a", "d = renormalised_weights(logits, sel) + a"),
    "gram_form_transposed_contraction": ('G = np.einsum("eth,fth->tef", Y, Y)', 'G = np.einsum("eth,fth->tef", Y, Y[::-1])'),
    "skip_rule_inverted": ("return e0, e1, delta < theta, delta", "return e0, e1, delta > theta, delta"),
    "skip_rule_on_weights_difference": ("theta = np.float32(-np.inf) if b <= 0.0 else np.float32(math.log(b))",
                                        "theta = np.float32(-np.inf) if b <= 0.0 else np.float32(b - 1.0)"),
    "skipped_tokens_not_renormalised": ("a0 = np.where(skip, 1.0, 1.0 / (1.0 + rho))", "a0 = 1.0 / (1.0 + rho)"),
    "skipping_tokens_skip_the_first_expert": ("        first = np.nonzero(e0 == e)[0]\n",
                                              "        first = np.nonzero((e0 == e) & ~skip)[0]\n"),
    "gram_form_argmin_ties_to_highest_index": ("    return loss, int(np.argmin(loss)), masks\n\n\ndef prune_enumerate_streamed",
                                               "    return loss, int(len(loss) - 1 - np.argmin(loss[::-1])), masks\n\n\n"
                                               "def prune_enumerate_streamed"),
    "median_is_mean": ("return float(np.median(rho))", "return float(np.mean(rho))"),
    "median_of_inverse_ratio": ("rho = np.exp(l64[t, order[:, 1]] - l64[t, order[:, 0]])\n    return float",
                                "rho = np.exp(l64[t, order[:, 0]] - l64[t, order[:, 1]])\n    return float"),
    "topk_rule_against_wrong_total": ("while tail[i] > b * total:", "while tail[i] > b * tail[1]:"),
    "topk_rule_keeps_one_fewer": ("        i_star[t] = i\n", "        i_star[t] = max(1, i - 1)\n"),
    "topk_skip_not_renormalised": ("coef = coef / coef.sum(axis=1, keepdims=True)",
                                   "coef = coef / w.sum(axis=1, keepdims=True)"),
    "stats_skip_the_first_expert": ("chosen = order[t, :k]", "chosen = order[t, 1:k + 1]"),
    "stats_pairs_counted_once": ("            for j in chosen:\n                co[i, j] += 1",
                                 "            for j in chosen:\n                co[i, j] += 1 if j >= i else 0"),
    "frequency_keeps_least_selected": ("key=lambda e: (-int(count[e]), e)", "key=lambda e: (int(count[e]), e)"),
    "frequency_ties_keep_higher_index": ("key=lambda e: (-int(count[e]), e)", "key=lambda e: (-int(count[e]), -e)"),
}


def run_pins_against(tmp_path, name, old, new):
    root = tmp_path / name
    pkg = root / "oracle"
    pkg.mkdir(parents=True)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            shutil.copy(os.path.join(ROOT, "oracle", f), pkg / f)
    src = (pkg / "moe_reference.py").read_text()
    if old is not None:
        assert src.count(old) == 1, f"{name}: the text to replace occurs {src.count(old)} times"
        (pkg / "moe_reference.py").write_text(src.replace(old, new))
    env = dict(os.environ, MOEP_TEST_ORACLE_ROOT=str(root), PYTHONDONTWRITEBYTECODE="1")
    proc = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p",
                           "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return name, proc.returncode, proc.stdout[-1500:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    tmp = tmp_path_factory.mktemp("oracle_mutants")
    jobs = [("unchanged", None, None)] + [(n, o, r) for n, (o, r) in MUTANTS.items()]
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        done = list(pool.map(lambda j: run_pins_against(tmp, *j), jobs))
    return {name: (rc, out) for name, rc, out in done}


def test_pins_pass_on_an_unchanged_copy(outcomes):
    rc, out = outcomes["unchanged"]
    assert rc == 0, out


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_a_pin_fails_for_each_planted_mistake(outcomes, name):
    rc, out = outcomes[name]
    assert rc == 1, f"no pin noticed the planted mistake {name!r} (pytest exit status {rc}):\n{out}"
