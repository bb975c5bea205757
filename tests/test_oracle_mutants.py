"""Planted mistakes, on the CPU and in the oracle only: each entry changes one
line of a copy of the oracle's source (a wrong sign, an index off by one, a
dropped term, swapped operands, a finishing rule left out) and the pins of
tests/test_oracle_pins.py are run against that copy; at least one of them has
to fail.  This is what says the pins would notice such a mistake.  The oracle
file itself is never touched and the GPU library is not involved."""
import os
import types

import pytest

import tests.test_oracle_pins as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "fdc_oracle.py")).read()

MUTANTS = [
    # Sec. 3.3 mask, Eq. 1
    ("own slot: offset t itself not visible",
     "vis[slot_start[f]: slot_start[f] + t + 1] = True", "vis[slot_start[f]: slot_start[f] + t] = True"),
    ("ancestors: direct parents only, no closure", "stack.extend(parents[g])", "pass"),
    ("ancestor slots: padding visible", "slot_start[g] + valid_len[g]] = True", "slot_start[g] + 99] = True"),
    # layer arithmetic
    ("rotary: wrong sign", "x1 * c - x2 * s, x2 * c + x1 * s", "x1 * c + x2 * s, x2 * c - x1 * s"),
    ("rotary: wrong exponent", "(-np.arange(half, dtype=F64) * 2.0 / D)", "(-np.arange(half, dtype=F64) * 1.0 / D)"),
    ("rotary: keys not rotated", "k = rope(k, pos[:, None], d.rope_base)", "k = k"),
    ("RMSNorm: eps outside the root", "np.sqrt(ms + eps)", "np.sqrt(ms) + eps"),
    ("GQA: wrong KV head", "kh = h // d.group", "kh = h % d.n_kv_heads"),
    ("SwiGLU: gate and up swapped", "h = silu(gu[:, :d.d_mlp]) * gu[:, d.d_mlp:]",
     "h = silu(gu[:, d.d_mlp:]) * gu[:, :d.d_mlp]"),
    ("MLP norm uses the attention gain", 'a = rmsnorm(x, lw["g2"], d.norm_eps)', 'a = rmsnorm(x, lw["g1"], d.norm_eps)'),
    ("softmax scale 1/D", "/ np.sqrt(F64(q.shape[-1]))", "/ F64(q.shape[-1])"),
    ("final norm dropped", 'xn = rmsnorm(x, self.w["gf"], d.norm_eps)', "xn = x"),
    ("MLP residual dropped", 'return x + h @ lw["wd"].T', 'return h @ lw["wd"].T'),
    # Algorithm 1
    ("schedule: one token too many per field", "if done[v] >= content_len[v]:", "if done[v] > content_len[v]:"),
    ("driver: no truncation at the slot length",
     "if t in eos or len(text[b][v]) >= dec.slot_len[v]:", "if t in eos or len(text[b][v]) > dec.slot_len[v]:"),
    ("driver: end tokens inverted", "if t in eos or len", "if t not in eos or len"),
    ("driver: output not fed back", "                last[b][v] = t", "                pass"),
    ("driver: successor released one signal early", "                        if d[b][u] == 0:",
     "                        if d[b][u] <= 1:"),
    ("driver: fixed fields never signal",
     "    d = [[len(preds[v] - set(fixed)) for v in range(F)] for _ in range(B)]",
     "    d = [[len(preds[v]) for v in range(F)] for _ in range(B)]"),
    ("driver: fixed fields decoded again", "if d[b][v] == 0 and v not in fixed}", "if d[b][v] == 0}"),
    ("driver: scenes share their feedback", "    last = [list(start_token) for _ in range(B)]",
     "    last = [list(start_token)] * B"),
    ("driver: every scene reads scene 0's tokens", '                t = int(out["tok"][b * R + i])',
     '                t = int(out["tok"][i])'),
]

PINS = [
    lambda: P.test_ancestors_all_small_dags_bruteforce(3),
    lambda: P.test_chain_dag_full_slots_is_causal_mask(),
    lambda: P.test_mask_invariants_of_the_figure_caption(),
    lambda: P.test_rmsnorm_against_closed_form_and_torch(),
    lambda: P.test_rope_closed_forms_and_invariants(),
    lambda: P.test_attention_single_key_and_against_sdpa(),
    lambda: P.test_schedule_is_optimal_and_respects_dependencies(0),
    lambda: P.test_chain_dag_equals_ordinary_causal_decoding(),
    lambda: P.test_masked_out_kv_has_no_effect_and_visible_kv_has(),
    lambda: P.test_dynamic_driver_without_end_tokens_fills_every_slot(),
    lambda: P.test_dynamic_driver_end_tokens_finish_fields_and_passes_are_minimal(0),
    lambda: P.test_dynamic_driver_scenes_diverge_and_stay_independent(),
    lambda: P.test_dynamic_driver_fixed_text_is_visible_like_a_longer_prefix(),
]


def _pins_all_pass():
    for pin in PINS:
        try:
            pin()
        except Exception:                      # an assertion, or the mistake makes the oracle raise
            return False
    return True


def test_the_pins_pass_on_the_oracle_as_it_is():
    assert _pins_all_pass()


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, what, old, new):
    assert SRC.count(old) >= 1, f"the oracle no longer contains the line this entry changes: {old!r}"
    mutant = types.ModuleType("fdc_oracle_mutant")
    exec(compile(SRC.replace(old, new, 1), "fdc_oracle_mutant.py", "exec"), mutant.__dict__)
    monkeypatch.setattr(P, "O", mutant)
    assert not _pins_all_pass(), f"no pin noticed: {what}"
