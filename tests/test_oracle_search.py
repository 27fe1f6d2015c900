"""Pins for the oracle's search rules.  Section 3 of the paper only says that the beam is
smaller than 8; pruning to the live beam, the shrink on end-of-sentence, the candidate order
(score descending, parent ascending, token ascending), the stopping rule and "the best
finished hypothesis wins" are this build's reading, and these tests fix them from outside the
oracle's own code:

* a model whose weight matrices are all zero has logits = the output bias at every step,
  whatever the state, so the whole search has a closed form; the expected translations
  below were derived by hand from the rules and are written out as literals;
* on tiny random models the oracle's translations are compared with a separate
  implementation of the rules that walks the oracle's (separately pinned) step functions,
  on inputs where hypotheses finish, the beam shrinks and candidates tie exactly;
* copies of the oracle with one rule broken are compiled here, on the CPU, and every one of
  them has to fail the closed-form checks.
"""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from workloads import synth


def _zero_model(oracle, out_b, E=4, H=4, A=4, R=4):
    """Every weight matrix zero: t = tanh(0) = 0 and logits = out.b at every step."""
    V = len(out_b)
    p = synth.full_model(seed=0, V=V, E=E, H=H, A=A, R=R)
    for k in p:
        p[k] = np.zeros_like(p[k])
    p["out.b"] = np.asarray(out_b, np.float32)
    return p, oracle.OracleModel(p)


def _logp(out_b):
    b = np.asarray(out_b, np.float64)
    return b - np.log(np.exp(b).sum())


# Each case: output bias, beam, k, max_steps -> tokens, number of steps, score as a sum of
# log-probabilities of the listed tokens (token 0 = end of sentence).
CLOSED_FORM = [
    # Ties.  Step 1: tokens 1, 2, 3 tie; the two kept are (parent 0, token 1) and (0, 2).
    # Step 2: all six candidates tie; lowest parent first, then lowest token: [1, 1] and
    # [1, 2].  Nothing finished, so the first live hypothesis is the result.
    dict(b=[-10, 0, 0, 0, -5, -5], beam=2, k=3, max_steps=2, tokens=[1, 1], steps=2, score_of=[1, 1]),
    # Shrink and stop.  Step 1 keeps token 0 (finished, empty translation, beam 2 -> 1) and
    # token 1.  Step 2 keeps ONE candidate, [1] + token 0: finished with a lower score, beam
    # 1 -> 0, search over after 2 of the 10 steps.
    dict(b=[2, 0, -1], beam=2, k=2, max_steps=10, tokens=[], steps=2, score_of=[0]),
    # A finished hypothesis wins over a live one with a higher score.  Step 1: token 1 (live),
    # token 0 (finished, log p = -1.349).  Step 2 keeps one candidate, [1, 1] with -0.698.
    dict(b=[-1, 0, -3], beam=2, k=2, max_steps=2, tokens=[], steps=2, score_of=[0]),
    # Beam 1 never sees token 0 (rank 2 of 3): three greedy steps.
    dict(b=[0, 1, -1], beam=1, k=2, max_steps=3, tokens=[1, 1, 1], steps=3, score_of=[1, 1, 1]),
    # Pruning to the live beam, not to k: step 1 keeps tokens 1, 2, 3 (beam 3 of k = 4);
    # step 2 has 12 candidates in score order 1+1, {1+2, 2+1}, {1+3, 2+2, 3+1}, ...:
    # kept are [1, 1], [1, 2] and (parent 1 = hypothesis [2]) [2, 1].  Step 3's best is [1, 1, 1].
    dict(b=[-20, 3, 2, 1, 0], beam=3, k=4, max_steps=3, tokens=[1, 1, 1], steps=3, score_of=[1, 1, 1]),
    # Token 0 is third at step 1 (order 1, 2, 0 of beam 3): it finishes with the empty
    # translation and the beam drops to 2.  Every later finished hypothesis scores lower, and
    # the two live slots never end: step 2 keeps [1, 1] and [1, 2] ([2, 1] ties with [1, 2] and
    # has the higher parent), steps 3 and 4 likewise.  Four steps, the empty translation wins.
    dict(b=[-2.5, 0, -1, -3], beam=3, k=3, max_steps=4, tokens=[], steps=4, score_of=[0]),
    # Pruning to the LIVE beam.  Step 1 (beam 3): token 1 live, token 0 finished, token 2 live;
    # beam 3 -> 2.  Step 2 keeps two candidates: [1, 1] and [1] + 0 (finished, lower score);
    # beam 2 -> 1.  Steps 3-5 keep one: [1, 1, 1], ... up to the step limit.  (Keeping three
    # candidates at step 2 and 3 would end the search after step 3.)
    dict(b=[-1, 0, -3], beam=3, k=3, max_steps=5, tokens=[], steps=5, score_of=[0]),
]


def _check_closed_form(oracle):
    for case in CLOSED_FORM:
        p, m = _zero_model(oracle, case["b"])
        src = np.array([1, 2], np.int32)
        toks, score, steps = m.translate(src, beam=case["beam"], topk=case["k"], max_steps=case["max_steps"])
        lp = _logp(case["b"])
        want = sum(lp[t] for t in case["score_of"])
        assert toks.tolist() == case["tokens"], (case, toks.tolist())
        assert steps == case["steps"], (case, steps)
        assert abs(float(score) - want) < 1e-5, (case, float(score), want)


def test_closed_form_searches(oracle):
    _check_closed_form(oracle)


def test_scores_of_equal_logits_are_equal(oracle):
    """What the tie cases rest on: equal biases give bit-equal log-probabilities."""
    p, m = _zero_model(oracle, [-10, 0, 0, 0, -5, -5])
    logits, lse, lp, idx = m.output(np.zeros(4, np.float32), 6)
    assert idx.tolist() == [1, 2, 3, 4, 5, 0]
    assert lp[0] == lp[1] == lp[2] and lp[3] == lp[4]


# ------------------------------------------------- a second implementation of the rules ----

def _reference_search(m, p, src, beam, k, max_steps):
    """The rules, written from their statement: live hypotheses as (score, tokens, state)."""
    enc = m.encode(p["E_src"][src])
    P = m.attention_precompute(enc)
    live = [(np.float32(0.0), [], enc[0, :m.H].copy())]
    b_live, finished, steps = beam, None, 0
    events = {"shrunk_then_continued": False, "replaced": False, "tie": False}
    while steps < max_steps and b_live > 0 and live:
        cands = []
        for parent, (sc, toks, s) in enumerate(live):
            y = p["E_tgt"][toks[-1] if toks else 0]
            _, _, ctx, s_new = m.cgru_step(P, enc, y, s)
            t = m.readout(s_new, y, ctx)
            _, _, lp, idx = m.output(t, k)
            for j in range(k):
                cands.append((np.float32(sc + lp[j]), parent, int(idx[j]), s_new))
        steps += 1
        cands.sort(key=lambda c: (-float(c[0]), c[1], c[2]))
        kept = cands[:b_live]
        if len(cands) > b_live and kept[-1][0] == cands[b_live][0]:
            events["tie"] = True
        new_live = []
        for sc, parent, tok, s_new in kept:
            if tok == 0:
                if finished is None or sc > finished[0]:
                    events["replaced"] |= finished is not None
                    finished = (sc, list(live[parent][1]))
                b_live -= 1
            else:
                new_live.append((sc, live[parent][1] + [tok], s_new))
        if b_live < beam and b_live > 0 and new_live and steps < max_steps:
            events["shrunk_then_continued"] = True
        live = new_live
    if finished is not None:
        return finished[1], finished[0], steps, events
    return live[0][1], live[0][0], steps, events


def test_translate_equals_reference_search_on_small_models(oracle):
    seen = {"shrunk_then_continued": 0, "replaced": 0, "tie": 0, "finished_nonempty": 0, "unfinished": 0}
    for seed in range(12):
        V = 9
        # (large weights make the end-of-sentence probability swing from step to step, so that a
        # later finished hypothesis can beat an earlier one)
        p = synth.full_model(seed=100 + seed, V=V, E=6, H=8, A=5, R=7, w_std=0.6 if seed < 6 else 2.5, b_std=0.3)
        p["out.b"][0] += 0.4 * (seed % 4)                    # how soon hypotheses finish
        if seed % 2:
            # tokens 3 and 4 made indistinguishable: equal logits and equal next states, so
            # candidates and hypotheses tie exactly
            p["out.W"][4] = p["out.W"][3]
            p["out.b"][4] = p["out.b"][3]
            p["E_tgt"][4] = p["E_tgt"][3]
        m = oracle.OracleModel(p)
        rng = np.random.default_rng(seed)
        src = rng.integers(1, V, size=int(rng.integers(1, 6))).astype(np.int32)
        for beam, k in ((2, 3), (3, 3), (4, 6)):
            toks, score, steps = m.translate(src, beam=beam, topk=k, max_steps=7)
            r_toks, r_score, r_steps, ev = _reference_search(m, p, src, beam, k, 7)
            assert toks.tolist() == r_toks and steps == r_steps, (seed, beam, k)
            assert score == r_score, (seed, beam, k)
            for key in ("shrunk_then_continued", "replaced", "tie"):
                seen[key] += bool(ev[key])
            seen["finished_nonempty"] += bool(r_toks) and r_steps < 7
            seen["unfinished"] += r_steps == 7
    # the inputs really exercise every rule
    assert all(v > 0 for v in seen.values()), seen


# ------------------------------------------------------------- mutants of the oracle ----

MUTANTS = {
    "beam never shrinks": ("--b_live;", ";"),
    "parents ordered descending": ("return a->parent < b->parent;", "return a->parent > b->parent;"),
    "tokens ordered descending": ("return a->token < b->token;", "return a->token > b->token;"),
    "last finished hypothesis wins": ("if (!have_fin || c->score > fin_score) {", "if (1) {"),
    "pruned to the beam, not to the live beam": ("int take = b_live < nc ? b_live : nc;", "int take = beam < nc ? beam : nc;"),
    "live hypothesis preferred": ("    if (have_fin) {\n        n_out = fin_len;", "    if (have_fin && n_live == 0) {\n        n_out = fin_len;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_closed_form_cases_catch_a_broken_rule(oracle, tmp_path, name):
    here = os.path.dirname(os.path.abspath(oracle.__file__))
    src = open(os.path.join(here, "q8_oracle.c")).read()
    old, new = MUTANTS[name]
    assert src.count(old) == 1, "the oracle's source no longer contains %r exactly once" % old
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_file.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-I" + here, str(c_file), "-o", str(so_file), "-lm"])
    saved = oracle._lib
    oracle._lib = oracle.load(str(so_file))
    try:
        with pytest.raises(AssertionError):
            _check_closed_form(oracle)
    finally:
        oracle._lib = saved
    _check_closed_form(oracle)                               # the real oracle is back and passes


# ------------------------------------------------------------------------ finiteness ----

def test_non_finite_inputs_are_an_error(oracle):
    x = np.ones(8, np.float32)
    oracle.quantize(x)
    for bad in (np.nan, np.inf, -np.inf):
        y = x.copy()
        y[3] = bad
        with pytest.raises(FloatingPointError):
            oracle.quantize(y)
        L = oracle.QLinear(np.ones((2, 8), np.float32))
        with pytest.raises(FloatingPointError):
            L.gemv(y)
        with pytest.raises(FloatingPointError):
            L.gemv_fp32(y)
    with pytest.raises(FloatingPointError):
        oracle.QLinear(np.array([[1.0, np.nan]], np.float32))
    oracle.quantize(x)                                       # the count does not stick
