"""Every GPU parity case must be able to FAIL: removing a sub-block (self-attention, cross-attention, feed-forward,
rotary embedding, causal mask) from the oracle has to move the case's asserted error measures to at least ten
times their bounds.  Otherwise a kernel that returned zeros for that sub-block would pass the case.

Small cases are mutated here, live.  The full-shape cases (one 8B-class layer, the 27-layer encoder, the 36-layer
decoder) take minutes per mutant; their ratios are written by tests/golden/make_full_depth.py, which calls only the
oracle, into tests/golden/full_depth_meta.json, and read back here."""
import json
import os

import pytest

from tests import parity_cases as PC

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "full_depth_meta.json")

_base = {}


def base_of(case):
    if case.name not in _base:
        _base[case.name] = PC.oracle_passes(case)
    return _base[case.name]


@pytest.mark.parametrize("mutation", list(PC.MUTATIONS))
@pytest.mark.parametrize("case", PC.CASES, ids=[c.name for c in PC.CASES])
def test_small_case_detects_mutation(case, mutation):
    applies, _ = PC.MUTATIONS[mutation]
    if not applies(case):
        pytest.skip("the module has no such sub-block")
    ratios = PC.mutation_ratio(case, mutation, base_of(case))
    seen = [r for r in ratios if r is not None]
    assert seen, "no pass of this case can see the mutation"
    if mutation in case.blind:
        # stated as blind: another case of the same module shape must see it (checked on that case)
        other = PC.CASE[case.covered_by]
        assert other.cfg.as_dict() == case.cfg.as_dict() and mutation not in other.blind
        return
    for (p, t), r in zip(case.passes, ratios):
        assert r is None or r >= PC.DISCRIMINATION, (case.name, mutation, (p, t), r)


def test_full_shape_cases_detect_mutations():
    with open(GOLDEN) as f:
        meta = json.load(f)
    # per case: mutation -> passes (indices) that must see it at 10x.  What a case is blind to is judged alone by its
    # companion case: next to the feed-forward, single-token attention over 3072 keys (dec8b_L1 passes 1, 2) and
    # cross-attention over 3072 context rows (act_L8) reach only 5-8x; with the other sub-blocks zeroed they reach 50x.
    want = {
        "dec8b_L1": {"self_attention": [0], "ffn": [0, 1, 2], "rope": [0], "causal_mask": [0]},
        "dec8b_L1_attn": {"self_attention": [0, 1, 2], "rope": [0, 1, 2], "causal_mask": [0]},
        "act_L8": {"self_attention": [0], "ffn": [0]},
        "act_L8_cross": {"cross_attention": [0]},
        "vit_L27": {"self_attention": [0], "ffn": [0]},
        "vit_L1_T8192": {"ffn": [0]},
        "vit_L1_T8192_attn": {"self_attention": [0]},
        "dec8b_L36": {"self_attention": [0], "ffn": [0], "rope": [0], "causal_mask": [0]},
    }
    for name, muts in want.items():
        got = meta["mutation_ratio"][name]
        for m, passes in muts.items():
            for i in passes:
                assert got[m][i] >= PC.DISCRIMINATION, (name, m, i, got[m])
    # every applicable mutation of every full-shape case is accounted for: seen here or by the named companion
    companions = {("dec8b_L1", "self_attention"): "dec8b_L1_attn", ("dec8b_L1", "rope"): "dec8b_L1_attn",
                  ("act_L8", "cross_attention"): "act_L8_cross", ("vit_L1_T8192", "self_attention"): "vit_L1_T8192_attn"}
    for name, case in PC.full_cases().items():
        for m, (applies, _) in PC.MUTATIONS.items():
            if not applies(case):
                continue
            n_pass = len(meta["mutation_ratio"][name][m])
            seen = set(want[name].get(m, []))
            if len(seen) < n_pass:
                assert (name, m) in companions and m in want[companions[(name, m)]], (name, m)


def test_long_prompt_chunks_detect_mutations():
    """The 16384-token case of tests/test_gpu_fullsize.py, mutated live on its three chunks of rows: the plain variant
    must see the feed-forward go, the attention-alone variant the attention, the rotary embedding and the causal mask."""
    for attention_alone, mutations in ((False, ["ffn"]), (True, ["self_attention", "rope", "causal_mask"])):
        case = PC.long_prompt_case(attention_alone)
        x = case.x()
        rows, base = PC.long_prompt_oracle(case, x=x)
        for m in mutations:
            applies, make = PC.MUTATIONS[m]
            assert applies(case)
            w, over = make(case)
            _, mut = PC.long_prompt_oracle(case, w, over, x=x)
            r = max(PC.stated_err(mut, base) / PC.TOL, PC.contrib_err(mut, base, x[rows]) / PC.TOL_CONTRIB)
            print("long prompt%s: %s removed -> %.1f x the bound" % (" (attention alone)" if attention_alone else "", m, r))
            assert r >= PC.DISCRIMINATION, (case.name, m, r)
