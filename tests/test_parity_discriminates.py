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
    want = {
        "dec8b_L1": ("self_attention", "ffn", "rope", "causal_mask"),
        "vit_L27": ("self_attention", "ffn"),
        "dec8b_L36": ("self_attention", "ffn", "rope", "causal_mask"),
    }
    for name, muts in want.items():
        got = meta["mutation_ratio"][name]
        for m in muts:
            assert min(got[m]) >= PC.DISCRIMINATION, (name, m, got[m])


_pipe_base = []


@pytest.mark.parametrize("module,mutation", PC.PIPE_MUTATIONS)
def test_pipeline_case_detects_mutation(module, mutation):
    """The reduced five-stage pipeline: removing any sub-block of any of its three stacks moves one of the asserted
    measures (or the greedy token ids, which are compared exactly) far past its bound."""
    if not _pipe_base:
        _pipe_base.append(PC.pipeline_oracle())
    base = _pipe_base[0]
    mut = PC.pipeline_oracle((module, mutation))
    m = PC.pipeline_measures(mut, base)
    assert max(m.values()) >= PC.DISCRIMINATION, (module, mutation, m)
    print(module, mutation, {k: round(v, 1) for k, v in m.items()}, mut["tokens"] != base["tokens"])
