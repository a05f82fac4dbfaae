"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
arithmetic (blob sizes, residency plan) agrees with the input format and the oracle's closed forms.
No compute call is made here."""
import ctypes
import os
import re

import pytest

import synth
from oracle import counts

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "specverify.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_0-9]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    import paper_2505_10259_amd as P
    names = _declared()
    assert len(names) >= 20
    lib = ctypes.CDLL(P.binding.SO_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in specverify.h but not exported"
    assert sorted(P.binding.EXPORTS) == names
    for n in names:
        assert hasattr(P, n) or hasattr(P.binding, n), f"binding lacks {n}"


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_blob_sizes_match_input_format(name):
    import paper_2505_10259_amd as P
    w = synth.workload(name)
    for s in (w.target, w.target.draft(2, True), w.target.draft(1, False)):
        assert P.spec_layer_blob_elems(s) == s.layer_layout()[1]
        assert P.spec_global_blob_elems(s) == s.global_layout()[1]


def test_bad_shapes_are_errors_not_aborts():
    import paper_2505_10259_amd as P
    from dataclasses import replace
    s = synth.workload("cfg3").target
    for bad in (replace(s, n_kv_heads=5), replace(s, head_dim=127), replace(s, n_experts=9),
                replace(s, n_experts=1), replace(s, d_model=0)):
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_layer_blob_elems(bad)
        assert e.value.code == P.SPEC_ERR_SHAPE
    assert "shape" in P.spec_last_error()


def test_residency_plan_respects_budget_and_memory_model():
    """Resident target parameters + draft + globals + staging ring <= budget, and one more resident
    layer (piece staging: one more piece) would not fit (decoding-phase GPU memory constraint,
    Appendix A.1)."""
    import paper_2505_10259_amd as P
    for name, slots in (("cfg3", 2), ("cfg4", 2), ("cfg5", 3), ("cfg3", 0), ("cfg4", 0)):
        w = synth.workload(name)
        t, d = w.target, w.draft
        R, streamed = P.spec_plan_residency(t, d, w.hbm_weight_budget, slots)
        blob = counts.layer_params(t) * 2
        expert = 3 * t.d_model * t.d_ff * 2
        fixed = (2 * t.vocab * t.d_model + t.d_model) * 2 + d.n_layers * counts.layer_params(d) * 2
        pad = 4096 * (t.n_layers + 8)                       # alignment padding inside blobs
        if slots:                                           # whole-layer slots, whole layers pinned
            ring, unit = slots * blob, blob
            assert abs(streamed - (t.n_layers - R) * blob) < pad
            pinned = 0
        else:                                               # three slots of one expert; pieces pinned too
            ring, unit = 3 * expert, expert
            pinned = (t.n_layers - R) * blob - streamed
            assert -pad < pinned < blob
        used = counts.v_decoding(R * blob + pinned + ring, fixed, 0, 0, 0, 0)
        assert used <= w.hbm_weight_budget + pad
        assert used + unit > w.hbm_weight_budget - pad
        assert 0 < R < t.n_layers
    # piece staging keeps more of each streamed model resident than two whole-layer slots do
    for name in ("cfg3", "cfg4"):
        w = synth.workload(name)
        r0, s0 = P.spec_plan_residency(w.target, w.draft, w.hbm_weight_budget, 0)
        r2, s2 = P.spec_plan_residency(w.target, w.draft, w.hbm_weight_budget, 2)
        blob = counts.layer_params(w.target) * 2
        assert r0 >= r2 + 1 and s2 - s0 > 1.5 * blob
    t = synth.workload("cfg3").target
    assert P.spec_plan_residency(t, None, 0, 2) == (t.n_layers, 0)          # no cap: all resident
    assert P.spec_plan_residency(t, None, 10 ** 12, 2) == (t.n_layers, 0)
    with pytest.raises(P.binding.SpecError) as e:
        P.spec_plan_residency(t, None, 3 * 10 ** 9, 2)
    assert e.value.code == P.SPEC_ERR_BUDGET


def test_null_arguments_are_errors():
    import paper_2505_10259_amd as P
    lib = P.binding.lib
    assert lib.spec_init(None, None, None, None, None, None) == P.SPEC_ERR_ARG
    assert lib.spec_sync(None, 0) == P.SPEC_ERR_ARG
    assert lib.spec_accept(None, None, None, None, None, 1.0, 0, 0, 0, 1, 1, 8, None, None, None) == P.SPEC_ERR_ARG
    assert lib.spec_host_alloc(0, None) == P.SPEC_ERR_ARG


def test_attention_resident_placement_plan():
    """SPEC_FLAG_PIN_ATTENTION at the two streamed model shapes: every attention part is resident, so
    only whole experts cross the link (the decoding-phase transfer of Section 4.1.2 / Appendix A.1, FFN
    parameters only); the budget is respected and no further expert would fit; bytes per pass are within
    one expert of the default placement's (the budget decides how much streams, the policy only which
    bytes) and agree with spec_plan_residency for the default policy."""
    import paper_2505_10259_amd as P
    for name in ("cfg3", "cfg4"):
        w = synth.workload(name)
        t, d = w.target, w.draft
        blob = P.spec_layer_blob_elems(t) * 2
        expert = 3 * ((t.d_model * t.d_ff + 127) // 128 * 128) * 2          # gate, up, down of one expert
        front = blob - t.n_experts * expert                                 # norm gains, QKV, O, router
        dflt = P.spec_plan_placement(t, d, hbm_weight_budget_bytes=w.hbm_weight_budget)
        assert (dflt["resident_layers"], dflt["streamed_bytes_per_pass"]) == P.spec_plan_residency(t, d, w.hbm_weight_budget, 0)
        pin = P.spec_plan_placement(t, d, hbm_weight_budget_bytes=w.hbm_weight_budget, flags=P.SPEC_FLAG_PIN_ATTENTION)
        assert pin["piece_staging"] == 1 and pin["n_slots"] == 3
        R = pin["resident_layers"]
        assert abs(front - (counts.attention_params(t) + 2 * t.d_model + t.n_experts * t.d_model) * 2) < 4096
        assert pin["streamed_bytes_per_pass"] % expert == 0
        assert pin["pinned_piece_bytes"] >= (t.n_layers - R) * front
        used = pin["fixed_bytes"] + pin["ring_bytes"] + R * blob + pin["pinned_piece_bytes"]
        assert used <= w.hbm_weight_budget < used + expert
        assert used + pin["streamed_bytes_per_pass"] == pin["fixed_bytes"] + pin["ring_bytes"] + t.n_layers * blob
        assert abs(pin["streamed_bytes_per_pass"] - dflt["streamed_bytes_per_pass"]) <= expert
    # whole-layer staging ignores the flag; a budget below the attention parts is refused
    w = synth.workload("cfg3")
    a = P.spec_plan_placement(w.target, w.draft, hbm_weight_budget_bytes=w.hbm_weight_budget, n_ring_slots=2)
    b = P.spec_plan_placement(w.target, w.draft, hbm_weight_budget_bytes=w.hbm_weight_budget, n_ring_slots=2,
                              flags=P.SPEC_FLAG_PIN_ATTENTION)
    assert a == b and a["piece_staging"] == 0
    with pytest.raises(P.binding.SpecError) as e:
        P.spec_plan_placement(w.target, w.draft, hbm_weight_budget_bytes=3 * 10 ** 9, flags=P.SPEC_FLAG_PIN_ATTENTION)
    assert e.value.code == P.SPEC_ERR_BUDGET
