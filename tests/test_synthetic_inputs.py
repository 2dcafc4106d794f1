"""The seeded workloads are well-formed problems (checked with the oracle's rules)."""
import numpy as np

import synthetic_inputs as S
from oracle import redist_oracle as O


def test_all_workload_pairs_are_valid_redistributions():
    for name, w in S.WORKLOADS.items():
        pairs = S.pairs_of(name)
        assert pairs
        for a, b in pairs:
            ta, tb = O.parse_type(a), O.parse_type(b)
            assert O.wf_type(w["mesh"], ta) and O.wf_type(w["mesh"], tb), (name, a, b)
            assert O.globaltype(ta) == w["gshape"] == O.globaltype(tb)
            assert ta != tb


def test_sampler_is_deterministic_and_covers_short_runs():
    p1, p2 = S.sample_pairs("c5_bf16_attn_8x8"), S.sample_pairs("c5_bf16_attn_8x8")
    assert p1 == p2 and len(p1) == 50
    last_tiles = {O.parse_type(t)[3].c for pr in p1 for t in pr}
    assert 128 in last_tiles and min(last_tiles) <= 16          # whole rows and short runs both occur


def test_global_arrays_are_seeded():
    a = S.global_array("c1_int32_2x2")
    b = S.global_array("c1_int32_2x2")
    assert a.dtype == np.int32 and a.shape == (64, 48) and np.array_equal(a, b)
    i = S.global_array("c1_int32_2x2", "iota")
    assert i[1, 0] == 48
    h = S.global_array("c2_bf16_act_1x8", gshape=(64, 64))
    assert h.dtype == np.uint16
    f = (h.astype(np.uint32) << 16).view(np.float32)
    assert abs(float(f.mean())) < 0.1 and 0.8 < float(f.std()) < 1.2


def test_adversarial_problems_are_the_printed_ones(paper_values):
    """The bench's copies of the four problems of Table "adversarial" against the golden file (which cites the table)."""
    from oracle import redist_oracle as O
    for name, a, b in S.ADVERSARIAL_PROBLEMS:
        ga, gb, _mb = [p.strip() for p in paper_values["adversarial_" + name].split(";")]
        assert O.parse_type(a) == O.parse_type(ga) and O.parse_type(b) == O.parse_type(gb)
        assert O.wf_type(S.PAPER_MESH, O.parse_type(a)) and O.wf_type(S.PAPER_MESH, O.parse_type(b))
