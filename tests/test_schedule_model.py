"""The schedule calculator against what the paper fixes: Equations 1-4 and Table 2 evaluated by
hand, the statements of Sections 2.3, 3.2, 4.2 and 4.5 that follow from them, Table 1's totals
and the memory picture of Figure 4."""
import itertools

import pytest

from paper_2507_00394_amd import schedule_model as M


def test_table2_closed_forms_by_hand():
    # p = 8 stages, L = 32 layers, pre : attention : post = 1 : 3 : 2 (the ratio used in Section 4.2)
    p, L, pre, attn, post = 8, 32, 1.0, 3.0, 2.0
    assert M.bubble_time("1f1b", p, L, pre, attn, post) == 3 * 7 * 6 * 4 == 504          # Equation 1
    assert M.bubble_time("zb1p", p, L, pre, attn, post) == 7 * 12 * 4 == 336             # Equation 3
    assert M.bubble_time("helix_naive", p, L, pre, attn, post) == 3 * 7 * 3 == 63        # Section 4.5
    assert M.bubble_time("helix_two_fold", p, L, pre, attn, post) == 126
    assert M.bubble_time("helix", p, L, pre, attn, post) == 8 * 7 * 3 == 168             # Table 2
    b, s, h, m = 1, 1024, 64, 16
    bsh = b * s * h
    assert M.activation_elements("1f1b", p, L, b, s, h, stage=3) == 16 * 5 * bsh * 4      # Equation 2
    assert M.activation_elements("zb1p", p, L, b, s, h) == 16 * bsh * 32                  # Equation 4
    assert M.activation_elements("helix", p, L, b, s, h, m=m) == 4 * bsh * 16 * 4         # Table 2
    with pytest.raises(ValueError):
        M.bubble_time("gpipe", p, L, pre, attn, post)


def test_statements_that_follow_from_the_closed_forms():
    p, L = 4, 16
    # attention is absent from HelixPipe's bubble, present in the others (Section 4.5)
    for sch in ("helix_naive", "helix_two_fold", "helix"):
        assert M.bubble_time(sch, p, L, 1, 3, 2) == M.bubble_time(sch, p, L, 1, 300, 2)
    for sch in ("1f1b", "zb1p"):
        assert M.bubble_time(sch, p, L, 1, 300, 2) > M.bubble_time(sch, p, L, 1, 3, 2)
    # ZB1P removes from 1F1B's bubble exactly the pre/post share that backward W can fill (Section 2.3)
    assert M.bubble_time("1f1b", p, L, 1, 3, 2) - M.bubble_time("zb1p", p, L, 1, 3, 2) == 2 * (p - 1) * (1 + 2) * L / p
    # first 1F1B stage: 16 b s h L, whatever p (Section 2.3); last stage a p-th of it
    for q in (2, 4, 8):
        assert M.activation_elements("1f1b", q, 32, 1, 4096, 128, stage=0) == 16 * 4096 * 128 * 32
        assert M.activation_elements("1f1b", q, 32, 1, 4096, 128, stage=q - 1) * q == 16 * 4096 * 128 * 32
    # recomputation without attention: a third more bubble than two-fold, a quarter of the memory (Section 4.5)
    assert M.bubble_time("helix", p, L, 1, 3, 2) * 3 == M.bubble_time("helix_two_fold", p, L, 1, 3, 2) * 4
    assert M.activation_elements("helix_two_fold", p, L, 1, 512, 64, m=8) == 4 * M.activation_elements("helix", p, L, 1, 512, 64, m=8)
    # two-fold doubles the naive bubble
    assert M.bubble_time("helix_two_fold", p, L, 1, 3, 2) == 2 * M.bubble_time("helix_naive", p, L, 1, 3, 2)


def test_helix_mapping():
    for p, L in ((2, 1), (4, 8), (8, 32), (3, 7)):
        assert M.stage_of_pre_attention(0, p) == 0
        assert M.stage_of_post_attention(L - 1, L, p) == 0
        for l in range(1, L):
            # post-attention of layer l-1 and pre-attention of layer l are concatenated on stage l mod p
            assert M.stage_of_pre_attention(l, p) == M.stage_of_post_attention(l - 1, L, p) == l % p
        for l in range(L):
            stages = [M.stage_of_attention(l, i, p) for i in range(p)]
            assert sorted(stages) == list(range(p))            # a loop of p micro batches fills every stage
            assert stages[0] == (l + 1) % p
    # Figure 5's example: one layer, two stages, two micro batches
    assert [M.stage_of_attention(0, i, 2) for i in range(2)] == [1, 0]


def test_boundary_volumes():
    b, s, h = 1, 131072, 4096
    v = M.boundary_elements(b, s, h)
    assert v["attention_to_post"] == 2 * b * s * h
    assert v["pre_to_attention"] == 2 * b * s * h + 3 * h * h
    assert M.boundary_elements(b, s, h, qkv_linear_on_attention_stage=False)["pre_to_attention"] == 4 * b * s * h
    # s >> h: the weights are a small addition (Section 4.2): 3h^2 / 2bsh = 3h / 2s
    assert v["pre_to_attention"] / v["attention_to_post"] == pytest.approx(1 + 3 * h / (2 * s))


def test_table1_totals():
    b, s, h = 2, 4096, 1024
    f = M.layer_flops(b, s, h)
    assert sum(f["forward"].values()) == 4 * b * s * h * (6 * h + s)
    assert sum(f["backward_b"].values()) == 4 * b * s * h * (6 * h + 2 * s)
    assert sum(f["backward_w"].values()) == 4 * b * s * h * 6 * h
    assert f["backward_w"]["attention"] == 0                    # attention has no parameters


def test_figure4_memory_picture():
    """13B-parameter GPT-3 (40 layers, hidden 5120: the paper names only the size), 8 stages of
    8 GPUs, 1F1B, FP16: at 128k tokens the first two stages exceed an 80 GiB GPU, the later ones
    do not, and shorter sequences fit (Section 3.2)."""
    gib = lambda s, stage: M.activation_elements("1f1b", 8, 40, 1, s, 5120, stage=stage) * 2 / 8 / 2 ** 30
    over = [gib(131072, i) > 80 for i in range(8)]
    assert over == [True, True] + [False] * 6
    assert gib(131072, 0) == 100.0 and gib(131072, 1) == 87.5
    assert all(gib(98304, i) <= 80 for i in range(8)) and all(gib(32768, i) <= 80 for i in range(8))


def test_prediction_and_cli(capsys):
    pr = M.predict("helix", 8, 32, 16, 0.0, 10.0, 5.0)
    assert pr.bubble == 8 * 7 * 5.0 and pr.busy == 16 * 4 * (3 * 15.0 + 5.0)
    assert 0 < pr.bubble_fraction < 1
    M.main(["--t-attn-ms", "14.9"])
    import json
    out = json.loads(capsys.readouterr().out)
    assert set(out["schedules"]) == set(M.SCHEDULES)
    assert out["schedules"]["helix"]["bubble_fraction"] < out["schedules"]["zb1p"]["bubble_fraction"] < out["schedules"]["1f1b"]["bubble_fraction"]
