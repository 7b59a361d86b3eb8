"""Seeded input generator: bf16 rounding, reproducibility, head independence (no GPU)."""
import numpy as np
import torch

from paper_2507_00394_amd import inputs as I


def test_bf16_rounding_matches_torch_and_ties_to_even():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    bits = I.float_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    t = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert I.bf16_bits_to_float(I.float_to_bf16_bits(t)).tolist() == [1.0, 1.0 + 2.0 ** -6]
    assert np.array_equal(I.float_to_bf16_bits(I.bf16_bits_to_float(bits, np.float32)), bits)


def test_heads_regenerate_alone_and_differ():
    cfg = I.CONFIGS[1]
    full = I.all_inputs_bits(cfg, threads=2)
    for t in ("q", "k", "v", "dO"):
        assert full[t].shape == (cfg.B, cfg.H, cfg.S, cfg.D) and full[t].dtype == np.uint16
        for bh in range(cfg.B * cfg.H):
            assert np.array_equal(full[t].reshape(-1, cfg.S, cfg.D)[bh], I.head_tensor_bits(cfg.cfg_id, t, bh, cfg.S, cfg.D))
    assert not np.array_equal(full["q"][0, 0], full["q"][0, 1])
    assert not np.array_equal(full["q"][0, 0], full["k"][0, 0])
    x = I.bf16_bits_to_float(full["q"])
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02


def test_k_multiplier_is_exact_doubling():
    a = I.bf16_bits_to_float(I.head_tensor_bits(5, "k", 3, 64, 128, 1.0))
    b = I.bf16_bits_to_float(I.head_tensor_bits(5, "k", 3, 64, 128, 2.0))
    assert np.array_equal(2 * a, b)


def test_samples_are_stratified_and_in_range():
    for cid in (2, 4, 5):
        cfg = I.CONFIGS[cid]
        rows = I.sample_rows(cfg)
        assert len(rows) == 256 and all(0 <= bh < cfg.B * cfg.H and 0 <= i < cfg.S for bh, i in rows)
        got = {i for _, i in rows}
        assert {0, 1, 127, 128, cfg.S // 2, cfg.S - 1} <= got
        full, mid, tail = I.sample_cols(cfg)
        BH = cfg.B * cfg.H
        assert set(full) == {0, BH - 1}
        assert all({0, 1, 127, 128, cfg.S - 1} <= set(c) for c in full.values())
        # the tail stratum reaches EVERY other (batch, head) slice, inside the last 4096 positions
        assert set(tail) == set(range(1, BH - 1))
        assert 120 <= sum(len(c) for c in tail.values()) <= 128 and all(cfg.S - 4096 <= j < cfg.S for c in tail.values() for j in c)
        # mid-range columns of a middle slice
        assert set(mid) == {BH // 2} and len(mid[BH // 2]) == 16
        assert all(cfg.S // 2 <= j < cfg.S - 4096 for j in mid[BH // 2])
        assert (full, mid, tail) == I.sample_cols(cfg)
        assert rows == I.sample_rows(cfg)
