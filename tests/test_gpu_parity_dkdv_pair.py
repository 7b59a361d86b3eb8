"""The head-dimension-128 dK/dV pass walks a key tile's query blocks in three regimes: a plain
path for the first blocks (those the causal diagonal cuts, up to a multiple of seven), a
pipelined path in groups of seven blocks, and the plain path again for what is left, including
a ragged last block.  The sequence lengths here put the boundaries between the regimes at every
remainder of the seven-block groups, with whole and ragged last blocks, for full and causal
attention; every result is compared with the fp64 oracle element by element."""
import pytest

from oracle import attention_ref as A
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu

# full attention: every key tile sees S // 32 whole blocks; the pipelined path needs 14 of them
# (8 to run one group after its first block, 6 that are left to the plain path)
FULL = [32 * 13, 32 * 14, 32 * 14 + 1, 32 * 15 + 31, 32 * 16, 32 * 17 + 5, 32 * 18, 32 * 19 + 30, 32 * 20, 32 * 21 + 1,
        32 * 22, 32 * 28 + 17, 32 * 35]
# causal: key tile t sees (S - 128 t) // 32 blocks, so one length covers many remainders at once
CAUSAL = [32 * 20, 32 * 21 + 9, 1216, 1409, 2047, 2304]


def _check(S, causal, seed):
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(seed, 1, 2, S, 128)
    out = G.run_fwd_bwd(bits, cfg.scale, causal)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], cfg.scale, causal)
    for n in ("dk", "dv", "dq", "o"):
        G.check(n, G.to_f64(out[n]), ref[n])


@pytest.mark.parametrize("S", FULL)
def test_full_attention_block_regimes(S):
    _check(S, False, 7100 + S)


@pytest.mark.parametrize("S", CAUSAL)
def test_causal_block_regimes(S):
    _check(S, True, 7200 + S)


def test_full_attention_many_groups_and_ragged_end():
    """Full attention at a length with 36 seven-block groups per key tile and a ragged last block: every key tile
    runs the pipelined path from its first block (there is no diagonal) for hundreds of blocks."""
    _check(32 * 259 + 17, False, 7300)
