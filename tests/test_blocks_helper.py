"""Host-only checks of the block-size helper: every suggestion satisfies the sketch's constraints
(the C library accepts it) and lands on the path it names."""
import math

import pytest

from oracle import blockperm as O
from paper_2602_06071_amd import binding as B
from paper_2602_06071_amd.blocks import suggest_blocks


@pytest.mark.parametrize("d,k,kappa,s,want", [
    (4194304, 8192, 8, 2, "in"),       # the gradient configuration's shape: Br = 16 or 8
    (65536, 4096, 4, 2, "in"),
    (16384, 1024, 8, 8, "in"),         # kappa*Br = 128 with Br = 16 >= s
    (16384, 1024, 8, 32, "out"),       # s = 32 needs Br >= 32: output-stationary
    (65536, 4096, 1, 8, "in"),
    (4000, 256, 2, 4, "in"),           # d not a multiple of the block: padded grid
    (1000, 90, 3, 5, "in"),            # k = 90: Br = 30, three slots of 32 tile rows
    (5000, 7 * 97, 2, 8, "generic"),   # k = 679: Br = 97 padded to 128 rows, twice
    (49152, 768, 3, 4, "in"),          # kappa = 3: 96 stacked rows in a 128-row tile
    (16896, 528, 32, 8, "grouped"),    # k = 16 * 33, s = 8: no block of 32 rows or more, kappa*16 = 512
    (1000, 384, 2, 4, "in"),           # M = 12: no multiple of 64 gives 12 blocks, Bc = 84
    (20480, 320, 5, 2, "in"),          # kappa = 5: Br = 16, 80 stacked rows in a 128-row tile
])
def test_suggestions_are_valid_and_on_the_named_path(d, k, kappa, s, want):
    Bc, Br, path = suggest_blocks(d, k, kappa, s)
    assert path == want
    p = O.Params(d, k, Bc, Br, kappa, s)
    p.check()                                        # the oracle's statement of the constraints
    assert k % Br == 0 and math.ceil(d / Bc) == k // Br and kappa <= k // Br and s <= Br
    if path == "in":
        padded = 1 << (Br - 1).bit_length()
        assert kappa * padded <= 128 and (Bc % 64 == 0 or Bc == -(-d // (k // Br)))
    if path == "grouped":
        assert Br in (1, 2, 4, 8, 16) and kappa * Br > 128 and (Bc % 64 == 0 or Bc == -(-d // (k // Br)))
    if path == "out":
        assert Br in (32, 64, 128) and (Bc % 64 == 0 or Bc == -(-d // (k // Br)))
    B.Sketch(d, k, Bc, Br, kappa, s).close()         # and the library's (host-side create)


def test_impossible_requests_raise():
    with pytest.raises(ValueError):
        suggest_blocks(1024, 8, 16, 1)               # kappa > any M
    with pytest.raises(ValueError):
        suggest_blocks(0, 8, 1, 1)
