"""Pins for the analytic cost (Section 3.2) and Strassen stop rule (Section 3.3.2), worked by hand."""
from oracle import cost_model as cm


def test_block_cost_hand_values():
    # k=3, i_c=o_c=64, n=4: alpha=6 -> 2*64*216 + 64*64*36 + 4*6*(8+2) = 27648 + 147456 + 240
    assert cm.block_cost(4, 3, 64, 64) == 27648 + 147456 + 240
    # n=1 (sliding window): alpha=3 -> 2*64*27 + 4096*9 + 1*3*4
    assert cm.block_cost(1, 3, 64, 64) == 3456 + 36864 + 12
    # k=2, i_c=3, o_c=16, n=2: alpha=3 -> 2*3*27 + 48*9 + 2*3*5
    assert cm.block_cost(2, 2, 3, 16) == 162 + 432 + 30


def test_plane_cost_uses_ceil_blocks():
    # 56x56 outputs, n=6 -> ceil(56/6)=10 blocks a side
    assert cm.plane_cost(6, 3, 64, 64, 56, 56) == 100 * cm.block_cost(6, 3, 64, 64)
    # 7x7 outputs, n=4 -> 2x2 blocks
    assert cm.plane_cost(4, 3, 512, 512, 7, 7) == 4 * cm.block_cost(4, 3, 512, 512)


def test_best_tile_examples():
    # 64ch 56x56, k=3, alpha<=8: plane costs / 1e6 for n=1..6 are
    # 126.5, 57.8, 42.8, 34.4, 35.3, 32.8 -> n=6
    costs = [cm.plane_cost(n, 3, 64, 64, 56, 56) for n in range(1, 7)]
    assert [round(c / 1e6, 1) for c in costs] == [126.5, 57.8, 42.8, 34.4, 35.3, 32.8]
    assert cm.best_tile(3, 64, 64, 56, 56) == 6
    # 512ch 7x7: n=4 (4 blocks) beats n=6 (4 blocks of a larger alpha) and n=7 is out of range
    assert cm.best_tile(3, 512, 512, 7, 7) == 4
    # 7x7 kernel with alpha<=8 only admits n in {1,2}
    assert cm.best_tile(7, 64, 64, 112, 112) == 2
    assert cm.scheme(1, 32, 64, 112, 112) == "gemm"
    assert cm.scheme(3, 64, 64, 56, 56) == "F(6,3)"
    # with alpha_max = k the only admissible n is 1 -> sliding window
    assert cm.scheme(3, 64, 64, 56, 56, alpha_max=3) == "sliding"


def test_strassen_rule():
    # 1024^3: saves 1024^3/8 multiplications against 15 * 512^2 additions -> recurse
    assert cm.strassen_should_recurse(1024, 1024, 1024)
    # left side mnk/8, right side (4mk + 4nk + 7mn)/4: for a cube of side s recurse iff s/8 > 15/4, s > 30
    assert cm.strassen_should_recurse(32, 32, 32)
    assert not cm.strassen_should_recurse(30, 30, 30)
    assert not cm.strassen_should_recurse(2, 2, 2)


def test_strassen_rule_on_the_papers_table():
    """The matrix sizes of the paper's Strassen table (tests/golden/strassen_table3.txt): the two sides of the rule as
    worked by hand in the fixture, and the rule's verdict -- the paper applied Strassen to all four."""
    import os
    from fractions import Fraction
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "strassen_table3.txt")
    rows = [[int(t) for t in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert [r[:3] for r in rows] == [[256, 256, 256], [512, 512, 512], [512, 512, 1024], [1024, 1024, 1024]]
    h = Fraction(1, 2)
    for a, b, c, ms_without, ms_with, saved, extra in rows:
        n, k, m = a, b, c
        assert m * n * k - 7 * (m * h) * (n * h) * (k * h) == saved
        assert 4 * (m * h) * (k * h) + 4 * (n * h) * (k * h) + 7 * (m * h) * (n * h) == extra
        assert cm.strassen_should_recurse(n, k, m) == (saved > extra) is True
        assert ms_with <= ms_without
