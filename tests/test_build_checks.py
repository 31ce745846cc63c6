"""The build's own checks of the generated assembly, on hand-written lines (no compiler run)."""
from paper_2605_15250_amd import build as Bd


def test_reads_of_a_scalar_register_are_told_from_writes():
    # a copy out of the register, a range that contains it, a compare and a lane write read it
    assert Bd._reads_register("s_mov_b32 s56, s51", "s51")
    assert Bd._reads_register("s_lshl_b64 s[0:1], s[50:51], 2", "s51")
    assert Bd._reads_register("s_cmp_lt_u32 s51, s18", "s51")
    assert Bd._reads_register("v_writelane_b32 v40, s51, 3", "s51")
    # a write to it, another register with the same digits in front, and an instruction without operands do not
    assert not Bd._reads_register("s_add_i32 s51, s4, s38", "s51")
    assert not Bd._reads_register("s_mov_b32 s56, s510", "s51")
    assert not Bd._reads_register("s_mov_b32 s5, s1", "s51")
    assert not Bd._reads_register("s_barrier", "s51")
