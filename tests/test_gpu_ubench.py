"""The instruction-issue microbenchmark: what a SIMD of this chip does with binary64 matrix and vector
instructions.  The figures under profiles/ come from `python -m paper_1910_11141_amd.ubench`; this test
checks the facts the roofline discussion rests on, with wide margins."""
import pytest

pytestmark = pytest.mark.gpu


def test_matrix_and_vector_instructions_of_one_simd_do_not_overlap():
    from paper_1910_11141_amd import ubench
    simd = ubench.pair("idle", "idle", 1)["simd"]
    assert simd[:4] == simd[4:] and sorted(simd[:4]) == [0, 1, 2, 3]      # waves w and w + 4 share a SIMD
    mfma = ubench.pair("mfma_f64_16x16x4", "idle")["a"]
    assert 60.0 < mfma["per_instr"] < 70.0                               # 1024 multiply-adds in 64 ticks
    fma = ubench.pair("v_fma_f64", "idle")["a"]
    assert 3.9 < fma["per_instr"] < 6.5                                  # 64 multiply-adds in 4 to 5 ticks
    both = ubench.pair("mfma_f64_16x16x4", "v_fma_f64")
    # the matrix wave is not slowed down, the vector wave ends only after both loops' worth of ticks
    assert both["a"]["ticks"] < 1.03 * mfma["ticks"]
    assert both["b"]["ticks"] > 0.95 * (mfma["ticks"] + fma["ticks"])
    one_wave = ubench.pair("mfma_f64+4*v_fma_f64 (one wave)", "idle")["a"]
    assert one_wave["per_instr"] > 0.95 * (mfma["per_instr"] + 4 * fma["per_instr"]) - 2.0
    small = ubench.pair("mfma_f64_4x4x4_4b", "idle")["a"]
    assert 15.0 < small["per_instr"] < 20.0                              # 256 multiply-adds in 17 ticks
    big32 = ubench.pair("mfma_f32_32x32x2", "idle")["a"]
    small32 = ubench.pair("mfma_f32_4x4x1_16b", "idle")["a"]
    assert 60.0 < big32["per_instr"] < 70.0                              # 2048 multiply-adds in 64 ticks
    assert 7.0 < small32["per_instr"] < 11.0                             # 256 multiply-adds in 8: the same rate in 4 x 4 pieces


def test_whole_chip_matrix_rate_is_below_the_published_peak():
    from paper_1910_11141_amd import ubench
    tflops, ms = ubench.mfma_peak(blocks=2048, iters=4000, reps=2)
    assert 40.0 < tflops < 79.0 and ms > 1.0
