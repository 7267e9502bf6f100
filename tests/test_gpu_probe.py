"""The hand-over probe (a measurement aid of the library): in every mode the results the stages hand over must be
the right ones, and no bounded wait may give up."""
import pytest

from paper_2410_00531_amd import binding as B


@pytest.mark.gpu
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("kib", [16, 64])
def test_handover_probe_exchanges_the_right_results(mode, kib):
    r = B.tpi_probe_handover(512 << 20, kib, mode, reps=2)
    assert r["results_ok"] == 1 and r["gave_up"] == 0
    assert r["segments"] == (512 << 20) // (2048 * 1024 * kib)
    assert 0.05 < r["tb_per_s"] < 8.0


def test_handover_probe_argument_errors():
    def code(*a):
        with pytest.raises(B.TpiError) as ei:
            B.tpi_probe_handover(*a, stream=0)
        return ei.value.code
    assert code(512 << 20, 8, 0) == B.TPI_EINVAL            # segment below the ring's depth
    assert code(512 << 20, 24, 0) == B.TPI_EINVAL           # not a multiple of 16 KiB
    assert code((512 << 20) + 4096, 16, 0) == B.TPI_EINVAL  # not whole segments
    assert code(512 << 20, 16, 4) == B.TPI_EINVAL
    assert code(512 << 20, 16, 0, 0) == B.TPI_EINVAL


@pytest.mark.gpu
def test_gemm_loop_probe_runs_every_variant_and_the_complete_loop_multiplies():
    """The loop probe launches the 256x256 tile's kernel as the library runs it (leave_out = 0: its result is
    checked against the same sums taken on the host) and with one or two of its activities left out (timing
    only).  A variant may be slower than the complete loop (without the matrix instructions the loop waits for every load), but not by a large factor."""
    full = B.tpi_probe_gemm_loop(0, reps=3)
    assert full["result_ok"] == 1
    assert abs(full["tflop_per_launch"] - 2 * 8 * 512 * 8192 * 3584e-12) < 1e-9
    assert 100.0 < full["tflops"] < 2500.0
    for leave_out in range(1, 7):
        r = B.tpi_probe_gemm_loop(leave_out, reps=3)
        assert r["result_ok"] == -1 and r["tflops"] == 0.0
        assert 0.0 < r["us_per_launch"] < 3.0 * full["us_per_launch"], (leave_out, r, full)


def test_gemm_loop_probe_argument_errors():
    for args in ((7, 1), (-1, 1), (0, 0), (0, 1001)):
        with pytest.raises(B.TpiError) as ei:
            B.tpi_probe_gemm_loop(*args, stream=0)
        assert ei.value.code == B.TPI_EINVAL
