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
