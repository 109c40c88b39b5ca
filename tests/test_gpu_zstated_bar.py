"""Summary of the stated layer bar (max|diff| <= 2e-2 x RMS of the oracle output) over every
7B-shape comparison the GPU tests of this process made.  helpers.assert_layer_close asserts a
bar derived from the bf16-operand floor at those shapes; whether the stated bar itself holds is
recorded there and reported here, as an expected failure while it does not."""
import pytest

from helpers import REPORT, STATED_BAR

pytestmark = pytest.mark.gpu


@pytest.mark.xfail(reason="at D = 4096 the worst of millions of elements exceeds 2e-2 x RMS already "
                          "for an exact layer with bf16 operands (test_bf16_operand_rounding_floor)",
                   strict=False)
def test_stated_bar_on_every_7b_shape_comparison():
    if not REPORT:
        pytest.skip("no 7B-shape layer comparison ran in this process")
    misses = [r for r in REPORT if r[1] > STATED_BAR]
    print(f"[stated bar] {len(REPORT) - len(misses)} of {len(REPORT)} comparisons within "
          f"{STATED_BAR} x RMS; worst {max(r[1] for r in REPORT):.4f} (floor of that sample "
          f"{max(REPORT, key=lambda r: r[1])[3]:.4f})", flush=True)
    for what, worst, rms_err, f_worst, f_rms in REPORT:
        print(f"[stated bar] {'MISS' if worst > STATED_BAR else 'ok  '} {what}: {worst:.4f} "
              f"(floor {f_worst:.4f}), rms {rms_err:.5f} (floor {f_rms:.5f})", flush=True)
    assert not misses
