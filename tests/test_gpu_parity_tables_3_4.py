"""The paper's accuracy experiment (Section 5.1, Tables 3 and 4) through the kernels: Q and the cache
from N(0, sigma^2) or U(-a, a), context 8K, BF16, relative Frobenius error against the fp64 oracle.
The MUL variant runs Algorithm 1's arithmetic ("Base"), ADD_COMP runs Algorithm 2's ("AMLA"); the
printed errors are in tests/golden/table3_table4_accuracy.txt, and the CPU emulations of both
algorithms reproduce them (tests/test_oracle_method.py).  The kernels run unsplit here, as the paper's kernel
does: under split-KV every split normalises by its own sum of rounded weights, which cancels more of the
weight-rounding error (FP32 emulation of this sample: 1.770e-3 unsplit, 1.740e-3 in 32 splits), so the
split figures sit a few per cent under the printed ones.  A statement about error levels, not parity: collected
after the parity files."""
import os

import numpy as np
import pytest

from test_gpu_parity import ADD, COMP, LSE_TOL, MUL, env, run_gpu, to_dev  # noqa: F401

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table3_table4_accuracy.txt")
with open(GOLD) as f:
    ROWS = [(a, float(b), float(c), float(d)) for a, b, c, d in
            (ln.split() for ln in f if ln.strip() and not ln.startswith("#"))]


@pytest.mark.parametrize("family,param,base_printed,amla_printed", ROWS)
def test_kernels_reproduce_the_printed_accuracy_tables(env, family, param, base_printed, amla_printed):
    torch, orc, amla, wl = env
    case = wl.make_accuracy_case(family, param)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    dev = to_dev(torch, case)
    err = {}
    for name, v in (("mul", MUL), ("add", ADD), ("comp", COMP)):
        out, lse = run_gpu(torch, amla, case, dev, variant=v, num_splits=1)
        err[name] = orc.frobenius_error(out.reshape(-1, 512), want.reshape(-1, 512))
        assert np.abs(lse - want_lse).max() <= LSE_TOL, name
    print(f"{family} {param:g}: printed Base {base_printed:.2e} AMLA {amla_printed:.2e} | "
          f"mul {err['mul']:.3e} add {err['add']:.3e} comp {err['comp']:.3e}", flush=True)
    # Band: the printed figures carry three digits (0.3 %); one 256-row sample spreads 0.3 % on the flat columns
    # (FP32 emulation of Algorithm 1 on four seeds: 1.770e-3 .. 1.777e-3) and 2-4 % on the peaked ones; 64-key
    # blocks against the paper's 512 and the normalisation by the sum of rounded weights move the emulated figure
    # by 0.1-0.6 %.  3 % / 8 % leave a factor of two to three on that.
    tol = 0.03 if param == 1.0 else 0.08
    assert abs(err["mul"] - base_printed) < tol * base_printed, err
    assert abs(err["comp"] - amla_printed) < tol * amla_printed, err
