"""The GPU tests' view of the harness plumbing (paper_2512_17910_amd/harness.py)."""
from paper_2512_17910_amd.harness import (DEV, TOL, DeviceBatch, check_grouping, host_operands, maxnorm_rel,  # noqa: F401
                                          raw_bits, to_dev, to_f64)
