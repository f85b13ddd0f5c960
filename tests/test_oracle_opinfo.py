"""The oracle against the ATen CPU operators on PyTorch's own OpInfo samples.

The paper's criterion for an operator is agreement with the ATen CPU operator on every OpInfo sample of every
supported dtype (Sections 3.2, 3.3).  Here that criterion is applied to the ORACLE: a pin that does not come from
the oracle or the HIP library, and that covers argument patterns (0-dim operands, Python scalars, broadcast and
non-contiguous views, empty tensors, keepdim / dim variants) this repository's own generators may not think of.
"""
import warnings

from tests import opinfo_driver as D


def test_oracle_matches_aten_cpu_on_every_supported_opinfo_sample():
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        report = D.sweep(D.OracleBackend())
    D.check(report)
    assert len(report) == len(D.ADAPTERS)
    assert sum(r["passed"] for r in report.values()) > 2500
