"""GPU: the HIP library against the ATen CPU operators on PyTorch's own OpInfo samples.

The paper's acceptance test (Section 3.3: an operator passes when all of its OpInfo samples pass for every dtype,
against the ATen CPU reference of Section 3.2), applied to every operator of the library through the C ABI.
Samples that ask for something outside the ABI are reported as unsupported by the driver, not passed.
"""
import warnings

import pytest

from tests import opinfo_driver as D

pytestmark = pytest.mark.gpu


def test_library_passes_every_supported_opinfo_sample():
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        report = D.sweep(D.LibraryBackend())
    print(D.summarise(report))
    D.check(report)
    assert len(report) == len(D.ADAPTERS)
    assert sum(r["passed"] for r in report.values()) > 2500
