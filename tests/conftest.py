import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _o
    _o.lib()
    return _o


@pytest.fixture(scope="session", autouse=True)
def contraction_mode():
    """NF_CONTRACTION=bf16x6 (or bf16x9) runs the whole suite with the wide contractions on the bf16
    matrix cores (three-way split operands, six or nine piece products); unset or f32: the default
    fp32 matrix-core instructions."""
    want = os.environ.get("NF_CONTRACTION", "")
    if want in ("", "f32"):
        yield
        return
    assert want in ("bf16x6", "bf16x9"), f"NF_CONTRACTION={want!r}: expected f32, bf16x6 or bf16x9"
    from paper_2402_14139_amd import binding as B
    prev = B.nf_contraction(B.NF_CONTRACT_BF16X6 if want == "bf16x6" else B.NF_CONTRACT_BF16X9)
    yield
    B.nf_contraction(prev)
