import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def blob():
    from paper_2212_01185_amd import synth
    return synth.make_blob(0)


@pytest.fixture(scope="session")
def sharp_blob():
    from paper_2212_01185_amd import synth
    return synth.make_blob(0, sharp=True)


@pytest.fixture(scope="session")
def orc(blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(blob)


@pytest.fixture(scope="session")
def orc_sharp(sharp_blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(sharp_blob)


@pytest.fixture(scope="session")
def logistic_blob():
    from paper_2212_01185_amd import synth
    return synth.make_blob(0, dist=synth.DIST_LOGISTIC)


@pytest.fixture(scope="session")
def orc_logistic(logistic_blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(logistic_blob)


@pytest.fixture(scope="session")
def paper_blob():
    from paper_2212_01185_amd import synth
    return synth.make_paper_blob(0)


@pytest.fixture(scope="session")
def paper_sharp_blob():
    from paper_2212_01185_amd import synth
    return synth.make_paper_blob(0, sharp=True)


@pytest.fixture(scope="session")
def orc_paper(paper_blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(paper_blob)


@pytest.fixture(scope="session")
def diagonal_blob():
    from paper_2212_01185_amd import synth
    return synth.make_diagonal_blob(0)


@pytest.fixture(scope="session")
def diagonal_sharp_blob():
    from paper_2212_01185_amd import synth
    return synth.make_diagonal_blob(0, sharp=True)


@pytest.fixture(scope="session")
def orc_diagonal(diagonal_blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(diagonal_blob)


@pytest.fixture(scope="session")
def predictor_blob():
    from paper_2212_01185_amd import synth
    return synth.make_predictor_blob()


@pytest.fixture(scope="session")
def orc_predictor(predictor_blob):
    from oracle import pcc_oracle
    return pcc_oracle.Oracle(predictor_blob)
