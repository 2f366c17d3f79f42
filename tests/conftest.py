import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    import __graft_entry__
    __graft_entry__.ensure_built()   # the tests load the library the tree holds and build one only when there is none


@pytest.fixture(scope="session")
def oracle():
    import os
    override = os.environ.get("OSDP_ORACLE_PY")   # the mutation test points this at a deliberately broken copy
    if override:
        import importlib.util
        spec = importlib.util.spec_from_file_location("oracle", str(Path(override) / "__init__.py"),
                                                      submodule_search_locations=[override])
        _oracle = importlib.util.module_from_spec(spec)
        sys.modules["oracle"] = _oracle
        spec.loader.exec_module(_oracle)
    else:
        import oracle as _oracle
    _oracle.build()
    return _oracle
