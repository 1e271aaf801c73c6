import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


# Mutation runs of the oracle's pins (see tests/oracle_mutations.py): with SP_ORACLE_MUTATION=<index>
# the oracle module is built from its source text with one planted mistake.  CPU only.
_MUT = os.environ.get("SP_ORACLE_MUTATION")
if _MUT is not None:
    import types

    import oracle
    from oracle_mutations import MUTATIONS

    _name, _old, _new = MUTATIONS[int(_MUT)]
    _path = os.path.join(ROOT, "oracle", "sp_oracle.py")
    _src = open(_path).read()
    assert _src.count(_old) == 1, "mutation %r does not apply exactly once" % _name
    _mod = types.ModuleType("oracle.sp_oracle")
    _mod.__file__ = _path
    exec(compile(_src.replace(_old, _new), _path, "exec"), _mod.__dict__)
    sys.modules["oracle.sp_oracle"] = _mod
    oracle.sp_oracle = _mod
