"""The oracle's pins must be able to fail: every planted mistake of tests/oracle_mutations.py, applied
to the oracle's source text, has to turn at least one pin red (and the unmodified oracle none).
The mistakes are planted in the oracle, on the CPU; nothing here touches a GPU."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

from oracle_mutations import MUTATIONS

HERE = os.path.dirname(os.path.abspath(__file__))
PINS = [os.path.join(HERE, f) for f in ("test_oracle_prefill.py", "test_oracle_saliency_topk.py",
                                        "test_oracle_decode_positions.py")]


def _run(idx):
    env = dict(os.environ)
    env.pop("SP_ORACLE_MUTATION", None)
    if idx is not None:
        env["SP_ORACLE_MUTATION"] = str(idx)
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + PINS,
                       env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=os.path.dirname(HERE))
    return p.returncode, p.stdout[-600:]


def test_every_planted_mistake_turns_a_pin_red():
    assert "SP_ORACLE_MUTATION" not in os.environ, "not to be run inside a mutation run"
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(_run, [None] + list(range(len(MUTATIONS)))))
    rc, tail = results[0]
    assert rc == 0, "the unmodified oracle fails its pins:\n" + tail
    survivors = [MUTATIONS[i][0] for i, (rc, _) in enumerate(results[1:]) if rc != 1]
    assert not survivors, "planted mistakes that no pin notices: %s" % survivors
