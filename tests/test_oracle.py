"""The CPU oracle against its pins (closed forms, library routines, brute force, finite differences,
the paper's invariants).  CPU only."""
import pytest

import oracle.ais_oracle as O
from tests import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(O)


def test_every_oracle_function_cites_the_passage_it_follows():
    """Each public function of the three oracle modules names the section, equation, algorithm, proposition or
    appendix of the paper that it writes out."""
    import ast
    import os
    import re
    root = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")
    for name in ("ais_oracle.py", "fp8_oracle.py", "lm_head_oracle.py"):
        tree = ast.parse(open(os.path.join(root, name)).read())
        for node in tree.body:
            if isinstance(node, ast.FunctionDef) and not node.name.startswith("_"):
                doc = ast.get_docstring(node) or ""
                assert re.search(r"\b(Alg\.|Eq\.|Sec\.|App\.|Prop\.)", doc), f"{name}: {node.name} cites nothing"
