"""The usage example of README.md, run as written and checked against the oracle."""
import os
import re

import numpy as np
import pytest
import torch

import oracle
from gnn_synth import config_graph

pytestmark = pytest.mark.gpu


def test_readme_example_runs_and_matches_the_oracle():
    from gpu_util import TOL
    from util import parity_errors
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "README.md")).read()
    code = re.search(r"```python\n(.*?)```", text, re.S).group(1)
    g = config_graph(4, shrink=32)
    rowptr0, colidx0 = g.rowptr.copy(), g.colidx.copy()
    torch.manual_seed(7)
    ns = {"rowptr": g.rowptr, "colidx": g.colidx}
    exec(compile(code, "README.md", "exec"), ns)
    assert ns["did"]  # a shuffled community graph is renumbered by the AES rule
    perm = ns["perm"]
    # the example's X is in renumbered order: row perm[i] belongs to original node i
    X, W1, W2, Y = (ns[k].cpu().numpy() for k in ("X", "W1", "W2", "Y"))
    ew0 = oracle.gcn_norm(rowptr0, colidx0)
    ref = oracle.gcn_model(rowptr0, colidx0, ew0, X[perm], [W1, W2])
    normwise, _ = parity_errors(Y[perm], ref, None)
    assert normwise <= TOL, normwise
