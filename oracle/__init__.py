"""CPU checker ("oracle") for the incremental dynamic-GNN hot path -- TEST INFRASTRUCTURE.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import
this package.  It shares no code with the HIP library and never calls it.

Everything here recomputes every snapshot from scratch in fp64 (paper Section 3.2, Eq. 1); the
incremental rule of Eq. 2 reaches exactly the same quantity, so the from-scratch definition is
the reference for the full, incremental and fallback GPU paths alike.

Pins (see tests/test_oracle_*.py): dense-adjacency matmul and textbook special cases for the
aggregation; a literal set-based Eq. 2 chained over snapshots for the incremental == full
invariant; the generator's own insert/delete lists and brute force for the edge deltas;
torch.nn.GRUCell / LSTMCell and closed forms for the recurrent cells; finite differences and
torch.autograd on a dense-adjacency model for the backward pass.

The max / min aggregators (`oracle.minmax`) are pinned to a dense masked-adjacency formula, the max/min
duality, closed-form special cases and the chained incremental == from-scratch invariant.

The cache-policy simulator (`oracle.cache_policy`: score = future accesses / size - imminence with expiration,
LRU, LFU) is pinned to a textbook page-replacement example, exhaustive search for the optimal policy, closed forms
for cyclic access and the shape of the paper's policy comparison; the paper's printed hit rates themselves are
unpinned (the model and the cache-size normalisation behind them are not given).

Node mini-batches (`oracle.minibatch`: the computational graphs of a set of nodes over the sequence, and the loss
restricted to those nodes) are pinned to hand-worked graphs, dense matrix powers, the full-graph model itself
(locality) and additivity over a partition of the nodes.

Parity unpinned by the paper (pinned only to this package's own definition): the symmetric
degree normalisation (absent from the paper), and the loss (mean squared error on a synthetic
target instead of the paper's forecasting MAE on datasets that are not available).
"""
from .dgnn import *  # noqa: F401,F403
from . import incremental  # noqa: F401
from . import minmax  # noqa: F401
from . import cache_policy  # noqa: F401
from . import minibatch  # noqa: F401
