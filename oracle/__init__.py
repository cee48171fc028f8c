"""CPU oracle for the ShadowSync data-parallel hot path (arXiv 2003.03477).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct numpy
implementation of (i) one trainer's CTR training step (Section 3.1 "Trainer",
Section 3.2 "Optimization Strategies", Algorithm 1 worker loop) and (ii) the three
shadow synchronisation rules (Algorithms 2, 3 and 4).  It exists to check the HIP
library; nothing in the product path may import it.  It imports nothing from the
HIP package and shares no code, constants or helpers with it.

All arithmetic is float64 unless a dtype is passed in.  Every function's docstring
names the passage of the paper it follows and which independent fact pins it
(see tests/test_oracle_*.py).

Parity status of each part (what independent fact pins it):
  mlp / interaction / loss gradients : finite differences + torch autograd (pinned)
  embedding_bag_forward              : dense multiplicity-matrix product (pinned)
  partial pooling over row shards    : multiplicity matrix restricted to each shard's
                                       rows; partials add up to the unsharded result (pinned)
  embedding backward segment sums    : transposed multiplicity matrix (pinned)
  table placement (LPT bin packing)  : brute-force optimum on small cases within the
                                       4/3 - 1/(3m) bound; every shard placed once (pinned)
  stable sort order                  : Python's sorted() on (key, position) (pinned)
  row-wise Adagrad                   : closed form of the first step (pinned)
  Adam on table rows                 : first-step closed form, torch.optim.Adam when every
                                       row is touched every step, untouched rows keep their
                                       state (pinned)
  S-EASGD / S-MA / S-BMUF            : conservation laws, fixed points, scalar
                                       recurrences (pinned)
  Hogwild (racy) schedules           : parity unpinned by nature; only the
                                       serialised schedule is defined here
  the paper's absolute NE figures    : parity unpinned (proprietary data)
"""

from .dlrm import (  # noqa: F401
    DenseLayout,
    adam_update,
    bf16_round,
    bce_with_logits,
    dlrm_forward,
    dlrm_backward,
    embedding_bag_forward,
    embedding_bag_forward_sharded,
    bag_lengths,
    embedding_row_gradients,
    interaction_backward,
    interaction_forward,
    mlp_backward,
    mlp_forward,
    rowwise_adagrad_update,
    stable_sort_by_row,
)
from .sync import (  # noqa: F401
    bmuf_nesterov_round,
    bmuf_round,
    easgd_round,
    easgd_round_literal,
    ma_round,
)
from .trainer import OracleTrainer, normalized_entropy  # noqa: F401
