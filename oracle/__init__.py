"""CPU oracle for the fast-process local step of system-aware biased local SGD.

TEST INFRASTRUCTURE ONLY.  Plain, slow NumPy float64 code written from the paper's
definitions; it shares nothing with the GPU library and must never be imported by it.
Only the tests, the smoke check and the benchmark's CPU-baseline leg call into here.

Pins (see tests/test_oracle_*.py): every function below is checked against closed forms,
finite differences, brute force or library special cases; none is "parity unpinned".
Whole-run accuracy claims of the paper's tables need its datasets and are not modelled.
"""
from .losses import softmax_cross_entropy                      # noqa: F401
from .selection import topk_by_loss, total_order_key            # noqa: F401
from .aggregation import weighted_aggregate, weights_from_tau   # noqa: F401
from .optim import sgd_update                                   # noqa: F401
from .models import MLP, ResNetCifar, WideResNet                            # noqa: F401
from .transformer import TransformerLM                          # noqa: F401
from .precision import round_bf16                               # noqa: F401
from .sampling import allocation, deal, sample_epoch                 # noqa: F401
from .local_sgd import score_losses, local_step, loss_and_grads, GradientProbe  # noqa: F401
from .round import communication_round                            # noqa: F401
from .epoch import multistep_lr, rounds_per_epoch, train_epochs   # noqa: F401
