"""MI355X-native fast path of system-aware biased local SGD (arXiv 2508.08540).

Thin ctypes binding over libbls.so: the functions here only marshal arguments (pointers, sizes,
the HIP stream); every step of the path runs in the library's HIP kernels.  Importing this
package loads the library and fails loudly if it has not been built
(`python -m paper_2508_08540_amd.build`).
"""
from .binding import (  # noqa: F401
    BlsError, Context, Model, lib, library_path, local_step, score_losses, topk_by_loss, topk_by_loss_static, TOPK_STATIC_MAX_N, weighted_aggregate,
    weights_from_tau, sum_limits, sample_epoch, communication_round, train_epochs, ROUND_UNIFORM_WEIGHTS, ROUND_SEQUENTIAL, epoch_allocation, worker_share, MODEL_MLP, MODEL_RESNET_CIFAR, MODEL_WRN, MODEL_ENCODER, AGG_NORMALISE, AGG_BROADCAST, DECLARED_SYMBOLS, PROFILE_CLASSES,
)
