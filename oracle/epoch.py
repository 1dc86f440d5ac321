"""The outer loop of Algorithm 1 on one set of workers: E epochs, each a sampling step followed by communication rounds
until the epoch's allocation is consumed, with the step-size schedule of the experiments (Appendix A.1: SGD with the
MultiStepLR schedule, decay at the listed epochs).

Per epoch t (0-based): the sampler (Section 4.2) assigns N_F samples to the fast and N_S to the slow workers from the
current loss table and that epoch's random keys; worker p's share is its round-robin deal.  Round r hands worker i the
next tau_i * B samples of its share; every worker with a non-empty hand runs its tau_i local steps from the global
model, losses are recorded in the table, models are aggregated (Eq. 4).  The epoch ends when every share is consumed.

Readings where the paper is silent: the loss table the first epoch ranks is an input (e.g. a scoring pass); a worker's
last hand of an epoch may be shorter than tau_i * B, it still takes tau_i steps and its batches wrap around the hand
(the batch rule of the local step), so the step counts behind Eq. (4) stay those of the algorithm's input; a worker whose
share is used up sits the round out (tau = 0: neither trains nor counts); workers keep their momentum across rounds and
epochs; the learning rate of epoch t is lr0 * gamma^(number of milestones <= t) with gamma = 0.1 (the default of the
scheduler the paper names; the tables give only the epochs); weight decay is constant.
"""
import numpy as np

from .round import communication_round
from .sampling import sample_epoch


def multistep_lr(lr0, milestones, gamma, epoch):
    """Learning rate during 0-based epoch `epoch`: one factor gamma per milestone already reached."""
    return float(lr0) * float(gamma) ** sum(1 for m in milestones if int(m) <= int(epoch))


def rounds_per_epoch(shares, taus, batch):
    """Rounds until every worker's share is consumed at tau_i * batch samples per round."""
    need = [-(-len(s) // (t * batch)) for s, t in zip(shares, taus) if t > 0 and len(s) > 0]
    return max(need) if need else 0


def train_epochs(model, params, buffers, momenta, x, y, loss_table, u_fast, u_slow, epochs, tau_f, P_f, tau_s, P_s, lam,
                 batch, lr0, momentum=0.0, weight_decay=0.0, milestones=(), gamma=0.1, scheme="separated",
                 high_loss_to="fast", uniform_weights=False):
    """momenta: list of P_f + P_s momentum dicts (fast workers first); u_fast, u_slow: [epochs, N] random keys.

    Returns (params, buffers, momenta, loss_table, log) with log = [(epoch, round, lr, [tau_i actually run])]."""
    table = np.array(loss_table, dtype=np.float64)
    momenta = [dict(m) for m in momenta]
    taus = [tau_f] * P_f + [tau_s] * P_s
    log = []
    for e in range(epochs):
        lr = multistep_lr(lr0, milestones, gamma, e)
        # the sampler ranks the table as the workers store it: one fp32 number per sample
        alloc = sample_epoch(table.astype(np.float32), u_fast[e], u_slow[e], tau_f, P_f, tau_s, P_s, lam, scheme, high_loss_to)
        shares = list(alloc["fast"]) + list(alloc["slow"])
        for r in range(rounds_per_epoch(shares, taus, batch)):
            workers = []
            for share, tau, mom in zip(shares, taus, momenta):
                hand = share[r * tau * batch:(r + 1) * tau * batch] if tau > 0 else share[:0]
                workers.append(dict(tau=tau if len(hand) else 0, idx=hand, momentum=mom))
            params, buffers, momenta, table = communication_round(model, params, buffers, workers, x, y, batch, lr, momentum,
                                                                 weight_decay, loss_table=table, uniform_weights=uniform_weights)
            log.append((e, r, lr, [w["tau"] for w in workers]))
    return params, buffers, momenta, table, log
