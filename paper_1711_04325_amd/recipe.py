"""Driver of the paper's recipe over many iterations (argument marshalling only): per iteration it asks the library for
the scalars of the current real-valued epoch (slow-start learning rate, Appendix A.2; RMSprop-warm-up blend, Appendix
A.1) and calls rn50_step.  The data pipeline is the caller's: `batches` yields (images, labels) device tensors."""
import torch

from . import binding as rn


class TrainState:
    """Flat device arenas of one worker: parameters, gradient, momentum, second moment, half-precision buffer."""

    def __init__(self, theta):
        self.theta = theta
        self.grad = torch.empty_like(theta)
        self.delta = torch.zeros_like(theta)      # Delta_0 = 0
        self.m = torch.zeros_like(theta)          # m_0 = 0, no bias correction (none in the paper's equations)
        self.grad16 = torch.empty(theta.numel(), dtype=torch.int16, device=theta.device)
        self.loss = torch.zeros(1, device=theta.device)


def run(ctx, state, batches, iterations, iterations_per_epoch, n_workers=1024, b_local=32, bn_eps=2e-5, start_iteration=0,
        on_step=None, transition=rn.TRANSITION_ELU):
    """Runs `iterations` steps; returns the list of losses (one host read per step, after the step was enqueued).
    `transition` selects the RMSprop -> SGD blend: the paper's ELU-like function, or one of the alternatives Appendix A.1
    reports as examined and rejected (rn.TRANSITION_LINEAR / _SIGMOID / _SUDDEN)."""
    losses = []
    it = start_iteration
    for images, labels in batches:
        if len(losses) >= iterations:
            break
        hp = rn.rn50_recipe_hparams_transition(it / float(iterations_per_epoch), transition, n_workers, b_local)
        ctx.step(images, labels, state.theta, state.grad, state.delta, state.m, state.grad16, hp, bn_eps, state.loss)
        losses.append(state.loss.item())
        if on_step is not None:
            on_step(it, hp, losses[-1])
        it += 1
    return losses
