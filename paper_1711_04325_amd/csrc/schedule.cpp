// Host scalars of Appendix A.1 (RMSprop warm-up blend) and A.2 (slow-start learning rate).
#include <math.h>

#include "rn50.h"

extern "C" double rn50_alpha_sgd(double epoch, double center, double period)
{
    // Exponential approach to 1/2 at `center`, then a straight line that reaches 1 at center+period/2.
    // The line's slope is 1/period: it continues the exponential's slope at the joint (ELU-like) and
    // hits 1 exactly where the text says the transition ends.
    const double t = (epoch - center) / period;
    if (t < 0.0) return 0.5 * exp(2.0 * t);
    if (t < 0.5) return 0.5 + t;
    return 1.0;
}

extern "C" double rn50_alpha_sgd_transition(double epoch, double center, double period, int transition)
{
    // Appendix A.1 names the alternatives it rejected without formulas; each is the plainest function of its name through
    // 1/2 at `center`, the smooth ones with the paper's own slope 1/period there.
    const double t = (epoch - center) / period;
    switch (transition) {
    case RN50_TRANSITION_ELU: return rn50_alpha_sgd(epoch, center, period);
    case RN50_TRANSITION_LINEAR: return fmin(1.0, fmax(0.0, 0.5 + t));
    case RN50_TRANSITION_SIGMOID: return 1.0 / (1.0 + exp(-4.0 * t));
    case RN50_TRANSITION_SUDDEN: return t < 0.0 ? 0.0 : 1.0;
    default: return nan("");
    }
}

extern "C" double rn50_alpha_rmsprop(double a_sgd, double eta_rmsprop, double eta_sgd)
{
    return (1.0 - a_sgd) * eta_rmsprop / eta_sgd;
}

extern "C" double rn50_lr_base(int n_workers, int b_local) { return 0.1 * n_workers * (double)b_local / 256.0; }

extern "C" double rn50_lr_slow_start(double epoch, int n_workers, int b_local)
{
    static const double until[3] = {40.0, 70.0, 85.0};
    static const double mult[4] = {0.5, 0.075, 0.01, 0.001};
    int stage = 0;
    while (stage < 3 && epoch >= until[stage]) ++stage;
    return mult[stage] * rn50_lr_base(n_workers, b_local);
}

extern "C" int rn50_recipe_hparams_transition(double epoch, int n_workers, int b_local, int transition, rn50_opt_hparams *hp)
{
    if (!hp || !(epoch >= 0.0) || n_workers <= 0 || b_local <= 0) return RN50_EINVAL;
    if (transition < RN50_TRANSITION_ELU || transition > RN50_TRANSITION_SUDDEN) return RN50_EINVAL;
    const double eta = rn50_lr_slow_start(epoch, n_workers, b_local);
    const double a_sgd = rn50_alpha_sgd_transition(epoch, 10.0, 5.0, transition);
    hp->eta = (float)eta;
    hp->mu1 = 0.9f;
    hp->mu2 = 0.99f;
    hp->eps = 1e-8f;
    hp->a_sgd = (float)a_sgd;
    hp->a_rms = (float)rn50_alpha_rmsprop(a_sgd, 3e-4, eta);
    hp->wd = 1e-4f;
    hp->g_scale = (float)(1.0 / n_workers);
    return RN50_OK;
}

extern "C" int rn50_recipe_hparams(double epoch, int n_workers, int b_local, rn50_opt_hparams *hp)
{
    return rn50_recipe_hparams_transition(epoch, n_workers, b_local, RN50_TRANSITION_ELU, hp);
}
