"""Oracle of the saturation threshold formulas (test infrastructure only).

Eq. 1 of the paper: a layer's transfer is hidden when the batch's compute lasts at least as
long, i.e. when its FLOPs reach T = t_EP * F_GPU * gamma (gamma >= 1 absorbs jitter).
App. B.4, Eq. 3: calibrated from per-layer wall times of one reference batch of n_ref tokens,
T = gamma * (t_e / t_c) * C_dummy with C_dummy = f_tok * n_ref; when transfers are hidden
(t_e <= t_c) it collapses to gamma * C_dummy, which is also the fallback before calibration.
f_tok for the MoE block alone: K * 6*H*I + 2*H*E counted flop per token.
App. B.4, delivery and fallback: an operator-pinned value overrides the calibration; without a
usable f_tok both the threshold and the work counters are kept in tokens (one unit per token).
"""


def flops_per_token(H, E, K, I):
    return K * 6.0 * H * I + 2.0 * H * E


def threshold_eq1(t_ep, f_gpu, gamma=1.2):
    return t_ep * f_gpu * gamma


def threshold_calibrated(t_c, t_e, c_dummy, gamma=1.2):
    if t_c is None or t_c <= 0:
        return gamma * c_dummy
    return gamma * max(t_e / t_c, 1.0) * c_dummy


def threshold_fallback(f_tok, n_ref, gamma=1.2):
    return gamma * f_tok * n_ref


def resolve_threshold(pinned, t_c, t_e, f_tok, n_ref, gamma=1.2):
    """(threshold, unit): unit "flops" when f_tok is usable, else "tokens"."""
    usable = f_tok is not None and f_tok > 0
    unit = "flops" if usable else "tokens"
    if pinned is not None and pinned > 0:
        return pinned, unit
    per_token = f_tok if usable else 1.0
    return threshold_calibrated(t_c, t_e, per_token * n_ref, gamma), unit
