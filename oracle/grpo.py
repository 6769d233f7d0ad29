"""GRPO token loss on selected tokens and its gradients, fp64.

Follows Sec. 2: ratio r_{i,t} (Eq. 1), group-relative advantage (Eq. 2),
clipped surrogate S_{i,t} (Eq. 3), token loss S - beta * KL (Eq. 4; beta = 0
in every experiment of Sec. 5.1), sequence/group mean objective (Eq. 5), and
Sec. 3.1: the Horvitz-Thompson estimator (Eq. 6, Eq. 9) whose gradient is the
weighted sum of token gradients (App. A).  Also the per-token entropy of the
policy, the quantity plotted in the entropy figure of Sec. 5.

Per-token KL term of Eq. 4: the paper keeps it abstract and names, in the
footnote to Eq. 4, the sampled-token log-probability difference as the usual
approximation.  Two sampled-token forms are provided, both functions of
d = logp_ref - logp of the sampled token:
  KL_LOG_RATIO   -d                     (the footnote's form)
  KL_NONNEG      exp(d) - d - 1 >= 0    (the estimator of the GRPO formulation
                                         the paper builds on, Shao et al. 2024)

The policy is a softmax language model head: pi_theta(v | context of token k)
= softmax(W h_k)_v with no bias and temperature 1 (App. C.3).

Sign: the paper maximises J; this module returns loss = -J_hat and the
gradients of that loss.

Test infrastructure: not used by the product path.
"""
import numpy as np

KL_LOG_RATIO, KL_NONNEG = 0, 1


def advantages(rewards, eps_adv=1e-6):
    """Eq. 2.  rewards [P, G] -> A_hat [P, G]: (R - mean) / (std + eps) with the
    population standard deviation (1/G) of the prompt's group."""
    R = np.asarray(rewards, dtype=np.float64)
    mu = R.mean(axis=1, keepdims=True)
    sigma = np.sqrt(((R - mu) ** 2).mean(axis=1, keepdims=True))
    return (R - mu) / (sigma + eps_adv)


def log_softmax_rows(Z):
    """log pi over the vocabulary for each row of logits Z [n, V]."""
    m = Z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(Z - m).sum(axis=1, keepdims=True))
    return Z - lse


def token_logp(hidden, W, ids):
    """log pi_theta(o_k | .) for each token: row k of log_softmax(hidden W^T) at ids[k]."""
    H = np.asarray(hidden, dtype=np.float64)
    Wd = np.asarray(W, dtype=np.float64)
    logpi = log_softmax_rows(H @ Wd.T)
    return logpi[np.arange(len(ids)), np.asarray(ids, dtype=np.int64)]


def forward_logp(hidden, W, ids):
    """Forward pass alone (the log-probability evaluation that precedes the loss in Sec. 2's cost
    structure: behaviour and reference log-probs are produced this way).  Returns dict(logp [n],
    entropy [n])."""
    Hm = np.asarray(hidden, dtype=np.float64)
    if Hm.shape[0] == 0:
        return dict(logp=np.zeros(0), entropy=np.zeros(0))
    logpi = log_softmax_rows(Hm @ np.asarray(W, dtype=np.float64).T)
    return dict(logp=logpi[np.arange(Hm.shape[0]), np.asarray(ids, dtype=np.int64)], entropy=entropy_rows(logpi))


def surrogate(logp, old_logp, A, eps_lo, eps_hi):
    """Eq. 1 and Eq. 3 for arrays of tokens.

    Returns (r, S, g) with g = dS/dlogp: r*A where the unclipped term is the
    active (smaller-or-equal) branch of the min and the clip passes r through
    (boundaries inclusive), 0 otherwise.
    """
    logp = np.asarray(logp, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    r = np.exp(logp - np.asarray(old_logp, dtype=np.float64))
    r_clip = np.clip(r, 1.0 - eps_lo, 1.0 + eps_hi)
    S = np.minimum(r * A, r_clip * A)
    active = ((A > 0) & (r <= 1.0 + eps_hi)) | ((A < 0) & (r >= 1.0 - eps_lo))
    g = np.where(active, r * A, 0.0)
    return r, S, g


def kl_term(logp, ref_logp, kind):
    """Sampled-token KL term of Eq. 4 and its derivative w.r.t. logp."""
    d = np.asarray(ref_logp, dtype=np.float64) - np.asarray(logp, dtype=np.float64)
    if kind == KL_LOG_RATIO:
        return -d, np.ones_like(d)
    if kind == KL_NONNEG:
        return np.exp(d) - d - 1.0, 1.0 - np.exp(d)
    raise ValueError("unknown KL form")


def entropy_rows(logpi):
    """-sum_v pi_v log pi_v for each row of log-probabilities [n, V]."""
    return -np.sum(np.exp(logpi) * logpi, axis=1)


def loss_and_grads(hidden, W, ids, old_logp, adv_tok, w, eps_lo=0.2, eps_hi=0.2,
                   grad_scale=1.0, ref_logp=None, beta_kl=0.0, kl_kind=KL_LOG_RATIO):
    """Masked, HT-weighted GRPO loss over the given (kept) tokens.

    hidden [n, H], W [V, H], ids [n] target token ids, old_logp [n],
    adv_tok [n] = A_hat of each token's rollout, w [n] = the per-token factor
    m/(n_rollouts * T_i * p_{i,t}) of Eq. 5-6; ref_logp [n] = log-probability of
    the sampled token under the reference policy (only read when beta_kl != 0).

    Token objective L_k = S_k - beta_kl * KL_k (Eq. 4); loss = -sum_k w_k L_k ;
    dlogits_k = c_k (onehot(ids_k) - softmax_k) with
    c_k = -grad_scale * w_k * (dS_k/dlogp_k - beta_kl * dKL_k/dlogp_k) ;
    dH = dlogits W ;  dW = dlogits^T H.
    Returns dict(loss, logp [n], dH [n, H], dW [V, H], S [n], r [n], kl [n],
    entropy [n], c [n]).
    """
    Hm = np.asarray(hidden, dtype=np.float64)
    Wd = np.asarray(W, dtype=np.float64)
    ids = np.asarray(ids, dtype=np.int64)
    w = np.asarray(w, dtype=np.float64)
    n = Hm.shape[0]
    if n == 0:
        return dict(loss=0.0, logp=np.zeros(0), dH=np.zeros_like(Hm), dW=np.zeros_like(Wd),
                    S=np.zeros(0), r=np.zeros(0), kl=np.zeros(0), entropy=np.zeros(0), c=np.zeros(0))
    logpi = log_softmax_rows(Hm @ Wd.T)            # [n, V]
    rows = np.arange(n)
    logp = logpi[rows, ids]
    r, S, g = surrogate(logp, old_logp, adv_tok, eps_lo, eps_hi)
    kl, dkl = np.zeros(n), np.zeros(n)
    if beta_kl != 0.0:
        kl, dkl = kl_term(logp, ref_logp, kl_kind)
    loss = -float(np.sum(w * (S - float(beta_kl) * kl)))
    c = -float(grad_scale) * w * (g - float(beta_kl) * dkl)     # dLoss/dlogp_k
    dZ = -np.exp(logpi) * c[:, None]                # -c * softmax
    dZ[rows, ids] += c                              # + c * onehot
    dH = dZ @ Wd
    dW = dZ.T @ Hm
    return dict(loss=loss, logp=logp, dH=dH, dW=dW, S=S, r=r, kl=kl, entropy=entropy_rows(logpi), c=c)


def objective_value(hidden, W, ids, old_logp, adv_tok, w, eps_lo=0.2, eps_hi=0.2,
                    ref_logp=None, beta_kl=0.0, kl_kind=KL_LOG_RATIO):
    """Only the scalar loss (used by finite-difference pins)."""
    logp = token_logp(hidden, W, ids)
    _, S, _ = surrogate(logp, old_logp, adv_tok, eps_lo, eps_hi)
    if beta_kl != 0.0:
        S = S - float(beta_kl) * kl_term(logp, ref_logp, kl_kind)[0]
    return -float(np.sum(np.asarray(w, dtype=np.float64) * S))
