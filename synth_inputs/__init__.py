"""Seeded synthetic inputs shaped like the paper's Qwen3 GRPO workloads.

Shared by the tests, the benchmark, the CPU oracle's callers and the HIP
path's callers.  This module only draws random inputs (lengths, hidden
states, head weights, token ids, rewards, log-prob noise); it holds none of
the method's arithmetic (no selection, no advantage, no soft-max, no loss).

The five workloads stand in for the paper's Qwen3 / DAPO-Math-17K rollouts
(Sec. 5.1, App. C.3: 8 rollouts per prompt, response length up to 8192); only
their shapes are taken: head sizes, group sizes and length distributions.
"""
import math
import numpy as np

# name -> P prompts, G rollouts/prompt, (H, V), element type, length law
WORKLOADS = {
    "tiny_fp32": dict(P=2, G=4, H=64, V=512, dtype="f32", lengths=("uniform", 16, 64)),
    "qwen3_0p6b_head": dict(P=8, G=8, H=1024, V=151936, dtype="bf16", lengths=("uniform", 256, 2048)),
    "qwen3_8b_head_rpc": dict(P=16, G=8, H=4096, V=151936, dtype="bf16",
                              lengths=("lognormal", 2048, 0.5, 1, 8192)),
    "qwen3_8b_long_cot": dict(P=8, G=16, H=4096, V=151936, dtype="bf16", lengths=("uniform", 4096, 16384)),
    "wide_head_stress": dict(P=32, G=8, H=5120, V=151936, dtype="bf16",
                             lengths=("pareto", 1.5, 128, 32768), equal_reward_frac=0.1),
    # the paper's second model (App. C.3): Qwen2.5-Math-7B head, responses up to 3000 tokens, run with
    # minimum-cutoff RPC (C = 100); a quarter of the prompts get all-equal rewards (zero-advantage groups)
    "qwen2p5_math_7b_head": dict(P=16, G=8, H=3584, V=152064, dtype="bf16",
                                 lengths=("lognormal", 900, 0.6, 1, 3000), equal_reward_frac=0.25),
}
WORKLOAD_ORDER = ["tiny_fp32", "qwen3_0p6b_head", "qwen3_8b_head_rpc", "qwen3_8b_long_cot", "wide_head_stress",
                  "qwen2p5_math_7b_head"]

W_STD = 0.02
LOGP_NOISE_STD = 0.05


def draw_lengths(law, n, rng):
    """Response lengths T_i (int64, >= 1) for n rollouts."""
    kind = law[0]
    if kind == "uniform":
        return rng.integers(law[1], law[2] + 1, size=n).astype(np.int64)
    if kind == "lognormal":
        median, sigma, lo, hi = law[1:]
        x = np.exp(rng.normal(math.log(median), sigma, size=n))
        return np.clip(np.rint(x), lo, hi).astype(np.int64)
    if kind == "pareto":
        alpha, lo, hi = law[1:]
        x = lo * (1.0 - rng.random(size=n)) ** (-1.0 / alpha)
        return np.clip(np.floor(x), lo, hi).astype(np.int64)
    if kind == "fixed":
        return np.asarray(law[1], dtype=np.int64)
    raise ValueError(kind)


def draw_rewards(P, G, rng, equal_reward_frac=0.0):
    """Bernoulli(0.5) verifier rewards [P, G]; the first ceil(frac*P) prompts get
    one reward value copied to all G rollouts (a zero-advantage group)."""
    R = (rng.random(size=(P, G)) < 0.5).astype(np.float32)
    n_eq = int(math.ceil(equal_reward_frac * P)) if equal_reward_frac > 0 else 0
    R[:n_eq, :] = R[:n_eq, :1]
    return R


def round_to_bf16(x):
    """float32 array -> (float32 array holding bf16-representable values, uint16 bits),
    round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bits = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32), bits


def batch_layout(name, seed, P=None, G=None, lengths=None):
    """Lengths, packed offsets and rewards of one batch (host, numpy)."""
    cfg = dict(WORKLOADS[name])
    P = cfg["P"] if P is None else P
    G = cfg["G"] if G is None else G
    law = cfg["lengths"] if lengths is None else lengths
    rng = np.random.default_rng([seed, 1])
    T = draw_lengths(law, P * G, rng)
    cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
    R = draw_rewards(P, G, rng, cfg.get("equal_reward_frac", 0.0))
    return dict(name=name, P=P, G=G, B=P * G, H=cfg["H"], V=cfg["V"], dtype=cfg["dtype"],
                lengths=T, cu_seqlens=cu, N=int(cu[-1]), rewards=R, seed=seed)


def make_batch_numpy(name, seed, P=None, G=None, lengths=None, H=None, V=None):
    """Full batch on the host: layout plus hidden [N,H], W [V,H] (float32 arrays;
    bf16-representable when the workload's dtype is bf16), ids [N] int32 and
    logp_noise [N] ~ N(0, 0.05) (to be added to the current log-probs to form
    the behaviour policy's)."""
    b = batch_layout(name, seed, P, G, lengths)
    if H is not None:
        b["H"] = H
    if V is not None:
        b["V"] = V
    rng = np.random.default_rng([seed, 2])
    N, Hd, Vd = b["N"], b["H"], b["V"]
    hidden = rng.standard_normal((N, Hd), dtype=np.float32)
    W = rng.standard_normal((Vd, Hd), dtype=np.float32) * np.float32(W_STD)
    if b["dtype"] == "bf16":
        hidden, _ = round_to_bf16(hidden)
        W, _ = round_to_bf16(W)
    b["hidden"] = hidden
    b["W"] = W
    b["ids"] = rng.integers(0, Vd, size=N).astype(np.int32)
    b["logp_noise"] = (rng.standard_normal(N) * LOGP_NOISE_STD).astype(np.float32)
    return b


def make_batch_torch(name, seed, device, P=None, G=None, lengths=None):
    """Same recipe drawn on `device` with torch's seeded generator (the values
    differ from make_batch_numpy's; a test draws once and hands the same
    tensors to both sides).  hidden/W are bf16 tensors for bf16 workloads."""
    import torch
    b = batch_layout(name, seed, P, G, lengths)
    gen = torch.Generator(device=device)
    gen.manual_seed(1_000_003 * seed + 7)
    dt = torch.bfloat16 if b["dtype"] == "bf16" else torch.float32
    N, Hd, Vd = b["N"], b["H"], b["V"]
    b["hidden"] = torch.randn((N, Hd), generator=gen, device=device, dtype=torch.float32).to(dt)
    W = torch.empty((Vd, Hd), device=device, dtype=dt)
    rows = 16384
    for v0 in range(0, Vd, rows):
        v1 = min(Vd, v0 + rows)
        W[v0:v1] = (torch.randn((v1 - v0, Hd), generator=gen, device=device, dtype=torch.float32) * W_STD).to(dt)
    b["W"] = W
    b["ids"] = torch.randint(0, Vd, (N,), generator=gen, device=device, dtype=torch.int32)
    b["logp_noise"] = torch.randn((N,), generator=gen, device=device, dtype=torch.float32) * LOGP_NOISE_STD
    return b


# ---- inputs of the widened selection stage: cut-length schedules, per-token
# ---- inclusion probabilities, prompt lengths (random draws only; what they mean
# ---- is the selection code's business)

def draw_schedule_weights(lengths, kind, seed, C=100):
    """Packed uint32 weights a_{i,l}, one per response position.

    kind: "uniform"   all ones;
          "min_cut"   zero below position C, one from C on (zero-length prefix when C > T);
          "tail_mass" ones, plus a point mass of T_i // 2 on the last position
                      (the survival function stays above 1/3);
          "random"    32-bit random values with ~25 % zeros, the last one forced positive;
          "sparse"    all zero except three random positions and the last one.
    """
    rng = np.random.default_rng([seed, 7])
    out = []
    for T in np.asarray(lengths, dtype=np.int64):
        T = int(T)
        if kind == "uniform":
            a = np.ones(T, dtype=np.uint32)
        elif kind == "min_cut":
            a = np.ones(T, dtype=np.uint32)
            a[:min(max(C - 1, 0), max(T - 1, 0))] = 0
        elif kind == "tail_mass":
            a = np.ones(T, dtype=np.uint32)
            if T:
                a[-1] += T // 2
        elif kind == "random":
            a = rng.integers(0, 2 ** 32, T, dtype=np.uint64).astype(np.uint32)
            a[rng.random(T) < 0.25] = 0
            if T:
                a[-1] |= 1
        elif kind == "sparse":
            a = np.zeros(T, dtype=np.uint32)
            if T:
                a[rng.integers(0, T, 3)] = rng.integers(1, 1000, 3)
                a[-1] = 5
        else:
            raise ValueError(kind)
        out.append(a)
    return np.concatenate(out) if out else np.zeros(0, np.uint32)


def draw_inclusion_probs(N, seed, floor=0.05):
    """Per-token probabilities in [floor, 1] (fp64): a stand-in for an information-aware
    score (e.g. normalised token entropy); ~10 % of tokens sit at exactly 1."""
    rng = np.random.default_rng([seed, 8])
    pi = floor + (1.0 - floor) * rng.random(N) ** 2
    pi[rng.random(N) < 0.1] = 1.0
    return pi


def draw_prompt_lengths(B, seed, lo=32, hi=512):
    """Prompt lengths P_i (int32) for B rollouts; rollouts of one prompt would share it, which
    changes nothing for the packing code, so they are drawn independently."""
    return np.random.default_rng([seed, 9]).integers(lo, hi + 1, B).astype(np.int32)
