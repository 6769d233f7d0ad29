#!/usr/bin/env python3
"""Benchmark of the partial-token GRPO loss stage on one MI355X.

One step = one pass of the whole hot path over one synthetic batch that is
already resident in HBM: nat_advantage -> nat_select -> nat_compact (with the
gather of kept rows) -> nat_loss_fwd_bwd.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--scheme rpc|urs|full|det]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
METRIC = "kept tokens/sec fused fwd+bwd at Qwen3-8B head shape; MFMA util % of bf16 peak"
GEMM_CLASSES = ("logits_gemm", "dhidden_gemm", "dweight_gemm")

# L2-miss traffic per launch (bytes, average over the launches of one default step) from two
# rocprofv3 --pmc runs of this file (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each scaled by
# what the same counter reads for the library's row-gather copy kernel of known size
# (factors 2.000 and 1.000; see profiles/).  Valid only for the kernel source they were taken
# on: bench.py reports null when the source hash differs.
TRAFFIC_SOURCE_SHA256_16 = "461c8f15aced70c5"
TRAFFIC_BYTES_PER_LAUNCH = {
    "logits_gemm": 16826311490 + 2456013870,
    "dhidden_gemm": 14593432430 + 69123641,
    "dweight_gemm": 34087232460 + 2548301824,
}


def measured_traffic(kernel, workload):
    import hashlib
    src = os.path.join(ROOT, "paper_2603_06619_amd", "csrc", "loss_bf16.hip")
    try:
        h = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if h != TRAFFIC_SOURCE_SHA256_16 or workload != "qwen3_8b_head_rpc":
        return None
    return TRAFFIC_BYTES_PER_LAUNCH.get(kernel)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="qwen3_8b_head_rpc")
    ap.add_argument("--scheme", default=None,
                    help="rpc | urs | full | det | schedule | poisson | mixed (even prompts URS, odd prompts Det.Trunc. 50%%); "
                         "default: the workload's own")
    ap.add_argument("--p", type=float, default=0.5)
    ap.add_argument("--min-cut", type=int, default=None, help="RPC minimum cutoff C (default 1; 100 for the "
                                                              "Qwen2.5-Math-7B head workload, as in the paper)")
    ap.add_argument("--drop-zero-adv", action="store_true",
                    help="rollouts with advantage exactly 0 keep nothing (exact when the loss has no KL term)")
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-single-thread-tokens", type=int, default=24,
                    help="kept tokens of the single-thread oracle timing (about 0.3 s each at the 8B head)")
    ap.add_argument("--kl-beta", type=float, default=0.0,
                    help="weight of the KL term of the token loss (reference log-probs are synthetic); 0 = off")
    ap.add_argument("--entropy", action="store_true", help="also accumulate the per-token entropy in the sweep")
    ap.add_argument("--logp-noise-scale", type=float, default=1.0,
                    help="multiplies the N(0, 0.05) noise of the behaviour log-probs (4 puts ~1/3 of the tokens on the "
                         "clipped branch at eps = 0.2)")
    ap.add_argument("--forward-only", action="store_true",
                    help="time nat_logp_fwd (log-probs of the kept tokens, 2VH flops per token) instead of the loss")
    ap.add_argument("--prefix-pack", action="store_true",
                    help="also build the truncated batch (prompt + kept prefix) each step; prefix schemes only")
    ap.add_argument("--prompts", type=int, default=None, help="override the number of prompts (smaller batch)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the loss benchmark: the practical ceilings on this GPU (HBM copy, matrix cores "
                         "with operands in registers, the vendor GEMM on the three contraction shapes of --workload)")
    ap.add_argument("--copy-probe-gib", type=int, default=0,
                    help="launch the library's plain copy kernel once on this many GiB before the timed region: a kernel "
                         "of known size next to the path's kernels in a counter run (scales FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--chunk-tokens", type=int, default=0,
                    help="cap the loss call's workspace so that it works in chunks of at most this many kept tokens "
                         "(a multiple of 256; 0 = the library's recommended workspace)")
    ap.add_argument("--stress-select", type=int, default=0, metavar="LOG2_TOKENS",
                    help="instead of the loss benchmark: time nat_select / nat_compact alone on 2^LOG2_TOKENS tokens")
    return ap.parse_args()


def cpu_baseline(batch, old_logp, scheme_code, args, torch):
    """The fp64 oracle, timed on the host on a bounded sample of the same batch: the first
    rollouts, each truncated to at most 256 tokens, through select -> compact -> loss."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import grpo as ogrpo
    from oracle import select as osel

    max_rollouts, max_len = 8, 256
    cu_full = batch["cu_seqlens"]
    rows, lens = [], []
    # the equal-reward prompts come first in the batch: with --drop-zero-adv sample the last rollouts instead
    n_s = min(max_rollouts, batch["B"])
    chosen = list(range(batch["B"] - n_s, batch["B"])) if args.drop_zero_adv else list(range(n_s))
    for i in chosen:
        T = int(min(max_len, cu_full[i + 1] - cu_full[i]))
        rows.append(np.arange(cu_full[i], cu_full[i] + T))
        lens.append(T)
    rows = np.concatenate(rows)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ridx = torch.from_numpy(rows).to(batch["hidden"].device)
    hidden = batch["hidden"][ridx].float().cpu().numpy()
    ids = batch["ids"][ridx].cpu().numpy()
    old = old_logp[ridx].cpu().numpy()
    W = batch["W"].float().cpu().numpy()
    R = batch["rewards"]
    t0 = time.perf_counter()
    adv = ogrpo.advantages(R).reshape(-1)[chosen]
    spr = None
    if args.scheme_name == "mixed":
        spr = np.array([osel.URS if (i // batch["G"]) % 2 == 0 else osel.DET for i in chosen])
    d = osel.select(cu, scheme_code, p=args.p, C=args.min_cut, beta=0.5, seed=args.seed, step=0, scheme_per_rollout=spr,
                    drop_zero_adv=adv if args.drop_zero_adv else None)
    c = osel.compact(d["mask"], cu, len(lens), scheme_code, p=args.p, C=args.min_cut, scheme_per_rollout=spr)
    k = c["kept_idx"]
    out = ogrpo.loss_and_grads(hidden[k], W, ids[k], old[k], adv[c["kept_seq"]], c["kept_w"].astype(np.float64))
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    # the same oracle call on one thread, on the first kept tokens of the sample
    from threadpoolctl import threadpool_limits
    k1 = k[:max(1, min(len(k), args.cpu_single_thread_tokens))]
    with threadpool_limits(limits=1):
        t1 = time.perf_counter()
        ogrpo.loss_and_grads(hidden[k1], W, ids[k1], old[k1], adv[c["kept_seq"][:len(k1)]],
                             c["kept_w"][:len(k1)].astype(np.float64))
        dt1 = time.perf_counter() - t1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return dict(value=c["n_kept"] / dt, unit="kept tokens/s", cores=int(threads), kind="oracle",
                sample=f"{'last' if args.drop_zero_adv else 'first'} {len(lens)} rollouts truncated to <= {max_len} tokens ({int(cu[-1])} tokens, "
                       f"{c['n_kept']} kept) at the full head shape, fp64 numpy, {dt:.1f} s",
                nproc=int(os.cpu_count() or 0), usable_cpus=int(usable or 0), blas_threads=int(threads),
                single_thread_value=len(k1) / dt1,
                single_thread_sample=f"the first {len(k1)} kept tokens of that sample, loss and gradients only, "
                                     f"BLAS limited to one thread, {dt1:.1f} s",
                loss=out["loss"])


def stress_select(args):
    """HBM-side measurement of the selection kernels on an inflated batch (they are launch-latency
    bound at the real workloads): algorithmic bytes = N/8 mask bytes written by nat_select;
    N/8 read + 12 bytes written per kept token by nat_compact."""
    import numpy as np
    import torch
    import paper_2603_06619_amd as nat
    dev = "cuda:0"
    N = 1 << args.stress_select
    B = 4096
    rng = np.random.default_rng(1)
    cuts = np.sort(rng.choice(np.arange(1, N), size=B - 1, replace=False))
    cu = torch.from_numpy(np.concatenate([[0], cuts, [N]]).astype(np.int64)).to(dev)
    out = {}
    cut_len = torch.empty(B, dtype=torch.int32, device=dev)
    mask = torch.empty(nat.mask_words(N), dtype=torch.int32, device=dev)
    kept_idx = torch.empty(N, dtype=torch.int32, device=dev)
    kept_seq = torch.empty(N, dtype=torch.int32, device=dev)
    kept_w = torch.empty(N, dtype=torch.float32, device=dev)
    cu_kept = torch.empty(B + 1, dtype=torch.int32, device=dev)
    n_kept = torch.empty(1, dtype=torch.int32, device=dev)
    ws = torch.empty(nat.compact_workspace_bytes(N), dtype=torch.uint8, device=dev)
    src = torch.empty(N, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(reps):
            a, b = ev(), ev()
            a.record(); fn(); b.record(); torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b))
        return best

    copy_ms = timed(lambda: dst.copy_(src))
    out["copy_GBps"] = 2 * 4 * N / copy_ms / 1e6
    for name, code, kw in (("urs", nat.URS, dict(p=0.5)), ("rpc", nat.RPC, dict(min_cut=1))):
        params = nat.SelectParams(code, seed=3, **kw)
        sel_ms = timed(lambda: nat.nat_select(params, cu, B, N, cut_len, mask))
        cmp_ms = timed(lambda: nat.nat_compact(params, B, mask, cu, B, N, kept_idx, kept_seq, kept_w, cu_kept, n_kept,
                                               None, ws))
        nk = int(n_kept.item())
        out[name] = dict(tokens=N, kept=nk, select_ms=sel_ms, compact_ms=cmp_ms,
                         select_GBps=(N / 8) / sel_ms / 1e6, compact_GBps=(N / 8 + 12.0 * nk) / cmp_ms / 1e6,
                         select_Gtok_per_s=N / sel_ms / 1e6, compact_Gtok_per_s=N / cmp_ms / 1e6)
    # widened selection stage: cut schedules (4 B read + 8 B written per token + mask), Poisson sampling
    # (8 B read per token + mask), weights from probabilities, prefix packing (8 B per row + 4 B per kept token)
    pi = torch.empty(N, dtype=torch.float64, device=dev)
    weights = torch.ones(N, dtype=torch.int32, device=dev)
    params = nat.SelectParams(nat.FULL, seed=3)
    sch_ms = timed(lambda: nat.nat_select_schedule(params, weights, cu, B, N, cut_len, mask, pi))
    cmp_ms = timed(lambda: nat.nat_compact_pi(B, mask, pi, cu, B, N, kept_idx, kept_seq, kept_w, cu_kept, n_kept,
                                              None, ws))
    nk = int(n_kept.item())
    out["schedule"] = dict(tokens=N, kept=nk, select_ms=sch_ms, compact_ms=cmp_ms,
                           select_GBps=(12.125 * N) / sch_ms / 1e6,
                           compact_GBps=(N / 8 + 20.0 * nk) / cmp_ms / 1e6)
    cu_packed, cu_loss, totals = (torch.empty(n, dtype=torch.int32, device=dev) for n in (B + 1, B + 1, 2))
    pack_ms = timed(lambda: nat.nat_prefix_pack(None, cu, cut_len, B, 0, N, N, cu_packed, cu_loss, kept_idx, kept_seq,
                                                src, totals, None))
    rows = int(totals[0].item())
    out["prefix_pack"] = dict(rows=rows, ms=pack_ms, GBps=12.0 * rows / pack_ms / 1e6)
    pi.uniform_(0.05, 1.0)
    poi_ms = timed(lambda: nat.nat_select_poisson(params, pi, cu, B, N, mask))
    out["poisson"] = dict(tokens=N, select_ms=poi_ms, select_GBps=(8.125 * N) / poi_ms / 1e6)
    print(json.dumps({"metric": "nat_select / nat_compact on an inflated batch", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": f"2^{args.stress_select} tokens in {B} rollouts"}, **out}))


def ceilings(args):
    """What bounds the loss stage's kernels on this GPU, measured with kernels of known work: an HBM copy,
    the matrix cores on operands held in registers (constant, then pseudo-random bits: the chip is power
    limited, so the rate depends on the data), and the vendor's GEMM (torch.matmul) on the three
    contraction shapes of the workload's head with one full token chunk.  The vendor GEMM is a stated
    ceiling only: nothing on the product path calls it."""
    import torch
    import synth_inputs as si
    import paper_2603_06619_amd as nat
    dev = "cuda:0"
    torch.cuda.set_device(0)
    nat.load_library()
    cfg = si.WORKLOADS[args.workload]
    H, V, chunk = cfg["H"], cfg["V"], 16384        # the library's chunk with the recommended workspace at these heads

    def timed_ms(fn, reps, warm=1):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    out = {}
    nbytes = 4 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    ms = timed_ms(lambda: nat.nat_probe_copy(dst, src, nbytes), 10)
    out["hbm_copy"] = dict(bytes_each_way=nbytes, ms=ms, GBps=2.0 * nbytes / ms / 1e6, frac_of_8TBps=2.0 * nbytes / ms / 1e6 / 8000.0)
    del src, dst
    scratch = torch.empty(nat.probe_mfma_scratch_bytes() // 4, dtype=torch.float32, device=dev)
    for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
        flops = [0.0]
        def launch():
            flops[0] = nat.nat_probe_mfma_bf16(rnd, 40000, scratch)
        ms = timed_ms(launch, 6)                      # ~70 ms per launch, ~0.4 s sustained
        out["mfma_only_" + label] = dict(ms_per_launch=ms, TFLOPs=flops[0] / ms / 1e9,
                                         frac_of_peak=flops[0] / ms / 1e9 / PEAK_BF16_TFLOPS)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    rnd_bf16 = lambda r, c, std: (torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)
    Wm, Hm = rnd_bf16(V, H, si.W_STD), rnd_bf16(chunk, H, 1.0)
    E = rnd_bf16(chunk, V, 1.0).abs_()                 # soft-max numerators are positive
    shapes = {"logits (W . H_chunk^T)": lambda: torch.matmul(Wm, Hm.t()),
              "dH (E . W)": lambda: torch.matmul(E, Wm),
              "dW (E^T . H_chunk)": lambda: torch.matmul(E.t(), Hm)}
    vend = {}
    for name, fn in shapes.items():
        ms = timed_ms(fn, 8, warm=2)
        vend[name] = dict(ms=ms, TFLOPs=2.0 * V * H * chunk / ms / 1e9, frac_of_peak=2.0 * V * H * chunk / ms / 1e9 / PEAK_BF16_TFLOPS)
    out["vendor_gemm_bf16"] = vend
    print(json.dumps({"metric": "practical ceilings for the loss stage's kernels", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": args.workload, "H": H, "V": V, "chunk_tokens": chunk},
                      "peak_bf16_TFLOPs": PEAK_BF16_TFLOPS, "peak_hbm_GBps": 8000.0, **out}))


def main():
    args = parse_args()
    if args.gpus != 1 and (args.stress_select or args.ceilings):
        sys.exit(2)
    if args.ceilings:
        return ceilings(args)
    if args.stress_select:
        return stress_select(args)
    if args.gpus != 1:
        print(f"bench.py measures one GPU only (got --gpus {args.gpus}): no multi-GPU path is built; the stage "
              "shards by rollout (each GPU holds the head, one sum of dW and the loss at the end)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2603_06619_amd as nat
    from paper_2603_06619_amd.stage import LossStage

    if not os.path.exists(nat.library_path()):
        from paper_2603_06619_amd import build
        build.build()
    nat.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stage = LossStage(dev)

    default_scheme = {"qwen3_8b_head_rpc": "rpc", "qwen3_0p6b_head": "urs", "qwen3_8b_long_cot": "urs",
                      "wide_head_stress": "mixed", "tiny_fp32": "urs", "qwen2p5_math_7b_head": "rpc"}[args.workload]
    if args.min_cut is None:
        args.min_cut = 100 if args.workload == "qwen2p5_math_7b_head" else 1
    scheme_name = args.scheme or default_scheme
    scheme_code = dict(full=nat.FULL, urs=nat.URS, rpc=nat.RPC, det=nat.DET, mixed=nat.URS,
                       schedule=nat.FULL, poisson=nat.FULL)[scheme_name]

    args.scheme_name = scheme_name
    batch = si.make_batch_torch(args.workload, args.seed, dev, P=args.prompts)
    P, G, B, N, H, V = batch["P"], batch["G"], batch["B"], batch["N"], batch["H"], batch["V"]
    # behaviour-policy log-probs: the current policy's (forward pass alone over every token) plus N(0, 0.05)
    old_logp = stage.logp(batch["hidden"], batch["W"], batch["ids"], N)["logp"][:N] + batch["logp_noise"] * args.logp_noise_scale
    torch.cuda.synchronize()
    rewards = torch.from_numpy(batch["rewards"].reshape(-1)).to(dev)
    cu = torch.from_numpy(batch["cu_seqlens"]).to(dev)
    spr = None
    if scheme_name == "mixed":
        spr = torch.tensor([nat.URS if (i // G) % 2 == 0 else nat.DET for i in range(B)], dtype=torch.int32, device=dev)
    params = nat.SelectParams(scheme_code, p=args.p, min_cut=args.min_cut, trunc_frac=0.5, seed=args.seed, step=0,
                              scheme_per_rollout=spr)
    dW = torch.empty((V, H), dtype=torch.float32, device=dev)
    dtype_code = nat.DTYPE_BF16 if batch["dtype"] == "bf16" else nat.DTYPE_F32

    # widened selection: a cut-length schedule with a point mass on the full length (survival >= 1/3), or
    # token-dependent inclusion probabilities; optionally the truncated batch for the model body
    sched_w = poisson_pi = prompt_len = None
    if scheme_name == "schedule":
        sched_w = torch.from_numpy(si.draw_schedule_weights(batch["lengths"], "tail_mass", args.seed).view(np.int32)).to(dev)
    if scheme_name == "poisson":
        poisson_pi = torch.from_numpy(si.draw_inclusion_probs(N, args.seed)).to(dev)
    if args.prefix_pack:
        plen = si.draw_prompt_lengths(B, args.seed)
        prompt_len, rows_cap = torch.from_numpy(plen).to(dev), int(plen.sum()) + N

    def step(step_no):
        params.step = step_no
        adv = stage.advantage(rewards, P, G)
        params.drop_zero_adv = adv if args.drop_zero_adv else None
        sc = stage.select_compact(params, cu, B, N, hidden=batch["hidden"], ids=batch["ids"], old_logp=old_logp,
                                  schedule_weights=sched_w, poisson_pi=poisson_pi)
        if args.prefix_pack:
            stage.prefix_pack(prompt_len, cu, sc["cut_len"], B, N, rows_cap, 1)
        nk = sc["n_kept"]
        if args.forward_only:
            return nk, stage.logp(sc["hidden_k"], batch["W"], sc["ids_k"], nk, want_entropy=args.entropy)
        kl = {}
        if args.kl_beta > 0 or args.entropy:
            # reference log-probs: the behaviour log-probs stand in (only their shape matters for the timing)
            kl = dict(ref_logp_k=sc["old_logp_k"], beta_kl=args.kl_beta, kl_kind=nat.KL_NONNEG,
                      want_kl=args.kl_beta > 0, want_entropy=args.entropy)
        ws_bytes = None
        if args.chunk_tokens:
            ws_bytes = nat.loss_workspace_bytes(args.chunk_tokens, H, V, dtype_code) + 4 * max(nk, 1) + 4096
        out = stage.loss(sc["hidden_k"], batch["W"], sc["ids_k"], sc["old_logp_k"], adv, sc["kept_seq"], sc["kept_w"],
                         nk, dW=dW, want_logp=True, ws_bytes=ws_bytes, **kl)
        return nk, out

    for w in range(args.warmup):
        step(w)
    torch.cuda.synchronize()
    if args.copy_probe_gib:
        nbytes = args.copy_probe_gib << 30
        src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        nat.nat_probe_copy(dst, src, nbytes)
        torch.cuda.synchronize()
        del src, dst
    nat.profile_collect()
    nat.profile_enable(True)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kept_total = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for s in range(args.steps):
        nk, out = step(args.warmup + s)
        kept_total += nk
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    nat.profile_enable(False)
    prof = nat.profile_collect()
    ms_total = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / args.steps
    value = kept_total / wall

    # roofline of the dominant kernel: algorithmic flops = 2*V*H per kept token for each of the
    # three contractions; every kept token passes through each GEMM class exactly once per step
    flops_per_class = 2.0 * V * H * kept_total
    dom = max(GEMM_CLASSES, key=lambda c: prof[c][0]) if dtype_code == nat.DTYPE_BF16 else "f32_path"
    dom_ms, dom_launches = prof[dom]
    if dtype_code == nat.DTYPE_BF16:
        achieved = flops_per_class / (dom_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", kernel=dom, achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=achieved / PEAK_BF16_TFLOPS, traffic=measured_traffic(dom, args.workload),
                        avg_launch_ms=dom_ms / max(dom_launches, 1), launches=int(dom_launches))
    else:
        achieved = 3 * flops_per_class / (dom_ms * 1e-3) / 1e12
        roofline = dict(bound="alu", kernel=dom, achieved=achieved, peak=157.3, unit="TFLOP/s",
                        frac=achieved / 157.3, traffic=None, avg_launch_ms=dom_ms / max(dom_launches, 1),
                        launches=int(dom_launches))
    kernels = {k: dict(ms_per_step=v[0] / args.steps, launches_per_step=v[1] / args.steps)
               for k, v in prof.items() if v[1] > 0}
    gemm_ms = sum(prof[c][0] for c in GEMM_CLASSES)
    n_gemms = 1.0 if args.forward_only else 3.0                    # contractions per kept token
    useful_tflops = 2.0 * n_gemms * V * H * kept_total / wall / 1e12

    result = {
        "metric": METRIC, "value": value, "unit": "kept tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": batch["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "P": P, "G": G, "H": H, "V": V, "tokens": N,
                   "kept_tokens_per_step": kept_total / args.steps, "scheme": scheme_name,
                   "p": args.p if scheme_name == "urs" else None, "min_cut": args.min_cut if scheme_name == "rpc" else None,
                   "kl_beta": args.kl_beta, "entropy": bool(args.entropy),
                   "drop_zero_adv": bool(args.drop_zero_adv),
                   "forward_only": bool(args.forward_only), "logp_noise_scale": args.logp_noise_scale,
                   "chunk_tokens": args.chunk_tokens or None,
                   "loss_workspace_gb": (nat.loss_workspace_bytes(args.chunk_tokens or int(kept_total / args.steps), H, V, dtype_code) / 1e9)},
        "mfma_util_pct_useful_6VH": 100.0 * useful_tflops / PEAK_BF16_TFLOPS,
        "mfma_util_pct_gemm_kernels_only": (100.0 * 2.0 * n_gemms * V * H * kept_total / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
                                            if gemm_ms > 0 else None),
        "gpu_event_ms_per_step": ms_total / args.steps,
        "loss": None if args.forward_only else float(out["loss"].item()),
        "peak_hbm_gb": torch.cuda.max_memory_allocated() / 1e9,
        "roofline": roofline,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline and scheme_name not in ("schedule", "poisson") and not args.forward_only:
        result["cpu_baseline"] = cpu_baseline(batch, old_logp, scheme_code, args, torch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
