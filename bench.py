#!/usr/bin/env python3
"""Benchmark of the SSD pre-speculation hot path on one MI355X.

One "step" = one whole SSD round on the draft side: the pre-speculation round (glue extend, top-F fan-out,
K batched branch-decode steps writing the speculation cache) on one HIP stream, the lossless verification
kernel on a second stream at the same time, then the cache lookup of the realised outcome.  The workload is
the Llama-3.2-1B-shaped bf16 draft with a 1024-token shared prefix, K=5, F=4 (24 branch rows), greedy, on
seeded synthetic weights / prefix KV / logits already resident in HBM.

Prints ONE JSON line: whole-job pre-speculated branch-tokens/s, ms per round, the HBM roofline of the dominant
kernel (the batched branch-decode step) measured with HIP events on its own stream, and the CPU oracle timed on a
bounded sample of the same workload (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MEASURED_STREAM_READ_GBS = 7100.0     # register-ring streaming read of 2 GiB, 256 workgroups x 8 wavefronts
WORKLOAD = "1b_p1024_f4"
WEIGHT_SEED = 2025
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "fused_decode_kernel_1b_p1024_f4_hbm_traffic.txt")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2603_03251_amd", "csrc", f) for f in ("kernels_fused.hip", "fused.h")]


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for path in KERNEL_SOURCES:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic_bytes():
    """HBM bytes per launch of the fused decode kernel from the rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, each
    scaled by a plain copy) summarised in the tracked profile, or None if that summary was taken with other kernel
    sources than the ones this run was built from (it names their hash)."""
    try:
        fields = {}
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                if ":" in line and line.split(":", 1)[0].strip() in ("traffic_bytes_per_launch", "kernel_sources_sha256"):
                    k, v = line.split(":", 1)
                    fields[k.strip()] = v.strip()
        if fields.get("kernel_sources_sha256") != kernel_source_hash():
            return None
        return int(fields["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def algorithmic_bytes_per_decode_step(shape, rnd, prefix_lens=None):
    """Bytes one batched branch-decode step must move: every weight once, the shared trunk KV once per
    sequence (not once per branch), the fp32 logits it has to keep, and the branch-private suffix KV."""
    d, f, V, L = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers
    qd, kvd = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    weights = (L * ((qd + 2 * kvd) * d + d * qd + 3 * d * f) + V * d) * 2
    positions = rnd.batch * rnd.prefix if prefix_lens is None else sum(prefix_lens)
    trunk = L * (positions + rnd.batch * (rnd.K + 1)) * 2 * kvd * 2
    logits = rnd.rows * V * 4
    suffix = rnd.rows * L * rnd.K * 2 * kvd * 2
    return weights + trunk + logits + suffix


def print_phase_clocks(B, ctx, one_round, shape):
    """Per-phase wall times inside the persistent kernel (last branch-decode step of one more round), from the
    100 MHz clocks every workgroup records at phase entry / after the grid barrier / at the end of its work."""
    import numpy as np
    B.ssd_ctx_enable_phase_clocks(ctx, True)
    one_round(3000)
    t = B.ssd_ctx_read_phase_clocks(ctx).astype(np.int64)
    B.ssd_ctx_enable_phase_clocks(ctx, False)
    L = shape.n_layers
    w = sys.stderr.write
    if B.ssd_ctx_views(ctx).pass_rows > 48:
        # wide passes: every phase is a launch of its own; slots 0 entry, 3 operands of the first stage requested,
        # 4 last MFMA of the first pair, 2 end (the attention kernel records entry and end only)
        w("phase clocks of one wide decode step (us after the phase's first workgroup entered; mean over layers of the mean / "
          "slowest workgroup)\n")
        names = {0: "qkv", 1: "attention", 2: "merge of key splits", 3: "o-proj", 4: "gate/up", 5: "down"}
        for sub, name in names.items():
            rows = []
            for l in range(L):
                x = t[1 + 6 * l + sub] / 100.0
                busy = x[2] > 0
                if not busy.any():
                    continue
                t0 = x[0][x[0] > 0].min()
                rows.append([(x[s_][busy] - t0).mean() if (x[s_][busy] > 0).all() else np.nan for s_ in (3, 4, 2)]
                            + [(x[2][busy] - t0).max(), busy.sum()])
            if rows:
                a_ = np.array(rows, dtype=np.float64)
                r_ = [a_[:, i][~np.isnan(a_[:, i])].mean() if (~np.isnan(a_[:, i])).any() else None for i in range(5)]
                f_ = lambda v: "    -" if v is None else f"{v:5.1f}"
                w(f"  {name:19s} workgroups {int(r_[4]):3d}  first operands requested {f_(r_[0])}  MFMAs done {f_(r_[1])}  "
                  f"end {f_(r_[2])}  slowest {f_(r_[3])}\n")
        return
    us = (t - t[0, 0].min()) / 100.0
    entry, after, end = us[:, 0], us[:, 1], us[:, 2]
    names = ["qkv", "attention", "merge of key splits", "o-proj", "gate/up", "down"]
    done = end.max(axis=1)
    w("phase clocks of one fused decode kernel (us; mean over layers; per workgroup: wait = barrier wait, body = work)\n")
    w(f"kernel span {end[-1].max() - entry[0].min():.1f}; embedding {done[0] - entry[0].min():.1f}; "
      f"per layer {(done[6 * L] - done[0]) / L:.2f}; LM head {done[-1] - done[6 * L]:.1f}\n")
    for s_ in range(6):
        ph = [1 + 6 * l + s_ for l in range(L)]
        if (t[ph, 2] == 0).all():                         # the merge phase does not exist with one key split
            continue
        # (a workgroup that does not wait in a phase records no "after": its work starts at entry.  That is the case in
        # the attention phase, where only workgroups with a unit wait, for the qkv units of their KV head's group)
        aft = [np.where(t[p_, 1] > 0, after[p_], entry[p_]) for p_ in ph]
        wait = np.mean([(a_ - entry[p_]).mean() for a_, p_ in zip(aft, ph)])
        body_mean = np.mean([(end[p_] - a_).mean() for a_, p_ in zip(aft, ph)])
        body_max = np.mean([(end[p_] - a_).max() for a_, p_ in zip(aft, ph)])
        w(f"  {names[s_]:19s} wait {wait:6.2f}  body mean {body_mean:6.2f}  body max {body_max:6.2f}\n")


def algorithmic_bytes_target_forward(shape, prefix, T):
    """Bytes one verification forward of the target must move: every weight once (the embedding is gathered, the LM
    head is a matrix of its own here), the trunk KV once, the fp32 logits of the T positions."""
    d, f, V, L = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers
    qd, kvd = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    weights = (L * ((qd + 2 * kvd) * d + d * qd + 3 * d * f) + V * d) * 2
    return weights + L * (prefix + T) * 2 * kvd * 2 + T * V * 4


def bench_target_verify(args):
    """Workload 70b_verify_1b_draft (Sec. 2.1: verification is one target forward over the K+1 positions; Sec. 4 "Setup"): the target's verification forward over the K+1 pending
    positions at the 70B shape, alone and beside the draft's pre-speculation round, both on this one GPU (so the two
    share one HBM: this shows the overlap mechanics and the target forward's own rate, not the paper's two-device
    latency hiding).  The target's 80 layers of random weights and its prefix KV are generated on the device.  Prints
    one JSON line; not the default bench line."""
    import numpy as np
    import torch
    import ssd_inputs as I
    from paper_2603_03251_amd import binding as B

    wl = I.WORKLOADS["70b_verify_1b_draft"]
    dshape, tshape, r = wl.draft, wl.target, wl.round
    K, F, P, nb = r.K, r.F, r.prefix, r.batch
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    to_bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    note = lambda m: (sys.stderr.write(m + "\n"), sys.stderr.flush())

    # 80 distinct random layers (139 GB of weights) and the synthetic prefix, generated on the device: no host copy
    target = B.ssd_model_create_random(tshape, WEIGHT_SEED + 1)
    note("target model generated on the device")
    tctx = B.ssd_ctx_create(target, nb, K, 1, P + 2 * K + 2)
    B.ssd_ctx_fill_synthetic_kv(tctx, [P] * nb, wl.seed + 7)
    draft = B.ssd_model_create(dshape, I.make_weights(dshape, WEIGHT_SEED))
    dctx = B.ssd_ctx_create(draft, nb, K, F, P + 2 * K + 2)
    kd, vd = I.make_prefix_kv(dshape, nb, P, wl.seed)
    B.ssd_ctx_load_trunk(dctx, to_bf16(kd), to_bf16(vd), P)
    del kd, vd
    note("draft model and both trunks on the device")

    V = tshape.vocab
    pending = dev(I.make_pending(dshape, nb, K, wl.seed), np.int32)
    pending_spec = pending[:, 1:].contiguous()
    temps = dev(np.full(nb, r.temperature), np.float32)
    zt = torch.empty((nb, K + 1, V), dtype=torch.float32, device="cuda")
    zd = dev(I.make_logits(nb * K, V, wl.seed + 2).reshape(nb, K, V), np.float32)   # stands in for last round's draft logits
    k_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    t_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
    hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
    spec = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
    s_draft, s_target = torch.cuda.Stream(), torch.cuda.Stream()
    verified = torch.cuda.Event()

    def target_side(seed):
        B.ssd_ctx_extend(tctx, pending, 0, zt, stream=s_target)
        B.ssd_verify(zt, zd, pending_spec, temps, seed, k_out, t_out, ws, stream=s_target)
        verified.record(s_target)

    def draft_side(seed):
        B.ssd_prespeculate(dctx, pending, temps, seed, stream=s_draft)

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(100 + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3

    def both(seed):
        target_side(seed)
        draft_side(seed)
        s_draft.wait_event(verified)
        B.ssd_cache_lookup(dctx, k_out, t_out, hit, branch, spec, stream=s_draft)

    for i in range(args.warmup):
        both(i)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(zt).all()), "target logits are not finite"
    n = max(1, args.steps)
    t_target = timed(target_side, n)
    t_draft = timed(draft_side, n)
    t_both = timed(both, n)
    bytes_t = algorithmic_bytes_target_forward(tshape, P, K + 1)
    achieved = bytes_t / (t_target * 1e-3) / 1e9
    out = {
        "metric": "us_per_ssd_round", "value": t_both * 1e3, "unit": "us", "n_gpus": 1, "steps": n, "warmup": args.warmup,
        "ms_per_step": t_both, "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "70b_verify_1b_draft: Llama-3.1-70B-shaped target verifies K+1=6 positions (prefix 4096) on one "
                               "stream while the Llama-3.2-1B-shaped draft pre-speculates (K=5, F=4) on another; both on one GPU"},
        "target_forward_plus_verify_ms": t_target, "draft_round_ms": t_draft, "concurrent_round_ms": t_both,
        "roofline": {"kernel": "target verification forward (per-operator kernels, 80 layers)", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_launch": bytes_t, "avg_ms": t_target},
    }
    print(json.dumps(out))
    B.ssd_ctx_destroy(tctx)
    B.ssd_ctx_destroy(dctx)
    B.ssd_model_destroy(target)
    B.ssd_model_destroy(draft)


def sub_record(B, I, model, shape, name, steps, flags=0):
    """Kernel time and roofline fraction of one branch-decode step of another workload (or another context
    configuration) of the same model: a few rounds on a context of its own, HIP events around the step's kernels on
    their stream."""
    import numpy as np
    import torch
    wl = I.WORKLOADS[name]
    r = wl.round
    K, F, P, nb, V = r.K, r.F, r.prefix, r.batch, shape.vocab
    ctx = B.ssd_ctx_create(model, nb, K, F, P + 2 * K + 2, flags)
    try:
        k, v = I.make_prefix_kv(shape, nb, P, wl.seed)
        to_bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
        B.ssd_ctx_load_trunk(ctx, to_bf16(k), to_bf16(v), P)
        del k, v
        pending = torch.from_numpy(I.make_pending(shape, nb, K, wl.seed)).cuda()
        temps = torch.full((nb,), r.temperature, dtype=torch.float32, device="cuda")
        B.ssd_ctx_enable_timing(ctx, True)
        seg = []
        for i in range(steps + 2):
            B.ssd_prespeculate(ctx, pending, temps, 3000 + i)
            if i >= 2:
                seg.append(B.ssd_ctx_read_timing(ctx, K, with_kernels=True))
        B.ssd_ctx_refresh_bounds(ctx)
        B.ssd_ctx_status(ctx)
        seg = np.array(seg)
        kernel_ms = float(seg[:, K + 2:].mean())
        round_ms = float(seg[:, :K + 2].sum(axis=1).mean())
        bytes_step = algorithmic_bytes_per_decode_step(shape, r)
        d_, f_, L_ = shape.d_model, shape.d_ffn, shape.n_layers
        qd_, kvd_ = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
        flops = 2.0 * r.rows * (L_ * ((qd_ + 2 * kvd_) * d_ + d_ * qd_ + 3 * d_ * f_) + V * d_)
        view = B.ssd_ctx_views(ctx)
        return {"branch_rows": r.rows, "pass_rows": int(view.pass_rows), "decode_step_kernels_ms": kernel_ms,
                "draft_round_ms": round_ms, "branch_tokens_per_s": r.rows * K / (round_ms * 1e-3),
                "hbm_frac": bytes_step / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_step": bytes_step,
                "mfma_frac": flops / (kernel_ms * 1e-3) / 2.5e15}
    finally:
        B.ssd_ctx_destroy(ctx)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and comparison (profiling runs)")
    ap.add_argument("--no-sub-records", action="store_true", help="skip the compact records of the other workloads")
    ap.add_argument("--phase-clocks", action="store_true",
                    help="also print (stderr) the per-phase times inside the fused decode kernel of the last branch step")
    ap.add_argument("--workload", default=WORKLOAD,
                    choices=[WORKLOAD, "1b_p8192_f8_t1", "1b_b16_p2048_f4", "70b_verify_1b_draft"],
                    help="default: the workload the headline metric is quoted on; the others print the same kind of line for "
                         "their shape (no CPU baseline, no counter traffic); 70b_verify_1b_draft: the target's verification "
                         "forward beside the draft round")
    ap.add_argument("--geometric-fanout", metavar="A,R", default=None,
                    help="spread the workload's (K+1) F branch rows over the accept lengths by the geometric cache shape for "
                         "acceptance rate A and power-law exponent R (e.g. 0.8,0.5) instead of F each")
    ap.add_argument("--ragged-prefix", action="store_true",
                    help="give every sequence of the batch its own prefix length (seeded, between a tenth of the workload's "
                         "prefix and all of it) instead of the same one")
    ap.add_argument("--one-plane", type=lambda x: int(x, 0), default=None, metavar="MASK",
                    help="activation tensors the narrow fused pass carries as ONE 16-bit plane instead of head + remainder: "
                         "bits 1 xn, 2 att, 4 act, 8 q, 16 p (0 = two planes everywhere, 31 = one everywhere; default: the "
                         "library's default configuration, 7)")
    ap.add_argument("--per-operator", action="store_true",
                    help="one kernel per operator instead of the fused passes (the path of models the fused passes do not take)")
    ap.add_argument("--paged", action="store_true",
                    help="keep the trunk KV in 32-position pages behind a block table (App. B) instead of one run per sequence")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy: the reference the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.workload == "70b_verify_1b_draft":
        bench_target_verify(args)
        return

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device copies of 1073741824 bytes (elementwise copy kernel)"}))
        return

    import ssd_inputs as I
    from paper_2603_03251_amd import binding as B

    headline = args.workload == WORKLOAD and not args.ragged_prefix and not args.geometric_fanout
    wl = I.WORKLOADS[args.workload]
    shape, r = wl.draft, wl.round
    K, F, P, nb, V = r.K, r.F, r.prefix, r.batch, shape.vocab
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()

    w = I.make_weights(shape, WEIGHT_SEED)
    model = B.ssd_model_create(shape, w)
    fan = None
    ctx_flags = 0 if args.one_plane is None else B.SSD_CTX_TWO_PLANES | (args.one_plane & 31) << 8
    if args.per_operator:
        ctx_flags |= B.SSD_CTX_PER_OPERATOR
    if args.geometric_fanout:
        a_rate, r_exp = (float(x) for x in args.geometric_fanout.split(","))
        fan = B.ssd_geometric_fanout((K + 1) * F, K, a_rate, r_exp)
        ctx = B.ssd_ctx_create_fanout(model, nb, K, fan, P + 2 * K + 2, ctx_flags)
    else:
        kv_pages = 1 + nb * ((P + 2 * K + 2 + 31) // 32 + 1) if args.paged else 0
        ctx = B.ssd_ctx_create(model, nb, K, F, P + 2 * K + 2, ctx_flags, kv_pages)
    k, v = I.make_prefix_kv(shape, nb, P, wl.seed)
    to_bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    B.ssd_ctx_load_trunk(ctx, to_bf16(k), to_bf16(v), P)
    prefix_lens = None
    if args.ragged_prefix:
        prefix_lens = [int(x) for x in np.random.default_rng(wl.seed).integers(P // 10, P + 1, nb)]
        B.ssd_ctx_truncate_trunk(ctx, prefix_lens)
    pending = dev(I.make_pending(shape, nb, K, wl.seed), np.int32)
    temps = dev(np.full(nb, r.temperature), np.float32)
    pending_spec = pending[:, 1:].contiguous()            # s_1..s_K, what the verifier checks
    # the verifier's inputs: target logits over the K+1 positions and the draft logits of the pending speculation
    zt = dev(I.make_logits(nb * (K + 1), V, wl.seed + 1).reshape(nb, K + 1, V), np.float32)
    zd = dev(I.make_logits(nb * K, V, wl.seed + 2).reshape(nb, K, V), np.float32)
    k_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    t_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
    hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
    spec = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
    s_draft, s_verify = torch.cuda.Stream(), torch.cuda.Stream()
    verified = torch.cuda.Event()
    torch.cuda.synchronize()

    def one_round(seed):
        B.ssd_verify(zt, zd, pending_spec, temps, seed, k_out, t_out, ws, stream=s_verify)
        verified.record(s_verify)
        B.ssd_prespeculate(ctx, pending, temps, seed, stream=s_draft)
        s_draft.wait_event(verified)
        B.ssd_cache_lookup(ctx, k_out, t_out, hit, branch, spec, stream=s_draft)

    B.ssd_ctx_enable_timing(ctx, True)
    for i in range(args.warmup):
        one_round(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_round(1000 + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # per-segment HIP-event times of the last round + a few extra rounds (the events are per-context)
    seg = []
    fused = True
    for i in range(min(max(args.steps, 1), 50)):
        one_round(2000 + i)
        try:
            seg.append(B.ssd_ctx_read_timing(ctx, K, with_kernels=fused))
        except B.SsdError:                                # per-operator kernels: step times only
            fused = False
            seg.append(B.ssd_ctx_read_timing(ctx, K))
    torch.cuda.synchronize()
    seg = np.array(seg)                                   # [rounds][2K+2] ms: glue, fan-out, K steps, K fused kernels
    step_ms = float(seg[:, 2:K + 2].mean())
    # the fused decode kernel alone, HIP events on its stream (the whole step if the per-operator kernels ran)
    kernel_ms = float(seg[:, K + 2:].mean()) if fused else step_ms
    if args.phase_clocks and fused:
        print_phase_clocks(B, ctx, one_round, shape)
    bytes_step = algorithmic_bytes_per_decode_step(shape, r, prefix_lens)
    achieved = bytes_step / (kernel_ms * 1e-3) / 1e9

    # ---- the line must not report a round that went wrong: the context's fault word (a grid barrier of the fused pass
    # that timed out), finite outputs, and a hit that returns the cached speculation
    B.ssd_ctx_refresh_bounds(ctx)
    B.ssd_ctx_status(ctx)
    view = B.ssd_ctx_views(ctx)
    rows_all = nb * (sum(fan) if fan else (K + 1) * F)
    gpu_keys = B.device_copy(view.d_keys, (rows_all,), torch.int32).cpu().numpy()
    gpu_toks = B.device_copy(view.d_tokens, (rows_all, K), torch.int32).cpu().numpy()
    assert gpu_keys.min() >= 0 and gpu_keys.max() < V and gpu_toks.min() >= 0 and gpu_toks.max() < V, "invalid token ids in the cache"
    probe_k = torch.zeros(nb, dtype=torch.int32, device="cuda")
    rps = rows_all // nb
    probe_t = torch.from_numpy(np.ascontiguousarray(gpu_keys.reshape(nb, rps)[:, 0])).cuda()       # outcome (k = 0, first key)
    B.ssd_cache_lookup(ctx, probe_k, probe_t, hit, branch, spec, stream=s_draft)
    torch.cuda.synchronize()
    assert bool(hit.all()) and np.array_equal(spec.cpu().numpy(), gpu_toks.reshape(nb, rps, K)[:, 0]), "lookup of a cached outcome failed"

    tokens_per_round = nb * (K + 1) * F * K
    ms_per_step = elapsed / args.steps * 1e3
    out = {
        "metric": "prespeculated_branch_tokens_per_s",
        "value": tokens_per_round / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "us_per_ssd_round": ms_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # bf16 model: weights, KV and the attention MFMAs; the linear layers of the fused passes multiply the same weight
        # values held as fp16 with fp16 activations (11 significant bits instead of 8); fp32 accumulation everywhere
        "dtype": "bf16", "linear_layer_mfma_dtype": "f16" if fused else "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: Llama-3.2-1B-shaped bf16 draft, B={nb}, prefix {P}, K={K}, F={F} "
                               f"({r.rows} branch rows), lookahead {K}, {'greedy' if r.temperature == 0 else 'temperature %g' % r.temperature}"
                               f"; verify on a second stream; lookup"
                               + (f"; prefix lengths {min(prefix_lens)}..{max(prefix_lens)}, mean {sum(prefix_lens) // nb}" if prefix_lens else "")
                               + (f"; geometric fan-out {fan}" if fan else "")
                               + ("; trunk KV in 32-position pages" if args.paged else ""),
                   "branch_rows": r.rows, "tokens_per_round": tokens_per_round},
        "segments_ms": {"glue_extend": float(seg[:, 0].mean()), "fan_out": float(seg[:, 1].mean()),
                        "branch_decode_step": step_ms, "decode_steps_total": float(seg[:, 2:K + 2].sum(axis=1).mean())},
        "decode_only_branch_tokens_per_s": tokens_per_round / (float(seg[:, 2:K + 2].sum(axis=1).mean()) * 1e-3),
        # the draft stream's own time per round (HIP events: glue extend + fan-out + K steps), over the segment-timing rounds
        "round_ms_percentiles": dict(zip(("p10", "p50", "p90"),
                                         (float(x) for x in np.percentile(seg[:, :K + 2].sum(axis=1), [10, 50, 90])))),
        "roofline": {"kernel": ((f"fused_kernel: one batched branch-decode step ({r.rows} rows) in one persistent launch"
                                 if B.ssd_ctx_views(ctx).pass_rows <= 48 else
                                 f"wide pass: one batched branch-decode step ({r.rows} rows), one launch per phase "
                                 f"(wide_gemm_kernel, wide_gemm_lds_kernel, wide_kernel)") if fused
                                else f"one batched branch-decode step ({r.rows} rows), one kernel per operator"),
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic_bytes() if headline and fused else None,
                     "bytes_per_launch": bytes_step, "avg_ms": kernel_ms,
                     # against what a plain streaming read reaches on this machine (profiles/microbenchmarks_mi355x.txt)
                     "frac_of_measured_stream_read": achieved / MEASURED_STREAM_READ_GBS},
    }
    # with hundreds of rows the linear layers approach the MFMA ridge: report their share of the dense 16-bit peak too
    d_, f_, L_ = shape.d_model, shape.d_ffn, shape.n_layers
    qd_, kvd_ = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    gemm_flops = 2.0 * r.rows * (L_ * ((qd_ + 2 * kvd_) * d_ + d_ * qd_ + 3 * d_ * f_) + V * d_)
    out["mfma"] = {"gemm_flops_per_step": gemm_flops, "achieved_tflops": gemm_flops / (kernel_ms * 1e-3) / 1e12,
                   "peak_tflops": 2500.0, "frac": gemm_flops / (kernel_ms * 1e-3) / 2.5e15}

    if headline and not args.no_sub_records:
        # the other single-GPU workloads of the same model, compactly (their own full lines: --workload)
        out["other_workloads"] = {name: sub_record(B, I, model, shape, name, steps=max(2, min(args.steps, 5)))
                                  for name in ("1b_p8192_f8_t1", "1b_b16_p2048_f4")}

    if headline and not args.no_cpu_baseline:
        # The CPU oracle on the SAME round: glue extend, then every branch from the key the GPU's round cached, one at a
        # time.  Timed as the reported baseline, and compared with the GPU's cache (the bench line checks itself).
        from oracle import ssd_oracle as O
        om = O.Model.from_weights(shape, w)
        trunk = O.KV([k[l, 0].astype(np.float64) for l in range(shape.n_layers)],
                     [v[l, 0].astype(np.float64) for l in range(shape.n_layers)])
        pend = pending.cpu().numpy()[0]
        glue_logits, _, trunk_glue = O.glue_extend(om, trunk, pend)
        gpu_glue = B.device_copy(view.d_glue_logits, (K + 1, V), torch.float32).cpu().numpy()
        worst = float((np.abs(gpu_glue - glue_logits).max(axis=1) / np.abs(glue_logits).max(axis=1)).max())
        n_branches = r.rows                        # every branch of one round, one at a time
        n_tok_checked = 0
        t0 = time.perf_counter()
        for j in range(n_branches):
            toks_o, logits_o, _, margins_o = O.decode_branch(om, trunk_glue, P, j // F, int(gpu_keys[j]), K, 0.0, 0, j)
            lg = B.device_copy(view.d_logits + j * K * V * 4, (K, V), torch.float32).cpu().numpy()
            for i in range(K):                     # the GPU ran free: compare while its inputs are the oracle's
                e = float(np.abs(lg[i] - logits_o[i]).max() / np.abs(logits_o[i]).max())
                worst = max(worst, e)
                decided = margins_o[i] > 2 * np.abs(lg[i] - logits_o[i]).max()
                if decided:
                    assert gpu_toks[j, i] == toks_o[i], f"branch {j} step {i}: token differs from the oracle's"
                    n_tok_checked += 1
                if gpu_toks[j, i] != toks_o[i]:
                    break
        dt = time.perf_counter() - t0
        assert worst < 5e-3, f"the GPU round differs from the oracle: rel err {worst}"
        out["self_check"] = {"logits_rel_err_vs_oracle": worst, "tokens_equal_where_decided": n_tok_checked,
                             "branches": n_branches, "bound": 5e-3}
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": n_branches * K / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{n_branches} of {r.rows} branches x {K} tokens, one branch at a time "
                                         f"(float64 numpy oracle, same weights and prefix), {dt:.1f} s"}
    print(json.dumps(out))
    B.ssd_ctx_destroy(ctx)
    B.ssd_model_destroy(model)


if __name__ == "__main__":
    main()
