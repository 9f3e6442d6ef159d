#!/usr/bin/env python3
"""Benchmark of the Flux Attention hot path on one MI355X.

A timed "step" is one prefill pass of the whole attention stack of the stack-prefill workload
(32 layers x [flux_kv_append + flux_attn_prefill], batch 1, 32768 tokens, 32/8 heads, D 128,
16 of 32 layers SA with 128 sinks + 4096 window), inputs resident in HBM.  `value` is prefill
tokens/s of that routed mix.  The same run also times the all-FA mask (speedup of the mix), the
long-context decode workload (32 layers, batch 8, 131072 cached tokens; ms per step, mix and all-FA),
the router, and the CPU oracle on a bounded sample (`cpu_baseline`).

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
CSRC = os.path.join(ROOT, "paper_2604_07394_amd", "csrc")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--decode-steps", type=int, default=128)
    ap.add_argument("--decode-warmup", type=int, default=10)
    ap.add_argument("--only", choices=["all", "prefill", "decode", "router"], default="all",
                    help="restrict the run (profiling); the JSON line then carries nulls for the rest")
    ap.add_argument("--mask", choices=["mix", "all-fa", "all-sa"], default="mix",
                    help="layer mask of the timed steps; all-fa / all-sa give single-kernel profiles")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--small", action="store_true", help="shrunken shapes for a quick functional check")
    ap.add_argument("--sweep", action="store_true",
                    help="also time one FA and one SA layer at context lengths 8K..256K (prefill and decode, batch 1)")
    ap.add_argument("--extra", action="store_true",
                    help="more repetitions of the high-sparsity prefill workload (28 layers, batch 2, 65536 tokens, 28/4 "
                         "heads, 21 SA layers) and of the end-to-end routed workload (32 layers, ragged batch "
                         "8K/32K/64K/128K, router decisions taken on the device); both run by default with few repetitions")
    ap.add_argument("--no-extra", action="store_true", help="skip those two workloads")
    return ap.parse_args()


def source_digest(names):
    """sha256 over the kernel sources a counter measurement belongs to (first 16 hex digits)."""
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(CSRC, n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(key, sources):
    """HBM bytes per launch recorded under profiles/ from rocprofv3 counter runs.  A record carries the digest
    of the kernel sources it was measured on; it is reported only while those sources are unchanged, so a
    later kernel change cannot leave a stale figure in the line.  Returns (bytes or None, note)."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")):
            f = line.split()
            if len(f) == 7 and f[0] == key:
                if f[6] != source_digest(sources):
                    return None, "the recorded counters were taken on other kernel sources (digest %s)" % f[6]
                return float(f[2]) + float(f[4]), "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, see profiles/"
    except OSError:
        pass
    return None, "no counter record for this workload"


def bf16_to_f64(t):
    """torch bf16 tensor -> float64 NumPy array, exactly (inputs for the CPU baseline leg)."""
    return t.detach().to("cpu", dtype=__import__("torch").float32).numpy().astype("float64")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2604_07394_amd import binding as F
    from paper_2604_07394_amd import synth, synth_gpu

    torch.cuda.set_device(0)
    dev = "cuda"
    ctx = F.flux_create(0, 0)

    def i32(x):
        return torch.tensor(x, dtype=torch.int32, device=dev)

    result = {}

    # ------------------------------------------------------------------ prefill: stack-prefill workload
    L, S, HQ, HKV, D, NS, W, N_SA, SEED = 32, 32768, 32, 8, 128, 128, 4096, 16, 1
    if args.small:
        L, S, N_SA = 4, 4096, 2
    G = HQ // HKV
    mask_mix = synth.random_layer_mask(SEED, L, N_SA)            # 1 = FA, 0 = SA
    if args.mask == "all-fa":
        mask_mix = np.ones(L, dtype=np.uint8)
    elif args.mask == "all-sa":
        mask_mix = np.zeros(L, dtype=np.uint8)
    cfg = F.attn_cfg(HQ, HKV, D, NS, W, 0.0, 0)                 # bf16 output, as the paper's BF16 runs

    def pairs_fa(s):
        return s * (s + 1) // 2

    def pairs_sa(s):
        return sum(min(i + 1, W) + max(0, min(NS, i + 1 - W)) for i in range(s))

    flops_fa = 4.0 * D * HQ * pairs_fa(S)
    flops_sa = 4.0 * D * HQ * pairs_sa(S)

    prefill = None
    roofline = None
    cpu_baseline = None
    if args.only in ("all", "prefill"):
        q = torch.empty(L, S, HQ, D, dtype=torch.bfloat16, device=dev)
        kn = torch.empty(L, S, HKV, D, dtype=torch.bfloat16, device=dev)
        vn = torch.empty(L, S, HKV, D, dtype=torch.bfloat16, device=dev)
        out = torch.empty(S, HQ, D, dtype=torch.bfloat16, device=dev)
        caches = [F.KVCache.empty(1, HKV, S, D) for _ in range(L)]
        for l in range(L):
            qs = torch.from_numpy(synth.head_scales(SEED, synth.stream_id(synth.STREAM_QSCALE, l), HQ)).to(dev)
            ks = torch.from_numpy(synth.head_scales(SEED, synth.stream_id(synth.STREAM_KSCALE, l), HKV)).to(dev)
            vs = torch.from_numpy(synth.head_scales(SEED, synth.stream_id(synth.STREAM_VSCALE, l), HKV)).to(dev)
            synth_gpu.fill_normal_bf16(q[l][None], SEED, synth.stream_id(synth.STREAM_Q, l), qs, 2)
            synth_gpu.fill_normal_bf16(kn[l][None], SEED, synth.stream_id(synth.STREAM_K, l), ks, 2)
            synth_gpu.fill_normal_bf16(vn[l][None], SEED, synth.stream_id(synth.STREAM_V, l), vs, 2)
        cu = i32([0, S])
        modes = {0: torch.zeros(1, dtype=torch.uint8, device=dev), 1: torch.ones(1, dtype=torch.uint8, device=dev)}
        torch.cuda.synchronize()

        def prefill_step(mask, events=None):
            for l in range(L):
                caches[l].kv_len.zero_()
                F.flux_kv_append(ctx, caches[l], HKV, D, kn[l], vn[l], cu, S, S)
                if events is not None:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                F.flux_attn_prefill(ctx, cfg, q[l], cu, S, S, caches[l], modes[int(mask[l])], out)
                if events is not None:
                    e1.record()
                    events.append((int(mask[l]), e0, e1))

        def time_steps(mask, steps, warmup, events=None):
            for _ in range(warmup):
                prefill_step(mask)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                prefill_step(mask, events)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

        ev = []
        t_mix = time_steps(mask_mix, args.steps, args.warmup, ev)
        fa_ms = [a.elapsed_time(b) for m, a, b in ev if m == 1]
        sa_ms = [a.elapsed_time(b) for m, a, b in ev if m == 0]
        # the all-FA comparison pass (skipped in single-mode profiling runs)
        t_fa = time_steps(np.ones(L, dtype=np.uint8), max(1, args.steps // 2), 1) if args.mask == "mix" else None
        fa_avg = sum(fa_ms) / max(len(fa_ms), 1)
        sa_avg = sum(sa_ms) / max(len(sa_ms), 1)
        n_fa = int(mask_mix.sum())
        pred = (L * flops_fa) / (n_fa * flops_fa + (L - n_fa) * flops_sa)
        prefill = {
            "tokens_per_s_mix": S / t_mix, "ms_per_step_mix": t_mix * 1e3,
            "tokens_per_s_all_fa": S / t_fa if t_fa else None, "ms_per_step_all_fa": t_fa * 1e3 if t_fa else None,
            "speedup_mix_vs_all_fa": t_fa / t_mix if t_fa else None, "predicted_speedup_from_flops": pred,
            "omega_msr": float((mask_mix == 0).mean()),
            "mask": args.mask, "fa_kernel_ms": fa_avg, "sa_kernel_ms": sa_avg,
            "fa_kernel_ms_median": float(np.median(fa_ms)) if fa_ms else None,
            "sa_kernel_ms_median": float(np.median(sa_ms)) if sa_ms else None,
            "sa_kernel_tflops": flops_sa / (sa_avg * 1e-3) / 1e12 if sa_ms else None,
        }
        achieved = flops_fa / (fa_avg * 1e-3) / 1e12 if fa_ms else 0.0
        roofline = {"kernel": "prefill_kernel<128, false, 8, 2> (FA layers; eight waves per workgroup on two heads of a GQA group from 32768-token prompts on)", "bound": "mfma", "achieved": achieved,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                    "traffic": None, "traffic_note": "not the profiled workload",
                    "traffic_unit": "bytes per launch",
                    "flops_per_launch": flops_fa, "launch_ms": fa_avg,
                    "launch_ms_source": "HIP events on the launch stream around every FA launch of the timed steps"}
        if not args.small:
            roofline["traffic"], roofline["traffic_note"] = measured_traffic(
                "prefill_fa_stack_prefill_32768", ["prefill.hip", "flux_internal.h"])

        # ---- block-sparse prefill over an explicit keep matrix of 64 x 64 blocks, and the XA block selection that
        # writes such a matrix (layer 0's tensors, one keep matrix per query head)
        if args.mask == "mix":
            nb = (S + 63) // 64
            caches[0].kv_len.zero_()
            F.flux_kv_append(ctx, caches[0], HKV, D, kn[0], vn[0], cu, S, S)

            def timed(fn, reps=3):
                fn()
                es = []
                for _ in range(reps):
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    fn()
                    e1.record()
                    es.append((e0, e1))
                torch.cuda.synchronize()
                return sum(a.elapsed_time(b) for a, b in es) / reps

            tri = torch.tril(torch.ones(nb, nb, dtype=torch.bool, device=dev), -1)
            eye = torch.eye(nb, dtype=torch.bool, device=dev)

            def visible_pairs(keep):                              # keep: uint8 [1, HQ, nb, nb]; whole prompt, S % 64 == 0
                k = keep[0].bool()
                return int((k & tri).sum().item()) * 64 * 64 + HQ * nb * (64 * 65 // 2)

            bs = {"block": 64, "blocks_per_side": nb, "fa_kernel_ms": fa_avg}
            gen = torch.Generator(device=dev)
            gen.manual_seed(SEED)
            for dens in (0.10, 0.25):
                keep = torch.rand(1, HQ, nb, nb, device=dev, generator=gen) < dens
                keep[..., 0] = True                               # the block of the first positions, as a sink
                keep = ((keep & tri) | eye).to(torch.uint8).contiguous()
                ms = timed(lambda: F.flux_attn_prefill_blocksparse(ctx, cfg, q[0], cu, S, S, caches[0], modes[0], keep,
                                                                   HQ, nb, nb, out))
                fl = 4.0 * D * visible_pairs(keep)
                bs["random_keep_%.2f" % dens] = {"kept_fraction_of_causal_blocks": float(keep.sum().item()) / (HQ * nb * (nb + 1) / 2),
                                                 "kernel_ms": ms, "tflops_over_kept_pairs": fl / (ms * 1e-3) / 1e12,
                                                 "speedup_vs_fa_launch": fa_avg / ms}
            # the same densities as whole key columns per head (every query block keeps the same key blocks) plus the
            # four most recent blocks: the shape attention maps usually have (vertical stripes and a local band), where
            # the query blocks of a 128-row tile agree on what they visit
            band = torch.tril(torch.ones(nb, nb, dtype=torch.bool, device=dev)) & ~torch.tril(torch.ones(nb, nb, dtype=torch.bool, device=dev), -4)
            for dens in (0.10, 0.25):
                cols = torch.rand(1, HQ, 1, nb, device=dev, generator=gen) < dens
                cols[..., 0] = True
                keep = (((cols.expand(1, HQ, nb, nb) & tri) | band)).to(torch.uint8).contiguous()
                ms = timed(lambda: F.flux_attn_prefill_blocksparse(ctx, cfg, q[0], cu, S, S, caches[0], modes[0], keep,
                                                                   HQ, nb, nb, out))
                fl = 4.0 * D * visible_pairs(keep)
                bs["striped_keep_%.2f" % dens] = {"kept_fraction_of_causal_blocks": float(keep.sum().item()) / (HQ * nb * (nb + 1) / 2),
                                                  "kernel_ms": ms, "tflops_over_kept_pairs": fl / (ms * 1e-3) / 1e12,
                                                  "speedup_vs_fa_launch": fa_avg / ms}
            xa_keep = torch.zeros(1, HQ, nb, nb, dtype=torch.uint8, device=dev)
            for thr in (0.9, 0.5):
                ms_sel = timed(lambda: F.flux_xa_select(ctx, cfg, q[0], cu, S, S, caches[0], 16, thr, xa_keep, nb, nb))
                ms = timed(lambda: F.flux_attn_prefill_blocksparse(ctx, cfg, q[0], cu, S, S, caches[0], modes[0], xa_keep,
                                                                   HQ, nb, nb, out))
                fl = 4.0 * D * visible_pairs(xa_keep)
                bs["xa_threshold_%.1f" % thr] = {"select_ms": ms_sel, "kept_fraction_of_causal_blocks": float(xa_keep.sum().item()) / (HQ * nb * (nb + 1) / 2),
                                                 "kernel_ms": ms, "tflops_over_kept_pairs": fl / (ms * 1e-3) / 1e12,
                                                 "select_plus_kernel_vs_fa_launch": fa_avg / (ms_sel + ms)}
            # the same selection on inputs WITH structure: every query leans towards a direction u_h of its head, and the
            # keys of 8 % of the 64-position blocks (whole columns, per KV head) lean the same way, so most of the
            # attention mass sits on those columns and on nothing else
            gq = torch.Generator(device=dev)
            gq.manual_seed(SEED + 77)
            u = torch.sign(torch.randn(HKV, D, device=dev, generator=gq))                     # |u|^2 = D
            qs = torch.randn(S, HQ, D, device=dev, generator=gq) + 0.8 * u.repeat_interleave(G, 0)[None]
            stripe = (torch.rand(HKV, nb, device=dev, generator=gq) < 0.08).repeat_interleave(64, 1)[:, :S]   # [HKV, S]
            ks_ = torch.randn(S, HKV, D, device=dev, generator=gq) + 0.8 * stripe.t()[:, :, None] * u[None]
            vs_ = torch.randn(S, HKV, D, device=dev, generator=gq)
            qs, ks_, vs_ = qs.to(torch.bfloat16), ks_.to(torch.bfloat16), vs_.to(torch.bfloat16)
            caches[0].kv_len.zero_()
            F.flux_kv_append(ctx, caches[0], HKV, D, ks_, vs_, cu, S, S)
            ms_sel = timed(lambda: F.flux_xa_select(ctx, cfg, qs, cu, S, S, caches[0], 16, 0.9, xa_keep, nb, nb))
            ms = timed(lambda: F.flux_attn_prefill_blocksparse(ctx, cfg, qs, cu, S, S, caches[0], modes[0], xa_keep,
                                                               HQ, nb, nb, out))
            ms_fa = timed(lambda: F.flux_attn_prefill(ctx, cfg, qs, cu, S, S, caches[0], modes[1], out))
            fl = 4.0 * D * visible_pairs(xa_keep)
            bs["xa_threshold_0.9_structured_input"] = {
                "input": "q = N(0,1) + 0.8 u_head, k = N(0,1) + 0.8 u_head on 8 percent of the key blocks (whole columns per KV head), seed %d" % (SEED + 77),
                "select_ms": ms_sel, "kept_fraction_of_causal_blocks": float(xa_keep.sum().item()) / (HQ * nb * (nb + 1) / 2),
                "kernel_ms": ms, "tflops_over_kept_pairs": fl / (ms * 1e-3) / 1e12, "fa_kernel_ms_same_input": ms_fa,
                "select_plus_kernel_vs_fa_launch": ms_fa / (ms_sel + ms)}
            del qs, ks_, vs_, stripe, u
            bs["note"] = ("seeded Gaussian queries and keys carry no attention structure, so the XA selection keeps most "
                          "blocks; the random keep matrices show the kernel at the densities a structured prompt gives")
            prefill["blocksparse"] = bs
            del keep, xa_keep, tri, eye, band

            # ---- one FA launch on a ragged batch with a small GQA group (16/8 heads, prompts of 8192 and 65536 tokens):
            # most workgroups past the short prompt's end are empty, and where they fall among the others decides whether
            # every CU gets work (the launch order takes the pairs of an XCD one after the other for this reason)
            if not args.small:
                rl, rhq = [8192, 65536], 16
                rt = sum(rl)
                rcfg = F.attn_cfg(rhq, HKV, D, NS, W, 0.0, 0)
                rq = torch.empty(1, rt, rhq, D, dtype=torch.bfloat16, device=dev)
                rk = torch.empty(1, rt, HKV, D, dtype=torch.bfloat16, device=dev)
                synth_gpu.fill_normal_bf16(rq, SEED + 91, synth.stream_id(synth.STREAM_Q))
                synth_gpu.fill_normal_bf16(rk, SEED + 91, synth.stream_id(synth.STREAM_K))
                rcache = F.KVCache.empty(len(rl), HKV, max(rl), D)
                rcu = torch.tensor(np.concatenate([[0], np.cumsum(rl)]), dtype=torch.int32, device=dev)
                F.flux_kv_append(ctx, rcache, HKV, D, rk[0], rk[0], rcu, rt, max(rl))
                rout = torch.empty(rt, rhq, D, dtype=torch.bfloat16, device=dev)
                rmode = torch.ones(len(rl), dtype=torch.uint8, device=dev)
                ms = timed(lambda: F.flux_attn_prefill(ctx, rcfg, rq[0], rcu, max(rl), max(rl), rcache, rmode, rout))
                rflops = 4.0 * D * rhq * sum(n * (n + 1) // 2 for n in rl)
                prefill["ragged_small_group_fa"] = {"workload": "one FA launch, batch of 2 prompts (8192 and 65536 tokens), 16/8 heads, D 128",
                                                    "kernel_ms": ms, "tflops": rflops / (ms * 1e-3) / 1e12}
                del rq, rk, rcache, rout

        # ---- CPU oracle on a bounded sample of the same workload (rank 0, N = 1)
        if not args.no_cpu_baseline:
            from oracle import flux_oracle as O
            try:
                from threadpoolctl import threadpool_info
                cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
            except Exception:
                cores = 1
            rng = np.random.default_rng(0)
            per_layer, n_rows = {}, {}
            t_used = 0.0
            budget = 1.0 if args.small else 9.0                 # seconds of oracle time per mode
            for m in (1, 0):
                layer = int(np.nonzero(mask_mix == m)[0][0])
                kf = bf16_to_f64(kn[layer][:, 0])                # KV head 0 of that layer, [S, D]
                vf = bf16_to_f64(vn[layer][:, 0])
                qf = bf16_to_f64(q[layer][:, :G])                # its G query heads, [S, G, D]
                rows = rng.integers(0, S, size=100000)
                t0 = time.perf_counter()
                done = 0
                while time.perf_counter() - t0 < budget and done < len(rows):
                    i = int(rows[done])
                    O.attention_row(qf[i], kf, vf, i, m, NS, W)
                    done += 1
                dt = time.perf_counter() - t0
                t_used += dt
                n_rows[m] = done
                per_layer[m] = dt / done * S * HKV               # seconds for one whole layer
            t_full = n_fa * per_layer[1] + (L - n_fa) * per_layer[0]
            cpu_baseline = {"value": S / t_full, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                            "sample": "fp64 NumPy oracle (attention_row), %d FA + %d SA uniformly drawn query "
                                      "positions of one KV group (%d heads) in one FA and one SA layer, %.1f s of CPU "
                                      "work, extrapolated to %d layers x %d positions x %d groups"
                                      % (n_rows[1], n_rows[0], G, t_used, L, S, HKV)}

            # ---- the Tiny configuration through the oracle IN FULL (nothing extrapolated): 4 layers [FA, SA, FA,
            # SA], 512 tokens, 8/2 heads, D 64, 16 sinks + 128 window, prefill then 16 decode steps; once with
            # the BLAS pool limited to one thread and once with all the threads it takes by default
            def tiny_oracle():
                t0 = time.perf_counter()
                for layer, m in enumerate((1, 0, 1, 0)):
                    draw = lambda kind, rows, heads, step=0: O.bf16_to_f64(synth.normal_bf16(
                        0, synth.stream_id(kind, layer, step), (rows, heads, 64)))
                    oc = O.KVCache(1, 2, 64)
                    O.prefill(oc, [draw(synth.STREAM_Q, 512, 8)], [draw(synth.STREAM_K, 512, 2)],
                              [draw(synth.STREAM_V, 512, 2)], [m], 16, 128)
                    for step in range(16):
                        O.decode_step(oc, draw(synth.STREAM_QDEC, 1, 8, step), draw(synth.STREAM_KDEC, 1, 2, step),
                                      draw(synth.STREAM_VDEC, 1, 2, step), [m], 16, 128)
                return time.perf_counter() - t0

            tiny_oracle()                                        # first call pays imports and page faults
            t_all = min(tiny_oracle() for _ in range(3))
            try:
                from threadpoolctl import threadpool_limits
                with threadpool_limits(limits=1):
                    t_one = min(tiny_oracle() for _ in range(3))
            except Exception:
                t_one = None
            cpu_baseline["tiny_config_in_full"] = {
                "what": "oracle wall-clock for the whole Tiny configuration (4 layers x [512-token prefill + 16 decode "
                        "steps]), input generation included, best of 3",
                "seconds_single_thread": t_one, "seconds_all_cores": t_all, "cores": cores,
                "prefill_tokens_per_s_all_cores": 512 / t_all}
        del q, kn, vn, out, caches
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ decode: long-context decode workload
    decode = None
    if args.only in ("all", "decode"):
        LD, B, N, SEED_D = 32, 8, 131072, 2
        n_dec = args.decode_steps + args.decode_warmup
        if args.small:
            LD, B, N = 4, 2, 16384
        cap = N + 2 * n_dec + 8
        mask_d = synth.random_layer_mask(SEED_D, LD, LD // 2)
        if args.mask == "all-fa":
            mask_d = np.ones(LD, dtype=np.uint8)
        elif args.mask == "all-sa":
            mask_d = np.zeros(LD, dtype=np.uint8)
        kc = torch.empty(LD, B, HKV, cap, D, dtype=torch.bfloat16, device=dev)
        vc = torch.empty(LD, B, HKV, cap, D, dtype=torch.bfloat16, device=dev)
        for l in range(LD):
            synth_gpu.fill_normal_bf16(kc[l][:, :, :N], SEED_D, synth.stream_id(synth.STREAM_K, l))
            synth_gpu.fill_normal_bf16(vc[l][:, :, :N], SEED_D, synth.stream_id(synth.STREAM_V, l))
        kv_len = torch.full((LD, B), N, dtype=torch.int32, device=dev)
        dcaches = [F.KVCache(kc[l], vc[l], kv_len[l]) for l in range(LD)]
        qd = torch.empty(1, LD, B * HQ, D, dtype=torch.bfloat16, device=dev)
        kd = torch.empty(1, LD, B * HKV, D, dtype=torch.bfloat16, device=dev)
        vd = torch.empty(1, LD, B * HKV, D, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(qd, SEED_D, synth.stream_id(synth.STREAM_QDEC))
        synth_gpu.fill_normal_bf16(kd, SEED_D, synth.stream_id(synth.STREAM_KDEC))
        synth_gpu.fill_normal_bf16(vd, SEED_D, synth.stream_id(synth.STREAM_VDEC))
        outd = torch.empty(B, HQ, D, dtype=torch.bfloat16, device=dev)
        cu1 = i32(list(range(B + 1)))
        dmodes = {0: torch.zeros(B, dtype=torch.uint8, device=dev), 1: torch.ones(B, dtype=torch.uint8, device=dev)}
        torch.cuda.synchronize()
        cur = {"n": N}

        def decode_step(mask, events=None, fused=True):
            """One decode step of the stack: per layer, append the new K/V row of every sequence and attend.
            fused: one flux_attn_decode_append call per layer (two launches); else flux_kv_append followed by
            flux_attn_decode (three launches, the same results bit for bit)."""
            cur["n"] += 1
            for l in range(LD):
                if not fused:
                    F.flux_kv_append(ctx, dcaches[l], HKV, D, kd[0, l], vd[0, l], cu1, B, 1)
                if events is not None:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                # the cached mask is known on the host after prefill: SA layers are sized for sinks + window
                bound = cur["n"] if mask[l] else min(cur["n"], NS + W)
                if fused:
                    F.flux_attn_decode_append(ctx, cfg, qd[0, l], kd[0, l], vd[0, l], bound, dcaches[l],
                                              dmodes[int(mask[l])], outd)
                else:
                    F.flux_attn_decode(ctx, cfg, qd[0, l], bound, dcaches[l], dmodes[int(mask[l])], outd)
                if events is not None:
                    e1.record()
                    events.append((int(mask[l]), e0, e1))

        def time_decode(mask, steps, warmup, events=None, fused=True):
            for _ in range(warmup):
                decode_step(mask, fused=fused)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                decode_step(mask, events, fused)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

        ev = []
        half = max(1, args.decode_steps // 2)
        # the step time is taken without events on the stream (two event records per layer cost a 36 us layer some
        # microseconds each); the per-layer durations come from a second, shorter pass that records them
        td_mix = time_decode(mask_d, args.decode_steps, args.decode_warmup)
        kv_len.fill_(N)
        cur["n"] = N
        time_decode(mask_d, half, 2, ev)
        fa_ms = [a.elapsed_time(b) for m, a, b in ev if m == 1]
        sa_ms = [a.elapsed_time(b) for m, a, b in ev if m == 0]
        kv_len.fill_(N)
        cur["n"] = N
        td_fa = time_decode(np.ones(LD, dtype=np.uint8), half, 2) if args.mask == "mix" else None
        kv_len.fill_(N)
        cur["n"] = N
        td_mix_3 = time_decode(mask_d, args.decode_steps, args.decode_warmup, fused=False) if args.mask == "mix" else None
        # ---- sparse-decode residency (Sec. 3.3): the SA layers keep only sinks + window rows in a ring cache,
        # compacted from the full cache as after a prefill; FA layers keep the full cache
        ring_info = None
        if args.mask == "mix":
            kv_len.fill_(N)
            cur["n"] = N
            sa_layers = [l for l in range(LD) if not mask_d[l]]
            rk = torch.empty(len(sa_layers), B, HKV, NS + W, D, dtype=torch.bfloat16, device=dev)
            rv = torch.empty_like(rk)
            rlen = torch.zeros(len(sa_layers), B, dtype=torch.int32, device=dev)
            rings = {}
            for i, l in enumerate(sa_layers):
                rings[l] = F.KVCache(rk[i], rv[i], rlen[i])
                F.flux_kv_compact_ring(ctx, dcaches[l], rings[l], HKV, D, NS, W)

            def ring_step():
                cur["n"] += 1
                for l in range(LD):
                    if mask_d[l]:
                        F.flux_kv_append(ctx, dcaches[l], HKV, D, kd[0, l], vd[0, l], cu1, B, 1)
                        F.flux_attn_decode(ctx, cfg, qd[0, l], cur["n"], dcaches[l], dmodes[1], outd)
                    else:
                        F.flux_kv_append_ring(ctx, rings[l], HKV, D, NS, W, kd[0, l], vd[0, l], cu1, B, 1)
                        F.flux_attn_decode_ring(ctx, cfg, qd[0, l], rings[l], outd)

            for _ in range(3):
                ring_step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(half):
                ring_step()
            torch.cuda.synchronize()
            row_bytes = 2 * B * HKV * D * 2
            ring_info = {"ms_per_step_mix": (time.perf_counter() - t0) / half * 1e3,
                         "kv_cache_bytes_all_full": LD * N * row_bytes,
                         "kv_cache_bytes_ring_residency": int(mask_d.sum()) * N * row_bytes + len(sa_layers) * (NS + W) * row_bytes}
            del rk, rv, rings
        # ---- the same routed step replayed from a HIP graph (no host launch cost): the calls are plain
        # launches on the caller's stream, FA layers are sized for the cache capacity so one capture stays valid
        graph_ms = None
        if args.mask == "mix":
            kv_len.fill_(N)
            cur["n"] = N

            def graph_step():
                for l in range(LD):
                    F.flux_attn_decode_append(ctx, cfg, qd[0, l], kd[0, l], vd[0, l], cap if mask_d[l] else NS + W,
                                              dcaches[l], dmodes[int(mask_d[l])], outd)

            graph_step()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                graph_step()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(half):
                g.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t0) / half * 1e3
            del g
        fa_avg = sum(fa_ms) / max(len(fa_ms), 1)
        sa_avg = sum(sa_ms) / max(len(sa_ms), 1)
        n_mid = N + 2 + (half + 1) // 2                                          # mean length over the pass that recorded the events
        bytes_fa = 2.0 * B * n_mid * HKV * D * 2 + 2.0 * B * HQ * D * 2         # K and V rows once + q + out
        bytes_sa = 2.0 * B * (NS + W) * HKV * D * 2 + 2.0 * B * HQ * D * 2
        n_fa = int(mask_d.sum())
        ach = bytes_fa / (fa_avg * 1e-3) / 1e9 if fa_ms else 0.0
        decode = {
            "workload": "long-context decode: %d layers, batch %d, %d cached tokens, %d/%d heads, D %d, "
                        "%d of %d layers SA (%d sinks + %d window), seed %d" % (LD, B, N, HQ, HKV, D, LD - n_fa, LD, NS, W, SEED_D),
            "ms_per_step_mix": td_mix * 1e3, "ms_per_step_all_fa": td_fa * 1e3 if td_fa else None,
            "speedup_mix_vs_all_fa": td_fa / td_mix if td_fa else None,
            "layer_call": "flux_attn_decode_append (the new row of every sequence is appended inside the decode call)",
            "ms_per_step_mix_append_then_decode": td_mix_3 * 1e3 if td_mix_3 else None,
            "predicted_speedup_from_bytes": (LD * bytes_fa) / (n_fa * bytes_fa + (LD - n_fa) * bytes_sa),
            "fa_layer_ms": fa_avg, "sa_layer_ms": sa_avg,
            "fa_layer_ms_median": float(np.median(fa_ms)) if fa_ms else None,
            "sa_layer_ms_median": float(np.median(sa_ms)) if sa_ms else None,
            "roofline": {"kernel": "decode_splitk_kernel<128, true, true> + decode_combine_kernel<128> (FA layers)",
                         "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": ach / PEAK_HBM_GBS,
                         "traffic": None, "traffic_note": "not the profiled workload",
                         "bytes_per_launch": bytes_fa,
                         "launch_ms": fa_avg},
            "sa_achieved_gbs": bytes_sa / (sa_avg * 1e-3) / 1e9 if sa_ms else None,
            "sparse_decode_residency": ring_info,
            "ms_per_step_mix_hip_graph": graph_ms,
        }
        if not args.small:
            decode["roofline"]["traffic"], decode["roofline"]["traffic_note"] = measured_traffic(
                "decode_fa_long_context_131072", ["decode.hip", "flux_internal.h"])
        del kc, vc, dcaches
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ router (end-to-end routed workload shape)
    lens = [8192, 32768, 65536, 131072] if not args.small else [512, 2048]
    hidden, inner, pool = 4096, 256, 100
    T = sum(lens)
    x = torch.empty(1, 1, T, hidden, dtype=torch.bfloat16, device=dev)
    synth_gpu.fill_normal_bf16(x, 4, synth.stream_id(synth.STREAM_X))
    w1 = torch.empty(1, 1, inner, hidden, dtype=torch.bfloat16, device=dev)
    w2 = torch.empty(1, 1, 2, inner, dtype=torch.bfloat16, device=dev)
    s02 = torch.full((1,), 0.02, dtype=torch.float32, device=dev)
    synth_gpu.fill_normal_bf16(w1, 4, synth.stream_id(synth.STREAM_W1), s02, 0)
    synth_gpu.fill_normal_bf16(w2, 4, synth.stream_id(synth.STREAM_W2), s02, 0)
    cu_r = i32([0] + list(np.cumsum(lens)))
    mode_r = torch.zeros(len(lens), dtype=torch.uint8, device=dev)
    def time_router(pool_rows, reps):
        for _ in range(10):
            F.flux_router(ctx, x, cu_r, len(lens), hidden, pool_rows, w1, None, w2, None, inner, mode_r)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            F.flux_router(ctx, x, cu_r, len(lens), hidden, pool_rows, w1, None, w2, None, inner, mode_r)
        e1.record()
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3, t_host / reps * 1e6

    us_pool, us_host = time_router(pool, 200)
    us_full, _ = time_router(0, 20)          # the "Full" pooling point of App. D.2: mean over every row
    # the router's cost against the prompt length (Sec. 4.3 reports 0.20 ms per layer, flat from 512 to 1M
    # tokens): one sequence of S rows, same weights; only the first and last `pool` rows are read
    del x
    torch.cuda.empty_cache()
    flat = {}
    if not args.small:
        s_max = 1 << 20
        xl = torch.empty(1, 1, s_max, hidden, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(xl, 4, synth.stream_id(synth.STREAM_X))
        mode_1 = torch.zeros(1, dtype=torch.uint8, device=dev)
        for s_len in (512, 8192, 131072, s_max):
            cu_s = i32([0, s_len])
            for _ in range(5):
                F.flux_router(ctx, xl, cu_s, 1, hidden, pool, w1, None, w2, None, inner, mode_1)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(100):
                F.flux_router(ctx, xl, cu_s, 1, hidden, pool, w1, None, w2, None, inner, mode_1)
            e1.record()
            torch.cuda.synchronize()
            flat[str(s_len)] = e0.elapsed_time(e1) / 100 * 1e3
        del xl
    router = {"us_per_layer_call": us_pool, "host_launch_us": us_host, "batch": len(lens), "pool": pool,
              "us_per_call_vs_prompt_tokens": flat,
              "us_per_layer_call_pool_all_rows": us_full, "rows_all": T,
              "hidden": hidden, "inner": inner, "paper_ms_per_layer": 0.20}

    # ------------------------------------------------------------------ optional: one layer against the context length
    sweep = None
    if args.sweep:
        sweep = {}
        for s_len in (8192, 32768, 131072, 262144):
            qs_ = torch.empty(1, s_len, HQ, D, dtype=torch.bfloat16, device=dev)
            ks_ = torch.empty(1, s_len, HKV, D, dtype=torch.bfloat16, device=dev)
            vs_ = torch.empty(1, s_len, HKV, D, dtype=torch.bfloat16, device=dev)
            synth_gpu.fill_normal_bf16(qs_, 6, synth.stream_id(synth.STREAM_Q))
            synth_gpu.fill_normal_bf16(ks_, 6, synth.stream_id(synth.STREAM_K))
            synth_gpu.fill_normal_bf16(vs_, 6, synth.stream_id(synth.STREAM_V))
            cache_s = F.KVCache.empty(1, HKV, s_len, D)
            cu_s = i32([0, s_len])
            F.flux_kv_append(ctx, cache_s, HKV, D, ks_[0], vs_[0], cu_s, s_len, s_len)
            out_s = torch.empty(s_len, HQ, D, dtype=torch.bfloat16, device=dev)
            outd_s = torch.empty(1, HQ, D, dtype=torch.bfloat16, device=dev)
            row = {}
            for name, md, reps in (("fa", 1, 3), ("sa", 0, 3)):
                mdev = torch.full((1,), md, dtype=torch.uint8, device=dev)
                F.flux_attn_prefill(ctx, cfg, qs_[0], cu_s, s_len, s_len, cache_s, mdev, out_s)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    F.flux_attn_prefill(ctx, cfg, qs_[0], cu_s, s_len, s_len, cache_s, mdev, out_s)
                e1.record()
                torch.cuda.synchronize()
                row["prefill_%s_ms" % name] = e0.elapsed_time(e1) / reps
                bound = s_len if md else min(s_len, NS + W)
                for _ in range(3):
                    F.flux_attn_decode(ctx, cfg, qs_[0, s_len - 1], bound, cache_s, mdev, outd_s)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(50):
                    F.flux_attn_decode(ctx, cfg, qs_[0, s_len - 1], bound, cache_s, mdev, outd_s)
                e1.record()
                torch.cuda.synchronize()
                row["decode_%s_us" % name] = e0.elapsed_time(e1) / 50 * 1e3
            row["prefill_speedup_sa_over_fa"] = row["prefill_fa_ms"] / row["prefill_sa_ms"]
            row["decode_speedup_sa_over_fa"] = row["decode_fa_us"] / row["decode_sa_us"]
            sweep[str(s_len)] = row
            del qs_, ks_, vs_, cache_s, out_s
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ optional: the two other full-size workloads
    extra = None
    if args.small or args.no_extra or args.only != "all":
        extra = {"not_run": "--small, --no-extra or --only given"}
    else:
        extra = {}
        long_form = args.extra

        def timed(fn, reps, warm=True):
            if warm:
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        # ---- high-sparsity prefill: one set of inputs serves every layer (the cost does not depend on the values)
        L4, B4, S4, HQ4, HKV4, NS4, W4, SEED4 = 28, 2, 65536, 28, 4, 64, 2048, 3
        mask4 = synth.random_layer_mask(SEED4, L4, 21)
        cfg4 = F.attn_cfg(HQ4, HKV4, D, NS4, W4, 0.0, 0)
        q4 = torch.empty(1, B4 * S4, HQ4, D, dtype=torch.bfloat16, device=dev)
        k4 = torch.empty(1, B4 * S4, HKV4, D, dtype=torch.bfloat16, device=dev)
        v4 = torch.empty(1, B4 * S4, HKV4, D, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(q4, SEED4, synth.stream_id(synth.STREAM_Q))
        synth_gpu.fill_normal_bf16(k4, SEED4, synth.stream_id(synth.STREAM_K))
        synth_gpu.fill_normal_bf16(v4, SEED4, synth.stream_id(synth.STREAM_V))
        out4 = torch.empty(B4 * S4, HQ4, D, dtype=torch.bfloat16, device=dev)
        caches4 = [F.KVCache.empty(B4, HKV4, S4, D) for _ in range(L4)]
        cu4 = i32([0, S4, 2 * S4])
        m4 = {0: torch.zeros(B4, dtype=torch.uint8, device=dev), 1: torch.ones(B4, dtype=torch.uint8, device=dev)}

        def step4(mask):
            for l in range(L4):
                caches4[l].kv_len.zero_()
                F.flux_kv_append(ctx, caches4[l], HKV4, D, k4[0], v4[0], cu4, B4 * S4, S4)
                F.flux_attn_prefill(ctx, cfg4, q4[0], cu4, S4, S4, caches4[l], m4[int(mask[l])], out4)

        reps4 = (3, 2) if long_form else (2, 1)
        t4_mix = timed(lambda: step4(mask4), reps4[0])
        t4_fa = timed(lambda: step4(np.ones(L4, dtype=np.uint8)), reps4[1])
        vis_sa4 = sum(min(i + 1, W4) + max(0, min(NS4, i + 1 - W4)) for i in range(S4))
        fl_fa4 = 4.0 * D * HQ4 * B4 * pairs_fa(S4)
        fl_sa4 = 4.0 * D * HQ4 * B4 * vis_sa4
        n_fa4 = int(mask4.sum())
        extra["high_sparsity_prefill"] = {
            "workload": "%d layers, batch %d, seq_len %d, %d/%d heads, D %d, %d of %d layers SA (%d sinks + %d window), seed %d"
                        % (L4, B4, S4, HQ4, HKV4, D, L4 - n_fa4, L4, NS4, W4, SEED4),
            "ms_per_step_mix": t4_mix * 1e3, "ms_per_step_all_fa": t4_fa * 1e3,
            "tokens_per_s_mix": B4 * S4 / t4_mix, "tokens_per_s_all_fa": B4 * S4 / t4_fa,
            "all_fa_tflops": L4 * fl_fa4 / t4_fa / 1e12,
            "mix_tflops": (n_fa4 * fl_fa4 + (L4 - n_fa4) * fl_sa4) / t4_mix / 1e12,
            "speedup_mix_vs_all_fa": t4_fa / t4_mix,
            "predicted_speedup_from_flops": L4 * fl_fa4 / (n_fa4 * fl_fa4 + (L4 - n_fa4) * fl_sa4),
            "omega_msr": float((mask4 == 0).mean()),
            "timed_steps_mix_and_all_fa": list(reps4), "warmup_steps": 1}
        del q4, k4, v4, out4, caches4
        torch.cuda.empty_cache()

        # ---- end-to-end routed: per layer the router reads the query tensor and writes that layer's mode bytes
        # on the device, append + prefill use them with no host read-back; decode reuses the cached bytes
        L5, lens5, SEED5, n_steps5 = 32, [8192, 32768, 65536, 131072], 4, 256
        B5, T5, smax5 = len(lens5), sum(lens5), max(lens5)
        cap5 = smax5 + 2 * n_steps5 + 40
        q5 = torch.empty(1, T5, HQ, D, dtype=torch.bfloat16, device=dev)
        k5 = torch.empty(1, T5, HKV, D, dtype=torch.bfloat16, device=dev)
        v5 = torch.empty(1, T5, HKV, D, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(q5, SEED5, synth.stream_id(synth.STREAM_Q))
        synth_gpu.fill_normal_bf16(k5, SEED5, synth.stream_id(synth.STREAM_K))
        synth_gpu.fill_normal_bf16(v5, SEED5, synth.stream_id(synth.STREAM_V))
        w1_5 = torch.empty(1, L5, inner, hidden, dtype=torch.bfloat16, device=dev)
        w2_5 = torch.empty(1, L5, 2, inner, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(w1_5, SEED5, synth.stream_id(synth.STREAM_W1), s02, 0)
        synth_gpu.fill_normal_bf16(w2_5, SEED5, synth.stream_id(synth.STREAM_W2), s02, 0)
        out5 = torch.empty(T5, HQ, D, dtype=torch.bfloat16, device=dev)
        caches5 = [F.KVCache.empty(B5, HKV, cap5, D) for _ in range(L5)]
        cu5 = i32([0] + list(np.cumsum(lens5)))
        routed = torch.zeros(L5, B5, dtype=torch.uint8, device=dev)
        logits5 = torch.zeros(L5, B5, 2, dtype=torch.float32, device=dev)
        ones5 = torch.ones(L5, B5, dtype=torch.uint8, device=dev)

        def prefill5(mask_dev, route):
            for l in range(L5):
                if route:
                    F.flux_router(ctx, q5, cu5, B5, hidden, pool, w1_5[0, l], None, w2_5[0, l], None, inner, mask_dev[l],
                                  logits5[l])
                caches5[l].kv_len.zero_()
                F.flux_kv_append(ctx, caches5[l], HKV, D, k5[0], v5[0], cu5, T5, smax5)
                F.flux_attn_prefill(ctx, cfg, q5[0], cu5, smax5, smax5, caches5[l], mask_dev[l], out5)

        t5_mix = timed(lambda: prefill5(routed, True), 2 if long_form else 1)
        t5_fa = timed(lambda: prefill5(ones5, False), 1, warm=long_form)
        margin5 = float((logits5[..., 0] - logits5[..., 1]).abs().min())
        mask5 = routed.cpu().numpy()                       # read once after prefill: sizes the decode launches
        w_fa = {n: 4.0 * D * HQ * pairs_fa(n) for n in lens5}
        w_sa = {n: 4.0 * D * HQ * pairs_sa(n) for n in lens5}
        work_fa = L5 * sum(w_fa.values())
        work_mix = sum(w_fa[lens5[b]] if mask5[l, b] else w_sa[lens5[b]] for l in range(L5) for b in range(B5))

        qd5 = torch.empty(1, L5, B5 * HQ, D, dtype=torch.bfloat16, device=dev)
        kd5 = torch.empty(1, L5, B5 * HKV, D, dtype=torch.bfloat16, device=dev)
        vd5 = torch.empty(1, L5, B5 * HKV, D, dtype=torch.bfloat16, device=dev)
        synth_gpu.fill_normal_bf16(qd5, SEED5, synth.stream_id(synth.STREAM_QDEC))
        synth_gpu.fill_normal_bf16(kd5, SEED5, synth.stream_id(synth.STREAM_KDEC))
        synth_gpu.fill_normal_bf16(vd5, SEED5, synth.stream_id(synth.STREAM_VDEC))
        outd5 = torch.empty(B5, HQ, D, dtype=torch.bfloat16, device=dev)
        cu1_5 = i32(list(range(B5 + 1)))
        grown = {"n": 0}

        def decode5(mask_host, mask_dev):
            grown["n"] += 1
            for l in range(L5):
                F.flux_kv_append(ctx, caches5[l], HKV, D, kd5[0, l], vd5[0, l], cu1_5, B5, 1)
                # the launch is sized for the longest sequence that needs its whole cache in this layer
                need = [lens5[b] + grown["n"] if mask_host[l, b] else min(lens5[b] + grown["n"], NS + W) for b in range(B5)]
                F.flux_attn_decode(ctx, cfg, qd5[0, l], max(need), caches5[l], mask_dev[l], outd5)

        def decode_run(mask_host, mask_dev, steps):
            for _ in range(8):
                decode5(mask_host, mask_dev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                decode5(mask_host, mask_dev)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

        td5_mix = decode_run(mask5, routed, n_steps5)
        n_steps5_fa = n_steps5 // 4
        td5_fa = decode_run(np.ones_like(mask5), ones5, n_steps5_fa)
        rb = 2.0 * HKV * D * 2
        by_fa = L5 * sum(rb * n for n in lens5)
        by_mix = sum(rb * (lens5[b] if mask5[l, b] else min(lens5[b], NS + W)) for l in range(L5) for b in range(B5))
        extra["routed_end_to_end"] = {
            "workload": "%d layers, ragged batch %s (%d tokens), %d/%d heads, D %d, router %d->%d->SiLU->2 with N(0, 0.02) "
                        "weights per layer on the query tensor (pool %d + %d rows), %d sinks + %d window, seed %d, "
                        "prefill then %d decode steps" % (L5, lens5, T5, HQ, HKV, D, hidden, inner, pool, pool, NS, W, SEED5, n_steps5),
            "omega_msr": float((mask5 == 0).mean()),
            "sa_layers_per_sequence": [int((mask5[:, b] == 0).sum()) for b in range(B5)],
            "router_min_logit_margin": margin5,
            "router_min_logit_margin_note": "min |pi_FA - pi_SA| over the %d (sequence, layer) decisions, fp32 logits of "
                                            "the device; decisions are bit-exact against the fp64 oracle above 1e-6" % (L5 * B5),
            "prefill_timed_steps_routed_and_all_fa": [2 if long_form else 1, 1],
            "decode_timed_steps_routed_and_all_fa": [n_steps5, n_steps5_fa],
            "prefill_ms_routed": t5_mix * 1e3, "prefill_ms_all_fa": t5_fa * 1e3,
            "prefill_tokens_per_s_routed": T5 / t5_mix, "prefill_tokens_per_s_all_fa": T5 / t5_fa,
            "prefill_speedup": t5_fa / t5_mix, "prefill_predicted_speedup_from_flops": work_fa / work_mix,
            "prefill_all_fa_tflops": work_fa / t5_fa / 1e12,
            "decode_ms_per_step_routed": td5_mix * 1e3, "decode_ms_per_step_all_fa": td5_fa * 1e3,
            "decode_speedup": td5_fa / td5_mix, "decode_predicted_speedup_from_bytes": by_fa / by_mix,
            "decode_all_fa_gbs": by_fa / td5_fa / 1e9}
        del q5, k5, v5, out5, caches5
        torch.cuda.empty_cache()

    status = F.flux_last_device_status(ctx)
    F.flux_destroy(ctx)

    t_step = prefill["ms_per_step_mix"] if prefill else None
    line = {
        "metric": "prefill tokens/s and decode ms/step at 1 MI355X; speedup vs all-FA; % MFMA / HBM peak",
        "value": prefill["tokens_per_s_mix"] if prefill else None,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "stack prefill: %d layers, batch 1, seq_len %d, %d/%d heads, D %d, bf16 N(0,1) x per-head "
                               "U(0.5,2) scales, seed %d, %d of %d layers SA (%d sinks + %d window), fp32 accumulate"
                               % (L, S, HQ, HKV, D, SEED, N_SA, L, NS, W),
                   "layers": L, "batch": 1, "seq_len": S, "n_q_heads": HQ, "n_kv_heads": HKV, "head_dim": D,
                   "n_sink": NS, "window": W, "sa_layers": N_SA},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
        "prefill": prefill, "decode": decode, "router": router, "context_length_sweep": sweep, "extra_workloads": extra, "device_status": status,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
