#!/usr/bin/env python3
"""Headline benchmark: fused Quest select+attend decode on the recurrence-augmented KV
cache, OLMo2-7B-shaped layer (32 heads MHA, D=128), batch 4, 64K context, 16-token
pages, budget 1/16, one MI355X.

One step = one decode step of the layer's attention path for the whole batch:
rat_scan append of the new token (Eq. 1) with the page-metadata update of the touched page,
fused page selection + attention over the selected pages (Eq. 3-4).  The prefill scan
and bulk page metadata that build the 64K cache run once before the timed region and
are reported under "extra".  Prints ONE JSON line.
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

HBM_PEAK = 8.0e12  # B/s, MI355X published HBM3E bandwidth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="C3", choices=["C3", "C2"])
    ap.add_argument("--budget", type=float, default=1 / 16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=512)
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB device copy (the known-size kernel that scales "
                         "the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (every box has one; the path shards over batch "
              "and heads with no exchange, see DESIGN.md). --gpus %d is not supported." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_28640_amd import binding as rs
    from paper_2605_28640_amd import synth

    rs.load()  # raises if the HIP library is not built: there is no fallback
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = {"C3": synth.C3, "C2": synth.C2}[args.workload]
    B, Hq, Hkv, D, T, P = w.B, w.Hq, w.Hkv, w.D, w.T, w.P
    n_steps_total = args.warmup + args.steps
    Tcap = ((T + max(1024, n_steps_total + 16) + P - 1) // P) * P
    K = int(round(args.budget * (T // P)))
    n_first, n_local = 1, 1
    scale = 1.0 / math.sqrt(D)
    dt = torch.bfloat16
    s = rs.make_shape(B, Hq, Hkv, D, Tcap, P, dt)

    def log(*a):
        print("[bench]", *a, file=sys.stderr, flush=True)

    # ---- inputs (seeded, synthetic, needle-structured) -------------------------------
    t_gen = time.time()
    k, v, g = synth.prefill(w)
    log("generated prefill inputs in %.1fs" % (time.time() - t_gen))
    tk = torch.from_numpy(k).to(dev).to(dt)
    tv = torch.from_numpy(v).to(dev).to(dt)
    tg = torch.from_numpy(g).to(dev)
    keep_host = not args.no_cpu_baseline
    if not keep_host:
        del k, v, g
    steps_in = [synth.decode_step(w, i) for i in range(n_steps_total + args.cpu_steps)]
    dk = torch.from_numpy(np.stack([x[0] for x in steps_in])).to(dev).to(dt)
    dv = torch.from_numpy(np.stack([x[1] for x in steps_in])).to(dev).to(dt)
    dg = torch.from_numpy(np.stack([x[2] for x in steps_in])).to(dev)
    dq = torch.from_numpy(np.stack([x[3] for x in steps_in])).to(dev).to(dt)

    kc = torch.zeros(B, Hkv, Tcap, D, dtype=dt, device=dev)
    vc = torch.zeros_like(kc)
    meta = torch.zeros(B, Hkv, Tcap // P, 2, D, dtype=dt, device=dev)
    sk = torch.zeros(B, Hkv, D, device=dev)
    sv = torch.zeros_like(sk)
    out = torch.zeros(B, Hq, D, dtype=dt, device=dev)
    ws = rs.Workspace(max(rs.rat_scan_workspace_bytes(s, T),
                          rs.sparse_attn_decode_workspace_bytes(s, Tcap, max(K, (T // P) // 4))))

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- prefill: chunked scan + bulk page metadata (outside the timed region) -------
    extra = {}
    e0, e1, e2 = ev(), ev(), ev()
    torch.cuda.synchronize()
    e0.record()
    rs.rat_scan(s, tk, tv, tg, sk, sv, kc, vc, 0, T, ws)
    e1.record()
    rs.quest_page_meta(s, kc, meta, 0, T)
    e2.record()
    torch.cuda.synchronize()
    ws.async_status()
    scan_ms, meta_ms = e0.elapsed_time(e1), e1.elapsed_time(e2)
    scan_bytes = B * Hkv * T * D * 12  # read k, v (bf16) and g (f32); write k~, v~ (bf16)
    meta_bytes = B * Hkv * T * D * 2 + B * Hkv * (T // P) * 2 * D * 2
    extra["rat_scan_prefill"] = {"ms": round(scan_ms, 4), "GB/s": round(scan_bytes / scan_ms / 1e6, 1),
                                 "frac_hbm_peak": round(scan_bytes / (scan_ms * 1e-3) / HBM_PEAK, 4),
                                 "algorithmic_bytes": scan_bytes, "note": "first (cold) call"}
    extra["quest_page_meta_bulk"] = {"ms": round(meta_ms, 4), "GB/s": round(meta_bytes / meta_ms / 1e6, 1),
                                     "frac_hbm_peak": round(meta_bytes / (meta_ms * 1e-3) / HBM_PEAK, 4)}
    state_after_prefill = (sk.clone(), sv.clone())
    del tk, tv, tg
    torch.cuda.empty_cache()
    log("prefill scan %.3f ms, bulk meta %.3f ms" % (scan_ms, meta_ms))

    # ---- decode loop ---------------------------------------------------------------
    def decode_step(i, events=None):
        t = T + i
        rs.rat_scan(s, dk[i], dv[i], dg[i], sk, sv, kc, vc, t, 1, None, meta)  # append + page-meta update
        if events is not None:
            events[0].record()
        rs.sparse_attn_decode(s, dq[i], kc, vc, t + 1, scale, None, K, meta, n_first, n_local, out,
                              None, None, ws)
        if events is not None:
            events[1].record()

    for i in range(args.warmup):
        decode_step(i)
    pairs = [(ev(), ev()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(args.steps):
        decode_step(args.warmup + j, pairs[j])
    host_enqueue = time.perf_counter() - t0
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    log("host enqueue time %.4f ms/step (GPU wall %.4f ms/step)" % (host_enqueue * 1e3 / args.steps,
                                                                     wall * 1e3 / args.steps))
    ws.async_status()
    fused_ms = [a.elapsed_time(b) for a, b in pairs]
    ms_per_step = wall * 1e3 / args.steps
    tok_s = B * args.steps / wall

    # algorithmic bytes of the fused select+attend launch pair, per step
    def fused_bytes(Tv):
        Np = (Tv + P - 1) // P
        per_unit = Np * 2 * D * 2 + K * P * D * 2 * 2  # all page metadata + selected K and V pages
        return B * Hq * per_unit + B * Hq * D * 2 * 2  # + q and out
    bytes_per_step = [fused_bytes(T + args.warmup + j + 1) for j in range(args.steps)]
    mean_bytes = sum(bytes_per_step) / len(bytes_per_step)
    mean_fused_ms = sum(fused_ms) / len(fused_ms)
    achieved = mean_bytes / (mean_fused_ms * 1e-3)
    # HBM bytes per launch from the committed rocprofv3 counter summary of this workload
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "decode_fused_%s_budget_1_16_hbm_traffic.md" % args.workload)
    if os.path.exists(tpath) and abs(args.budget - 1 / 16) < 1e-9:
        import re
        m = re.search(r"^hbm_bytes_per_launch\s*=\s*(\d+)", open(tpath).read(), re.M)
        traffic = int(m.group(1)) if m else None
    roofline = {"bound": "hbm", "kernel": "decode_fused_kernel (sparse_attn_decode, fused select+attend, one launch per step)",
                "achieved": round(achieved / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK, 4), "traffic": traffic,
                "algorithmic_bytes_per_step": int(mean_bytes), "mean_ms": round(mean_fused_ms, 5),
                "min_ms": round(min(fused_ms), 5), "median_ms": round(sorted(fused_ms)[len(fused_ms) // 2], 5)}
    log("decode: %.4f ms/step wall, fused pair %.4f ms mean -> %.0f GB/s (%.1f%% of HBM peak)" %
        (ms_per_step, mean_fused_ms, achieved / 1e9, 100 * achieved / HBM_PEAK))

    # ---- extra: other budgets and the dense path on the same cache (not the headline) --
    if not args.no_extra:
        Tv = T + n_steps_total
        qx = dq[0]
        for name, Kx, use_meta in (("fused_budget_1_4", (T // P) // 4, True), ("dense_full_budget", 0, False)):
            for _ in range(3):
                rs.sparse_attn_decode(s, qx, kc, vc, Tv, scale, None, Kx, meta if use_meta else None, 1, 1, out,
                                      None, None, ws)
            a, b = ev(), ev()
            reps = 10
            a.record()
            for _ in range(reps):
                rs.sparse_attn_decode(s, qx, kc, vc, Tv, scale, None, Kx, meta if use_meta else None, 1, 1, out,
                                      None, None, ws)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            Np = (Tv + P - 1) // P
            byt = B * Hq * ((Np * 2 * D * 2 + Kx * P * D * 4) if use_meta else Tv * D * 4)
            extra[name] = {"ms": round(ms, 4), "GB/s": round(byt / ms / 1e6, 1),
                           "frac_hbm_peak": round(byt / (ms * 1e-3) / HBM_PEAK, 4), "tok/s": round(B / (ms * 1e-3), 1)}

    if args.calibrate:
        src = torch.empty(1 << 29, dtype=dt, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the test oracle, as it stands, on this machine's host cores ----------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t_c = time.time()
        hk = kc.to(torch.float32).cpu().numpy()
        hv = vc.to(torch.float32).cpu().numpy()
        hmeta = meta.to(torch.float32).cpu().numpy()
        osk = sk.double().cpu().numpy()
        osv = sv.double().cpu().numpy()
        log("copied cache to host in %.1fs" % (time.time() - t_c))
        worst = 0.0
        sel_equal = 0
        t_cpu = 0.0
        idx_gpu = torch.zeros(B, Hq, K, dtype=torch.int32, device=dev)
        for c in range(args.cpu_steps):
            i = n_steps_total + c
            t = T + i
            kd, vd, gd, qd = steps_in[i]
            t1 = time.perf_counter()
            ko, vo, osk, osv = oracle.rat_scan(kd, vd, gd, osk, osv)
            hk[:, :, t] = oracle.round_to_bf16(ko[:, :, 0])
            hv[:, :, t] = oracle.round_to_bf16(vo[:, :, 0])
            p = t // P
            hmeta[:, :, p] = oracle.quest_page_meta(hk[:, :, p * P:(p + 1) * P], P, t - p * P + 1)[:, :, 0]
            Np = (t + 1 + P - 1) // P
            sc = oracle.quest_scores(qd, hmeta, Np)
            oidx = oracle.quest_select(sc, K, n_first, n_local)
            oout, _ = oracle.sparse_attn_decode(qd, hk, hv, P, t + 1, scale, oidx)
            t_cpu += time.perf_counter() - t1
            # the same step on the GPU, checked against the oracle
            rs.rat_scan(s, dk[i], dv[i], dg[i], sk, sv, kc, vc, t, 1, None, meta)
            rs.sparse_attn_decode(s, dq[i], kc, vc, t + 1, scale, None, K, meta, n_first, n_local, out, None,
                                  idx_gpu, ws)
            torch.cuda.synchronize()
            got = out.to(torch.float32).cpu().numpy()
            ref = np.maximum(np.abs(oout).max(-1), np.sqrt((oout ** 2).mean(-1)))
            worst = max(worst, float((np.abs(got - oout).max(-1) / ref).max()))
            sel_equal += int(np.array_equal(idx_gpu.cpu().numpy(), oidx))
        cpu = {"value": round(B * args.cpu_steps / t_cpu, 2), "unit": "tok/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "%d full decode steps of the same workload (all %d (batch, head) units: scan append, page "
                         "meta update, page scores, top-K, attention over %d pages), continuing the timed run's cache"
                         % (args.cpu_steps, B * Hq, K),
               "seconds": round(t_cpu, 2), "gpu_vs_oracle_max_rel_err": round(worst, 5),
               "gpu_selection_identical_steps": "%d/%d" % (sel_equal, args.cpu_steps)}

    line = {
        "metric": "sparse decode tok/s + % HBM peak, OLMo2-7B-shaped layer @64K ctx, 1/16 budget",
        "value": round(tok_s, 1), "unit": "tok/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: one decode layer, B=%d, Hq=%d, Hkv=%d, D=%d, context %d (+1 per step), "
                               "%d-token pages, K=%d of %d pages (budget %.4g), first+last page kept"
                               % (w.name, B, Hq, Hkv, D, T, P, K, T // P, args.budget),
                   "step": "rat_scan append (with page-meta update) + fused select/attend, two launches; tok/s is for ONE layer "
                           "(a 32-layer model divides it by 32)",
                   "pct_hbm_peak": round(100 * achieved / HBM_PEAK, 2)},
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
