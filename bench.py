#!/usr/bin/env python3
"""Benchmark of the Compact NGP encoding path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: bake (argmax of the confidence values into the index codebook), forward
encoding, backward pass (gradient arrays cleared, then accumulated).  The default workload
is the 3D NeRF-shaped configuration the headline metric is quoted on (d = 3, L = 16, F = 2,
N_f = 2^16, N_c = 2^14, N_p = 16, 2^18 points = 4096 rays x 64 samples, fp16 features and I/O).

Prints ONE JSON line: throughput in encoded points/s, the roofline of the dominant kernel
(algorithmic bytes per launch / its average duration measured with HIP events on the launch
stream, against the 8 TB/s HBM peak) and the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def algorithmic_bytes(w, n, index_level_bytes=None):
    """Compulsory HBM bytes per launch of each kernel kind: every input read once, every output
    written once (tables included; random re-reads of cached rows are not algorithmic)."""
    fb = 2 if w.feat_dtype == "f16" else 4
    iob = 2 if w.io_dtype == "f16" else 4
    D_f = w.L * w.N_f * w.F * fb
    D_c = w.L * (w.N_c if index_level_bytes is None else index_level_bytes)
    Dhat = w.L * w.N_c * w.N_p * 4
    gD_f = w.L * w.N_f * w.F * 4
    pts = n * (4 * w.d + w.L * w.F * iob)
    return {
        "encode_fwd": pts + D_f + D_c,
        # inference in one kernel: the points in, three fp32 outputs per point out, tables and decoder weights once
        "encode_mlp_fwd": n * (4 * w.d + 3 * 4) + D_f + D_c + 2 * (64 * w.L * w.F + 64 * 64 + 64 * 3),
        "encode_bwd": pts + D_f + Dhat + gD_f + Dhat,
        "bake_probes": Dhat + D_c,
        "zero": gD_f + Dhat,
        # parameters, two moments and the gradient read, the first three written, for both tables;
        # plus the storage copy of D_f when that is fp16, plus D_c
        "adam_step_bake": 7 * (gD_f + Dhat) + (D_f if fb == 2 else 0) + D_c,
    }



def sources_sha16():
    """Hash of the library's sources: profiles/hbm_traffic.json is only quoted while it was measured on these."""
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2312_17241_amd", "csrc")
    kernel_sources = [f for f in sorted(os.listdir(base)) if not f.endswith("_main.cpp")]     # (not the host-only check program)
    for f in kernel_sources + [os.path.join("..", "..", "include", "cngp.h")]:
        h.update(open(os.path.join(base, f), "rb").read())
    return h.hexdigest()[:16]


def distinct_vertices(np, x_h, res, sample=1 << 20):
    """Per level: the grid vertices the batch touches and its corner references, counting only corners whose
    interpolation weight is not exactly zero (a point on a face of its cell has corners that contribute nothing, in
    either direction; the kernels skip them, so the bound must not count them either).  Exact up to `sample` points; a
    larger batch is extrapolated from its first `sample` points with the occupancy law V(R) = G (1 - exp(-R / G)), G
    fitted to the sample.  Measurement of the input, used only for the roofline.  Returns (vertices, references)."""
    n, d = x_h.shape
    xs = x_h[:sample]
    out_v, out_r = [], []
    for nl in res:
        pos = xs * np.float32(nl)                                 # fp32 product, as the kernels form it
        fl = np.floor(pos)
        on_face = (pos - fl) == 0                                 # fraction exactly zero along that axis
        v0 = fl.astype(np.int64)
        ids = []
        for c in range(1 << d):
            bits = [(c >> i) & 1 for i in range(d)]
            v = v0 + np.array(bits, dtype=np.int64)
            dead = np.zeros(xs.shape[0], dtype=bool)              # weight zero: an upper corner along an axis with fraction 0
            for i in range(d):
                if bits[i]:
                    dead |= on_face[:, i]
            vid = v[:, 0]
            for i in range(1, d):
                vid = vid * (int(nl) + 2) + v[:, i]
            ids.append(vid[~dead])
        ids = np.concatenate(ids)
        V = int(np.unique(ids).size)
        R = int(ids.size)
        if n > xs.shape[0] and V < R:
            lo, hi = float(V), float(V) * 1e6                 # solve G (1 - exp(-R / G)) = V for G by bisection
            for _ in range(200):
                G = 0.5 * (lo + hi)
                if G * -np.expm1(-R / G) < V:
                    lo = G
                else:
                    hi = G
            R = int(R * (n / xs.shape[0]))
            V = int(G * -np.expm1(-R / G))
        elif n > xs.shape[0]:
            R = int(R * (n / xs.shape[0]))
            V = R
        out_v.append(V)
        out_r.append(R)
    return out_v, out_r


def level_rooflines(w, n, index_level_bytes, res, V, refs, rates, fwd_only, lds_share=0.0):
    """The applicable roofline, level by level: t_l = max(t_stream, t_rand, t_atomic), summed over the levels.
      t_stream  the level's share of the compulsory bytes (points and outputs split evenly over the levels, the
                level's own tables) at the measured streaming rate of a cache-resident working set
      t_rand    rows that must be fetched at random AFTER reuse -- min(corner references, distinct vertices touched)
                per table -- at the measured random gather rate of the cache level that holds the level's tables
                (forward: one feature entry per vertex; backward: one softmax row and one feature row per vertex).
                Forward with the level-resident kernel: the share `lds_share` of a level's feature codebook that a
                CU's LDS holds is looked up there -- every reference, LDS has no reuse to offer -- at the measured
                random LDS read rate, the rest as above
      t_atomic  backward: every row of the two gradient tables that is touched must reach memory at least once,
                at the measured rate of global atomic row updates
    Times in microseconds."""
    fb = 2 if w.feat_dtype == "f16" else 4
    iob = 2 if w.io_dtype == "f16" else 4
    near = 4 << 20                                            # one XCD's L2
    rows = []
    for l in range(w.L):
        R = refs[l]                                           # corner references of weight != 0
        reused = min(R, V[l])
        D_f_l, D_c_l = w.N_f * w.F * fb, index_level_bytes
        Dhat_l, gD_f_l = w.N_c * w.N_p * 4, w.N_f * w.F * 4
        pts = n * (4 * w.d / w.L + w.F * iob)
        f_stream = (pts + D_f_l + D_c_l) / rates["copy_GBps"] * 1e-3
        f_rand = (1.0 - lds_share) * reused / (rates["gather4_Gps"] if D_f_l <= near else rates["gather4_far_Gps"]) * 1e-3
        if lds_share > 0.0:
            f_rand += lds_share * R / rates["lds_gather4_Gps"] * 1e-3
        row = {"level": l, "N_l": int(res[l]), "refs": R, "distinct_vertices": int(V[l]),
               "fwd": {"t_stream_us": round(f_stream, 3), "t_rand_us": round(f_rand, 3),
                       "t_roof_us": round(max(f_stream, f_rand), 3), "binds": "stream" if f_stream >= f_rand else "rand"}}
        if not fwd_only:
            b_stream = (pts + D_f_l + 2 * Dhat_l + gD_f_l) / rates["copy_GBps"] * 1e-3
            gather = rates["row_gather_Gps"] if D_f_l + Dhat_l <= near else rates["row_gather_far_Gps"]
            b_rand = (2 if w.N_p > 1 else 0) * reused / gather * 1e-3
            segs = min(reused, w.N_f // w.N_p) * max(1, w.N_p * w.F * 4 // 64) + (min(reused, w.N_c) * max(1, w.N_p * 4 // 64) if w.N_p > 1 else 0)
            b_atomic = segs / rates["global_atomic_Gseg"] * 1e-3
            t = max(b_stream, b_rand, b_atomic)
            row["bwd"] = {"t_stream_us": round(b_stream, 3), "t_rand_us": round(b_rand, 3), "t_atomic_us": round(b_atomic, 3),
                          "t_roof_us": round(t, 3), "binds": "stream" if t == b_stream else "rand" if t == b_rand else "atomic"}
        rows.append(row)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="nerf3d", help="nerf3d (headline) | image2d | sdf3d | tiny2d | infer3d | infer3d_plain | compact3d")
    ap.add_argument("--bwd", default="auto", choices=["auto", "direct", "sliced", "binned"],
                    help="force a variant of the backward pass (default: the library's own choice)")
    ap.add_argument("--with-optimizer", action="store_true",
                    help="a step becomes: Adam step fused with the bake (replaces the bake), forward, backward; "
                         "the tables then change from step to step.  Not the headline configuration.")
    ap.add_argument("--with-decoder", action="store_true",
                    help="adds the 64-wide decoder after the encoding: forward, residual against a fixed random target, "
                         "backward (its dL/dy feeds the encoding's backward), and with --with-optimizer its Adam step.  "
                         "Not the headline configuration.")
    ap.add_argument("--top-k", type=int, default=0, metavar="K",
                    help="backward: softmax over the K largest confidence values of a row only (the sparse variant; "
                         "0 = the paper's dense softmax, the headline)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements reported beside the headline: per-step median / min, cold caches, "
                         "Morton-ordered points")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one plain device-to-device copy of this many MiB (reads and writes that many "
                         "bytes): the reference that rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2312_17241_amd as cngp
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = W.WORKLOADS[args.workload]
    fwd_only = args.workload in ("infer3d", "infer3d_plain", "compact3d")
    fmt = {"infer3d": cngp.IDX_PACKED4, "compact3d": cngp.IDX_BITS}.get(args.workload, cngp.IDX_U8)
    bwd_flag = {"auto": 0, "direct": cngp.BWD_DIRECT, "sliced": cngp.BWD_SLICED, "binned": cngp.BWD_BINNED}[args.bwd]
    cfg = cngp.Config.from_workload(w, index_format=fmt, flags=cngp.ZERO_GRADS | bwd_flag, top_k=args.top_k)

    x_h = W.make_points(w)
    D_f_h = W.make_feature_codebook(w)
    Dhat_h = W.make_probe_logits(w)
    N = x_h.shape[0]
    x = torch.from_numpy(x_h).to(dev)
    D_f = torch.from_numpy(D_f_h).to(dev)
    Dhat = torch.from_numpy(Dhat_h).to(dev)
    D_c = torch.empty((w.L, cfg.index_cols), dtype=torch.uint8, device=dev)
    y = torch.empty((N, w.L * w.F), dtype=torch.float16 if w.io_dtype == "f16" else torch.float32, device=dev)
    ws = cngp.alloc_workspace(cfg, N, dev)
    if not fwd_only:
        dy_h = W.make_upstream_grad(w)
        dy = torch.from_numpy(dy_h).to(dev)
        gF = torch.empty((w.L, w.N_f, w.F), dtype=torch.float32, device=dev)
        gC = torch.empty((w.L, w.N_c, w.N_p), dtype=torch.float32, device=dev)

    with_opt = args.with_optimizer and not fwd_only
    if with_opt:
        half = w.feat_dtype == "f16"
        master = D_f.float()
        D_f_arg = D_f if half else None
        if not half:
            D_f = master
        moments = [torch.zeros_like(master), torch.zeros_like(master), torch.zeros_like(Dhat), torch.zeros_like(Dhat)]
        gF.zero_(); gC.zero_()
        cfg_opt = cngp.Config.from_workload(w, index_format=fmt)
        n_step = [0]

    fused_dec = args.with_decoder and fwd_only              # inference: encoding + decoder in one call
    if fused_dec:
        mcfg = cngp.MlpConfig(w.L * w.F, 3, cngp.F16 if w.io_dtype == "f16" else cngp.F32)
        g = torch.Generator(device="cpu").manual_seed(7)
        W_half = torch.cat([(torch.randn((r, c), generator=g) * (2.0 / c) ** 0.5).ravel()
                            for r, c in ((64, w.L * w.F), (64, 64), (3, 64))]).to(dev).half()
        out_dec = torch.empty((N, 3), dtype=torch.float32, device=dev)
    with_dec = args.with_decoder and not fwd_only
    if with_dec:
        n_out = 3
        mcfg = cngp.MlpConfig(w.L * w.F, n_out, cngp.F16 if w.io_dtype == "f16" else cngp.F32, flags=cngp.ZERO_GRADS)
        g = torch.Generator(device="cpu").manual_seed(7)
        W_master = torch.cat([(torch.randn((r, c), generator=g) * (2.0 / c) ** 0.5).ravel()
                              for r, c in ((64, w.L * w.F), (64, 64), (n_out, 64))]).to(dev)
        W_half = W_master.half()
        W_m, W_v, W_g = torch.zeros_like(W_master), torch.zeros_like(W_master), torch.zeros_like(W_master)
        target = torch.rand((N, n_out), generator=g).to(dev)
        out_dec = torch.empty((N, n_out), dtype=torch.float32, device=dev)
        dout = torch.empty_like(out_dec)
        loss_scale = 128.0

    def step():
        if with_dec:
            if with_opt:
                cngp.adam_step(cngp.Adam(lr=1e-3, eps=1e-15, grad_scale=1 / loss_scale, step=n_step[0] + 1),
                               W_master, W_half, W_m, W_v, W_g)
        if with_opt:
            n_step[0] += 1
            opt = cngp.Adam(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-15, step=n_step[0],
                            grad_scale=(1 / loss_scale) if with_dec else 1.0)
            cngp.adam_step_bake(cfg_opt, opt, opt, (master, D_f_arg, moments[0], moments[1], gF),
                                (Dhat, moments[2], moments[3], gC, D_c))
        else:
            cngp.bake_probes(cfg, Dhat, D_c)
        if fused_dec:
            cngp.encode_mlp_fwd(cfg, mcfg, x, D_f, D_c, W_half, out_dec, workspace=ws)
            return
        cngp.encode_fwd(cfg, x, D_f, D_c, y, workspace=ws)
        if with_dec:
            cngp.mlp_fwd(mcfg, y, W_half, out_dec)
            torch.sub(out_dec, target, out=dout)                      # residual of an L2 loss: plumbing, two tiny torch kernels
            dout.mul_(2.0 * loss_scale / dout.numel())
            cngp.mlp_bwd(mcfg, y, W_half, dout, dy, W_g)              # writes dL/dy for the encoding
        if not fwd_only:
            cngp.encode_bwd(cfg, x, D_f, Dhat, dy, gF, gC, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # timed region: exactly K steps, nothing else on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = N * args.steps / (t1 - t0)

    # The same K steps again, now with every kernel bracketed by HIP events on its launch stream: the
    # per-kernel durations the roofline is computed from.  The event records themselves cost a few
    # microseconds per launch (about 6 % of a step), which is why they are kept out of the timed region;
    # the step time of this pass is reported as "ms_per_step_with_events".
    cngp.profile_enable(True)
    cngp.profile_read()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    kernels = cngp.profile_read()
    cngp.profile_enable(False)

    # Beside the headline (never part of `value`): the spread of single steps, the same step with cold caches,
    # and the same batch in Morton order.
    extras = {}
    morton_perm = None
    if not args.no_extras:
        def steps_with_events(k, before=None):
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(k)]
            for a, b in ev:
                if before is not None:
                    before()
                a.record()
                step()
                b.record()
            torch.cuda.synchronize()
            return sorted(a.elapsed_time(b) for a, b in ev)

        t = steps_with_events(min(args.steps, 50))
        extras["single_steps_ms"] = {"median": round(t[len(t) // 2], 4), "min": round(t[0], 4), "n": len(t),
                                     "note": "each step bracketed by its own pair of events on the launch stream"}
        # cold: 512 MiB written between steps pushes tables, points and workspace out of L2 and the 256 MB memory-side cache
        scrub = torch.empty(1 << 29, dtype=torch.uint8, device=dev)
        t = steps_with_events(10, before=lambda: scrub.fill_(1))
        del scrub
        extras["cold_cache"] = {"ms_per_step_median": round(t[len(t) // 2], 4), "ms_per_step_min": round(t[0], 4), "n": len(t),
                                "value": round(N / (t[len(t) // 2] * 1e-3), 1), "unit": "points/s",
                                "note": "512 MiB scrub buffer written before every step"}
        if not with_opt and not args.with_decoder and w.io_dtype == "f16":
            # the same step with fp32 encodings and upstream gradients (y, dL/dy): twice the streamed bytes
            w32 = W.custom(name=w.name + "_f32io", cfg=w.cfg, d=w.d, L=w.L, F=w.F, N_f=w.N_f, N_c=w.N_c, N_p=w.N_p,
                           N_min=w.N_min, N_max=w.N_max, N=N, feat_dtype=w.feat_dtype, io_dtype="f32", points=w.points)
            cfg32 = cngp.Config.from_workload(w32, index_format=fmt, flags=cngp.ZERO_GRADS | bwd_flag, top_k=args.top_k)
            y32 = torch.empty((N, w.L * w.F), dtype=torch.float32, device=dev)
            ws32 = cngp.alloc_workspace(cfg32, N, dev)
            dy32 = None if fwd_only else dy.float()
            def step32():
                cngp.bake_probes(cfg32, Dhat, D_c)
                cngp.encode_fwd(cfg32, x, D_f, D_c, y32, workspace=ws32)
                if not fwd_only:
                    cngp.encode_bwd(cfg32, x, D_f, Dhat, dy32, gF, gC, workspace=ws32)
            for _ in range(args.warmup):
                step32()
            torch.cuda.synchronize()
            f0 = time.perf_counter()
            for _ in range(args.steps):
                step32()
            torch.cuda.synchronize()
            f1 = time.perf_counter()
            extras["fp32_io"] = {"value": round(N * args.steps / (f1 - f0), 1), "unit": "points/s",
                                 "ms_per_step": round((f1 - f0) * 1e3 / args.steps, 4),
                                 "note": "y and dL/dy as fp32 instead of fp16, everything else as in the headline"}
            del y32, ws32, dy32
            step()                                               # gF, gC, D_c of the headline configuration again
        if not with_opt and not args.with_decoder:
            # Morton order (cngp_morton_sort): the same batch with its points sorted along the Z-order curve
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            sort_ws = torch.empty(int(cngp._lib.cngp_morton_sort_workspace_bytes(w.d, N)), dtype=torch.uint8, device=dev)
            for attempt in range(3):                             # the last of three is the one reported
                e0.record()
                perm, x_sorted = cngp.morton_sort(x, workspace=sort_ws)
                e1.record()
                torch.cuda.synchronize()
            sort_ms = e0.elapsed_time(e1)
            morton_perm = perm.cpu().numpy()                     # compared with the oracle's order in the check below
            note = "the sort is the library's (cngp_morton_sort) and is not part of these steps"
            if fwd_only and not fused_dec:
                # inference: the whole pipeline -- sort, then the forward pass that writes y in the caller's order
                def sorted_step():
                    cngp.bake_probes(cfg, Dhat, D_c)
                    p_, xs_ = cngp.morton_sort(x, workspace=sort_ws)
                    cngp.encode_fwd_permuted(cfg, xs_, p_, D_f, D_c, y, workspace=ws)
                y_plain = y.clone()
                for _ in range(args.warmup):
                    sorted_step()
                torch.cuda.synchronize()
                m0 = time.perf_counter()
                for _ in range(args.steps):
                    sorted_step()
                torch.cuda.synchronize()
                m1 = time.perf_counter()
                assert torch.equal(y.view(torch.int16), y_plain.view(torch.int16)), "permuted forward differs from the plain one"
                note = "every step = bake + cngp_morton_sort + cngp_encode_fwd_permuted (y in the caller's order, identical bits)"
            else:
                x_nat, x = x, x_sorted
                dy_nat, dy = dy, dy.index_select(0, perm.long())
                for _ in range(args.warmup):
                    step()
                torch.cuda.synchronize()
                m0 = time.perf_counter()
                for _ in range(args.steps):
                    step()
                torch.cuda.synchronize()
                m1 = time.perf_counter()
                x, dy = x_nat, dy_nat
                step()                                           # y and the gradients of the natural order again, for the check
                torch.cuda.synchronize()
            del sort_ws
            extras["morton_order"] = {"value": round(N * args.steps / (m1 - m0), 1), "unit": "points/s",
                                      "ms_per_step": round((m1 - m0) * 1e3 / args.steps, 4),
                                      "sort_ms_gpu": round(sort_ms, 3), "note": note}

    # roofline of the dominant kernel kind
    alg = algorithmic_bytes(w, N, cfg.index_cols)
    per_kernel = {}
    for name, (ms, cnt) in kernels.items():
        kind = "encode_bwd" if name.startswith("encode_bwd") else "encode_fwd" if name in ("encode_fwd", "encode_fwd_rows") else name
        d = per_kernel.setdefault(kind, {"ms": 0.0, "launches": 0, "parts": {}})
        d["ms"] += ms
        d["launches"] += cnt
        d["parts"][name] = {"avg_us": round(ms * 1e3 / cnt, 2), "launches": cnt}
    dom = max(per_kernel, key=lambda k: per_kernel[k]["ms"])
    dom_ms_per_step = per_kernel[dom]["ms"] / args.steps        # all parts of that kind, per step
    achieved = alg[dom] / (dom_ms_per_step * 1e-3) / 1e9
    # HBM-side traffic of that kernel kind: rocprofv3 FETCH_SIZE / WRITE_SIZE of this same command, kept in
    # profiles/hbm_traffic.json with a hash of the library sources it was measured on; not quoted when stale
    traffic, traffic_note = None, "profiles/hbm_traffic.json has no entry for this workload"
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("_sources_sha16") != sources_sha16():
            traffic_note = "profiles/hbm_traffic.json was measured on other kernel sources: not quoted"
        elif f"{dom}:{args.workload}" in tj:
            traffic, traffic_note = tj[f"{dom}:{args.workload}"], "rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain 1 GiB copy"
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic, "traffic_note": traffic_note,
                "algorithmic_bytes_per_launch": alg[dom], "avg_launch_us": round(dom_ms_per_step * 1e3, 2)}

    out = {
        "metric": "encoded points/s fwd+bwd (d=3, L=16)" if not fwd_only else "encoded points/s fwd",
        "value": round(value, 1), "unit": "points/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_with_events": round((t3 - t2) * 1e3 / args.steps, 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "storage_dtypes": {"D_f": w.feat_dtype, "y_and_dy": w.io_dtype, "Dhat_c_and_gradients": "f32",
                           "note": "dtype is the arithmetic type: every product and sum is fp32 (fp64 in the LDS accumulators)"},
        "config": {"workload": f"{w.name}: d={w.d} L={w.L} F={w.F} N_f={w.N_f} N_c={w.N_c} N_p={w.N_p} "
                               f"N_min={w.N_min} N_max={w.N_max} points={N} ({w.points}) "
                               f"D_f={w.feat_dtype} y/dy={w.io_dtype}",
                   "step": ("bake + encoding and decoder forward in one call" if fused_dec else "bake + fwd") if fwd_only else
                           (("decoder fwd/bwd + " if with_dec else "") +
                            ("Adam step fused with bake + fwd + bwd (grads cleared each step)" if with_opt else
                             "bake + fwd + bwd (grads cleared each step)") +
                            (f"; sparse backward, top_k = {args.top_k}" if args.top_k else ""))},
        "roofline": roofline,
        "beside_the_headline": extras or None,
        "bwd_plan": None if fwd_only else cngp.bwd_plan_info(cfg, N),
        "fwd_plan": cngp.fwd_plan_info(cfg, N) if ws is not None else {"level_resident": 0},
        "kernels_us_per_step": {k: round(v["ms"] * 1e3 / args.steps, 2) for k, v in per_kernel.items()},
        "kernel_parts": {k: v["parts"] for k, v in per_kernel.items() if len(v["parts"]) > 1},
    }

    # Applicable roofline, level by level (level_rooflines above): the tables are cache resident, so what binds a level is
    # the larger of its streaming share, its random row fetches after reuse, and (backward) the gradient rows that must
    # reach memory.  Rates are measured now, on this device; every level is also timed alone through the same entry
    # points (an L = 1 configuration at that level's resolution with that level's tables).
    rates = cngp.measure_rates(dev)
    res = cngp.level_resolutions(cfg)
    V, refs = distinct_vertices(np, x_h, res)
    fplan = cngp.fwd_plan_info(cfg, N) if ws is not None else {"level_resident": 0}
    lds_share = fplan["resident_entries"] / w.N_f if fplan["level_resident"] else 0.0
    levels = level_rooflines(w, N, cfg.index_cols, res, V, refs, rates, fwd_only, lds_share)
    # (with the decoder: the one call runs the level-resident forward and the decoder kernel, or the one fused kernel)
    fwd_kinds = ("encode_mlp_fwd", "encode_fwd", "mlp_fwd") if fused_dec else ("encode_fwd",)
    t_fwd = sum(per_kernel[k]["ms"] for k in fwd_kinds if k in per_kernel) / args.steps * 1e3                # us
    if not args.no_extras:
        y_l = torch.empty((N, w.F), dtype=y.dtype, device=dev)
        for l, row in enumerate(levels):
            w_l = W.custom(name="level", cfg=w.cfg, d=w.d, L=1, F=w.F, N_f=w.N_f, N_c=w.N_c, N_p=w.N_p, N_min=int(res[l]),
                           N_max=int(res[l]), N=N, feat_dtype=w.feat_dtype, io_dtype=w.io_dtype, points=w.points)
            cfg_l = cngp.Config.from_workload(w_l, index_format=fmt, flags=cngp.ZERO_GRADS | bwd_flag, top_k=args.top_k)
            ws_l = cngp.alloc_workspace(cfg_l, N, dev)
            if not fwd_only:
                dy_l = dy[:, l * w.F:(l + 1) * w.F].contiguous()
            def one_level():
                cngp.encode_fwd(cfg_l, x, D_f[l:l + 1], D_c[l:l + 1], y_l, workspace=ws_l)
                if not fwd_only:
                    cngp.encode_bwd(cfg_l, x, D_f[l:l + 1], Dhat[l:l + 1], dy_l, gF[l:l + 1], gC[l:l + 1], workspace=ws_l)
            for _ in range(2):
                one_level()
            cngp.profile_enable(True)
            cngp.profile_read()
            for _ in range(5):
                one_level()
            torch.cuda.synchronize()
            kl = cngp.profile_read()
            cngp.profile_enable(False)
            row["fwd"]["alone_us"] = round(sum(ms for k, (ms, c) in kl.items() if k in ("encode_fwd", "encode_fwd_rows")) * 1e3 / 5, 2)
            if not fwd_only:
                row["bwd"]["alone_us"] = round(sum(ms for k, (ms, c) in kl.items() if k.startswith("encode_bwd") or k == "zero") * 1e3 / 5, 2)
                row["bwd"]["alone_variant"] = "binned" if cngp.bwd_plan_info(cfg_l, N)["binned"] else "sliced" if cngp.bwd_plan_info(cfg_l, N)["sliced"] else "direct"
            del ws_l
        step()                                                   # y, gF, gC of the whole configuration again, for the check below
        torch.cuda.synchronize()
    roof_fwd = sum(r["fwd"]["t_roof_us"] for r in levels)
    out["applicable_roofline"] = {
        "definition": "per level t_l = max(streaming share, random row fetches after reuse, gradient rows to memory) at rates "
                      "measured in this run; t_roof = sum over levels; frac = t_roof / measured time of the whole call",
        "measured_rates": {k: round(v, 1) for k, v in rates.items()},
        "fwd": {"t_roof_us": round(roof_fwd, 2), "measured_us": round(t_fwd, 2), "frac": round(roof_fwd / t_fwd, 4)},
        "per_level": levels}
    if not fwd_only:
        t_bwd = (per_kernel["encode_bwd"]["ms"] + per_kernel.get("zero", {"ms": 0.0})["ms"]) / args.steps * 1e3
        roof_bwd = sum(r["bwd"]["t_roof_us"] for r in levels)
        out["applicable_roofline"]["bwd"] = {"t_roof_us": round(roof_bwd, 2), "measured_us": round(t_bwd, 2),
                                             "frac": round(roof_bwd / t_bwd, 4)}
        out["applicable_roofline"]["frac"] = round((roof_fwd + roof_bwd) / (t_fwd + t_bwd), 4)
    else:
        out["applicable_roofline"]["frac"] = out["applicable_roofline"]["fwd"]["frac"]

    if with_opt:
        t_opt = per_kernel["adam_step_bake"]["ms"] / args.steps * 1e-3
        if with_dec:                                    # the decoder's Adam launch is counted in the same kernel kind
            alg["adam_step_bake"] += 30 * W_master.numel()
        out["optimizer_roofline"] = {"bound": "hbm", "kernel": "adam_step_bake",
                                     "achieved": round(alg["adam_step_bake"] / t_opt / 1e9, 1), "peak": HBM_PEAK_GBS,
                                     "unit": "GB/s", "frac": round(alg["adam_step_bake"] / t_opt / 1e9 / HBM_PEAK_GBS, 4),
                                     "algorithmic_bytes_per_launch": alg["adam_step_bake"],
                                     "avg_launch_us": round(t_opt * 1e6, 2)}

    if with_dec:
        flops = 2.0 * N * (64 * w.L * w.F + 64 * 64 + 64 * n_out)          # one pass through the three products
        out["decoder_roofline"] = {
            "bound": "mfma", "peak": 2500.0, "unit": "TFLOP/s",
            "fwd": {"avg_launch_us": round(per_kernel["mlp_fwd"]["ms"] * 1e3 / args.steps, 2),
                    "achieved": round(flops / (per_kernel["mlp_fwd"]["ms"] * 1e-3 / args.steps) / 1e12, 1)},
            "bwd": {"avg_launch_us": round(per_kernel["mlp_bwd"]["ms"] * 1e3 / args.steps, 2),
                    "achieved": round(3 * flops / (per_kernel["mlp_bwd"]["ms"] * 1e-3 / args.steps) / 1e12, 1)},
            "note": "useful flops (2 per multiply-add of the unpadded products; backward = recompute + data + weight "
                    "gradients = 3 passes) over the kernel's average duration"}
        for k in ("fwd", "bwd"):
            out["decoder_roofline"][k]["frac"] = round(out["decoder_roofline"][k]["achieved"] / 2500.0, 4)

    if not args.no_check or not args.no_cpu_baseline:
        import oracle
        if with_opt:
            # the tables moved: the self-check compares against the oracle on their final state, which is
            # the state the last forward and backward pass of the timed loop ran on
            D_f_h = D_f.cpu().numpy()
            Dhat_h = Dhat.cpu().numpy()
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity import check_close, check_exact, plain_rel_err
        # bounded sample of the same workload for the CPU leg: the first n_cpu points
        n_cpu = min(N, 1 << 22 if fwd_only else 1 << 18)
        xs = x_h[:n_cpu]
        t0 = time.perf_counter()
        D_c_ref = oracle.bake_probes(Dhat_h)
        y_ref, ymag = oracle.encode_fwd(w, xs, D_f_h, D_c_ref)
        if fused_dec:
            Wh = W_half.float().cpu().numpy().astype(np.float64)
            a, b = 64 * w.L * w.F, 64 * w.L * w.F + 64 * 64
            dec_ref, dec_mag, _ = oracle.mlp_fwd(y_ref, Wh[:a].reshape(64, -1), Wh[a:b].reshape(64, 64), Wh[b:].reshape(3, 64), want_mag=True)
        if not fwd_only:
            g_ref = oracle.encode_bwd(w, xs, D_f_h, Dhat_h, dy_h[:n_cpu], want_abs=not args.no_check, top_k=args.top_k)
        t_cpu = time.perf_counter() - t0
        if not args.no_cpu_baseline:
            # the same pass again until about ten seconds of CPU work are on the clock.  The pass above is the self-check's
            # (it also sums the magnitudes the tolerances are scaled by) and is not counted: the baseline is the plain oracle
            t_cpu, cpu_passes = 0.0, 0
            while t_cpu < 10.0 and cpu_passes < 200:
                t0 = time.perf_counter()
                oracle.encode_fwd(w, xs, D_f_h, oracle.bake_probes(Dhat_h))
                if not fwd_only:
                    oracle.encode_bwd(w, xs, D_f_h, Dhat_h, dy_h[:n_cpu], want_abs=False, top_k=args.top_k)
                t_cpu += time.perf_counter() - t0
                cpu_passes += 1
            out["cpu_baseline"] = {"value": round(n_cpu * cpu_passes / t_cpu, 1), "unit": "points/s",
                                   "cores": oracle.num_threads(), "kind": "oracle",
                                   "sample": f"first {n_cpu} of {N} points, {cpu_passes} passes of bake + fwd"
                                             + ("" if fwd_only else " + bwd") + f", {t_cpu:.1f} s in all"}
            # and on one thread, one pass over a shorter run of the same points
            n_one = min(n_cpu, 1 << 16)
            threads = oracle.num_threads()
            oracle.set_threads(1)
            t0 = time.perf_counter()
            oracle.encode_fwd(w, x_h[:n_one], D_f_h, oracle.bake_probes(Dhat_h))
            if not fwd_only:
                oracle.encode_bwd(w, x_h[:n_one], D_f_h, Dhat_h, dy_h[:n_one], want_abs=False, top_k=args.top_k)
            t_one = time.perf_counter() - t0
            oracle.set_threads(threads)
            out["cpu_baseline"]["one_thread"] = {"value": round(n_one / t_one, 1), "unit": "points/s",
                                                 "sample": f"first {n_one} points, one pass, {t_one:.1f} s"}
        if not args.no_check:
            # self-check of the timed configuration against the oracle (same launch configuration)
            if fmt == cngp.IDX_BITS:
                check_exact("D_c", D_c.cpu().numpy(), oracle.pack_index_bits(D_c_ref, w.N_p))
            else:
                unpack = D_c if fmt == cngp.IDX_U8 else torch.stack([D_c & 0xF, D_c >> 4], dim=-1).reshape(w.L, w.N_c)
                check_exact("D_c", unpack.cpu().numpy(), D_c_ref)
            if fused_dec:
                err = np.abs(out_dec[:n_cpu].cpu().numpy() - dec_ref) / np.maximum(np.maximum(np.abs(dec_ref), dec_mag), 1e-30)
                assert err.max() <= 2e-3, f"decoder(encode(x)): rel err {err.max():.3e}"
                e = {"decoder_out": float(err.max())}
            else:
                e = {"y": check_close("y", y[:n_cpu].cpu().numpy(), y_ref, ymag, fp16_out=(w.io_dtype == "f16"))}
            # with the decoder in the loop the upstream gradient is the decoder's output: no oracle input may come
            # from the kernels, so the gradient check is left to the parity tests in that mode
            if not fwd_only and n_cpu == N and not with_dec:
                e["grad_D_f"] = check_close("grad D_f", gF.cpu().numpy(), g_ref[0], g_ref[2], fp16_out=False)
                e["grad_Dhat_c"] = check_close("grad Dhat_c", gC.cpu().numpy(), g_ref[1], g_ref[3], fp16_out=False)
            if morton_perm is not None:
                t0 = time.perf_counter()
                perm_ref, _ = oracle.morton_order(x_h)
                extras["morton_order"]["sort_ms_host_oracle"] = round((time.perf_counter() - t0) * 1e3, 1)
                check_exact("morton perm", morton_perm, perm_ref)
            out["parity_max_rel_err"] = {k: float(f"{v:.3e}") for k, v in e.items()}
            # beside it, the plain max|gpu - ref| / max|ref| per tensor (no normalisation by the terms' magnitudes)
            pl = {}
            if not fused_dec:
                pl["y"] = plain_rel_err(y[:n_cpu].cpu().numpy(), y_ref)
            if "grad_D_f" in e:
                pl["grad_D_f"] = plain_rel_err(gF.cpu().numpy(), g_ref[0])
                pl["grad_Dhat_c"] = plain_rel_err(gC.cpu().numpy(), g_ref[1])
            out["parity_plain_max_rel_err"] = {k: float(f"{v:.3e}") for k, v in pl.items()}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
