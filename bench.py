#!/usr/bin/env python3
"""Benchmark of the GANQ per-layer solver on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3]

One "step" is one pass of the whole hot path over one synthetic layer whose
inputs already sit in HBM: H = X X^T, then one call that factors H (Cholesky),
builds the quantile codebooks and runs K_iters alternations of S-update and
T-update (Algorithm 1), and one evaluation of the objective.  The headline workload is the LLaMA-7B q_proj-shaped layer at 4 bits
(4096 x 4096, X 4096 x 262144 fp16, 10 alternations).

    python bench.py --decode [--config c5] [--nbits 4] [--steps K] [--warmup W]

times the deployment-side look-up-table product (batch-1 decoding from the stored form) instead;
see decode_main().

Prints ONE JSON line with the seconds per layer, a per-kernel-class breakdown
measured with HIP events on the library's stream inside the timed region, the
roofline figure of the dominant kernel, and the float64 CPU oracle timed on a
bounded sample of the same workload (baseline only).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_F16_TFLOPS = 2500.0
PEAK_F32_MFMA_TFLOPS = 157.3
# plain fp32 vector additions: 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2.4 GHz = 78.6e12 adds/s,
# i.e. half of the 157.3 TFLOP/s vector FMA figure (an add is one flop, an FMA two)
PEAK_F32_ADD_TOPS = 78.6
PEAK_I8_TOPS = 5000.0


# Kernels behind each timed class: (main kernel, [other kernels launched inside the class's bracket]).
# HBM traffic per class launch = sum over these kernels of (MiB per launch x launches in one step) of the
# table in profiles/<file> (FETCH_SIZE and WRITE_SIZE of rocprofv3 --pmc, already scaled there by the
# reading of a plain copy), divided by the main kernel's launches.
CLASS_KERNELS = {
    "hessian": ("hessian_f16_kernel", ["reduce_mirror_kernel"]),
    "cholesky": ("copy_lower_kernel", ["chol_panel_kernel", "gemm_f32_kernel", "syrk_f32_kernel", "fill_i32_kernel"]),
    "init": ("init_codebooks_kernel", ["convert_f16_f32_kernel"]),
    "update_s": ("update_S_kernel", ["rdiag_kernel"]),
    "update_s32": ("update_S32_kernel", ["rdiag_kernel"]),
    "t_prep": ("t_split_kernel", ["t_diag_kernel", "t_rowscale_kernel", "t_symscale_kernel"]),
    "t_pad": ("pad_q_kernel", ["t_flips_kernel", "t_chunks_kernel"]),
    "t_accum": ("t_accum_kernel", []),
    "t_delta": ("t_delta_kernel", []),
    "t_solve": ("t_solve_kernel", []),
}
TRAFFIC_FILES = {c: "bench_%s_hbm_traffic.txt" % c for c in ("c2", "c3", "c4a", "c4b", "c5", "c5_3")}


def load_traffic(config_name):
    """{class: HBM bytes per class launch} from the committed rocprofv3 summary of this workload, or {}."""
    fn = TRAFFIC_FILES.get(config_name)
    path = os.path.join(ROOT, "profiles", fn) if fn else None
    if not path or not os.path.exists(path):
        return {}
    rows = {}
    for ln in open(path):
        f = ln.split()
        if len(f) == 5 and not ln.startswith("#") and f[1].isdigit():
            rows[f[0].split("<")[0]] = (int(f[1]), float(f[4]) * 2 ** 20)        # launches, bytes per launch
    out = {}
    for cls, (main, others) in CLASS_KERNELS.items():
        if main not in rows:
            continue
        total = sum(rows[k][0] * rows[k][1] for k in [main] + others if k in rows)
        out[cls] = total / rows[main][0]
    if "update_s32" in out:          # the 32-row kernel is the S-update of the shapes that select it
        out["update_s"] = out.pop("update_s32")
    # the two split-fp16 products (G = W H inside the solver, F = E H in the loss) share their kernels
    if "gemm_split_kernel" in rows:
        g = rows["gemm_split_kernel"][1]
        aux = 2 * rows.get("absmax_kernel", (0, 0.0))[1] + 2 * rows.get("split_kernel", (0, 0.0))[1]
        out["gemm_wh"] = g + aux
        out["loss"] = g + aux + rows.get("residual_kernel", (0, 0.0))[1] + rows.get("rowdot_kernel", (0, 0.0))[1]
    return out


def kernel_work(cls, m, n, p, nbits, iters):
    """Algorithmic work of ONE launch of a kernel class: (bound, work, unit, peak)."""
    if cls == "hessian":
        return "mfma", float(n) * n * p, "TFLOP/s", PEAK_F16_TFLOPS          # symmetric half of 2 n^2 p
    if cls == "cholesky":
        return "mfma", float(n) ** 3 / 3.0, "TFLOP/s", PEAK_F32_MFMA_TFLOPS
    if cls == "gemm_wh":
        # runs as three fp16 piece products; one product's flops are counted
        return "mfma", 2.0 * m * n * n, "TFLOP/s", PEAK_F16_TFLOPS
    if cls == "update_s":
        return "mfma", float(m) * n * n, "TFLOP/s", PEAK_F32_MFMA_TFLOPS      # triangular: m n^2 / 2 MACs
    if cls == "t_accum":
        return "alu", 0.5 * m * n * n, "TFLOP/s", PEAK_F32_ADD_TOPS           # m n^2 / 2 additions
    if cls == "t_delta":
        # gather of the rows of H that belong to the changed columns: two digit bytes per entry; the
        # number of changed columns comes from the library's sweep log (filled in by main())
        return "hbm", 0.0, "GB/s", PEAK_HBM_GBS
    if cls == "loss":
        return "mfma", 2.0 * m * n * n, "TFLOP/s", PEAK_F16_TFLOPS
    if cls == "t_prep":
        return "hbm", 2 * 4.0 * n * n / 2 + 2.0 * n * n / 2, "GB/s", PEAK_HBM_GBS  # read tril(H) twice, write 2 digits
    if cls == "t_pad":
        return "hbm", 2.0 * m * n, "GB/s", PEAK_HBM_GBS
    if cls == "t_solve":
        return "hbm", 5.0 * m * n, "GB/s", PEAK_HBM_GBS                        # G (4 B) + Q (1 B) per element
    if cls == "init":
        return "hbm", 6.0 * m * n, "GB/s", PEAK_HBM_GBS
    return "hbm", 0.0, "GB/s", PEAK_HBM_GBS


def cpu_baseline(cfg, X_dev, W_dev, rows=256, tokens=16384):
    """The float64 oracle timed on the host cores on a bounded sample: H from `tokens`
    tokens, a full Cholesky, and the K alternations on `rows` rows of W; seconds are then
    scaled to the whole layer (rows are independent; H is a sum over tokens)."""
    import numpy as np
    from oracle import ganq_ref as ref
    tokens, rows = min(tokens, cfg.p), min(rows, cfg.m)
    try:
        from threadpoolctl import threadpool_info
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    Xs = X_dev[:, :tokens].cpu().numpy()
    Ws = W_dev[:rows].float().cpu().numpy().astype(np.float64)
    t0 = time.perf_counter()
    H = ref.build_hessian(Xs)
    t_h = time.perf_counter() - t0
    t0 = time.perf_counter()
    L, _ = ref.cholesky(H)
    t_c = time.perf_counter() - t0
    t0 = time.perf_counter()
    T0 = ref.init_codebooks(Ws, cfg.nbits)
    T, Q = ref.quantize_layer(Ws, H, T0, cfg.nbits, cfg.iters, L=L)
    loss = ref.layer_loss(Ws, H, T, Q)[0]
    t_s = time.perf_counter() - t0
    full = t_h * (cfg.p / tokens) + t_c + t_s * (cfg.m / rows)
    return {
        "value": full, "unit": "s/layer", "cores": int(threads), "kind": "oracle",
        "sample": "measured %.1f s: H from %d of %d tokens (%.2f s), full Cholesky (%.2f s), "
                  "%d alternations + loss on %d of %d rows (%.2f s); scaled linearly to the layer"
                  % (t_h + t_c + t_s, tokens, cfg.p, t_h, t_c, cfg.iters, rows, cfg.m, t_s),
    }


# HBM bytes per look-up-table product (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, KiB per dispatch, from
# profiles/decode_c5_kernel_stats.txt); other shapes report null.
TRAFFIC_DECODE_BYTES = {("c5", 4): (57757.9 * 2.000 + 32.0) * 1024}


def decode_main(args):
    """The look-up-table product y = W~ x from the stored form (N-bit codes + fp16 tables), timed over
    enough distinct layers of the given shape that the codes stream from HBM rather than from a cache
    (at least 768 MB in total).  One step = one product per layer copy; the line reports microseconds
    per product and the stored bytes per product over the kernel's average launch time against the HBM
    peak.  cpu_baseline: the float64 definition on a sample of rows."""
    import numpy as np
    import torch
    from paper_2501_12956_amd import binding, synth

    cfg = synth.CONFIGS[args.config]
    m, n, nbits = cfg.m, cfg.n, args.nbits
    C = 1 << nbits
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ctx = binding.Context(0)
    stored = m * n * nbits / 8 + m * C * 2
    copies = max(2, int(-(-768e6 // stored)))
    g = torch.Generator(device=dev).manual_seed(1)
    layers = []
    for _ in range(copies):
        Q = torch.randint(0, C, (m, n), dtype=torch.uint8, device=dev, generator=g)
        T = (torch.randn(m, C, device=dev, generator=g) * 0.02).sort(dim=1).values.contiguous()
        layers.append(ctx.pack_layer(Q, T, nbits))
    x = torch.randn(n, device=dev, generator=g).half()
    y = torch.empty(m, dtype=torch.float32, device=dev)

    def step():
        for packed, lut in layers:
            ctx.lut_gemv(packed, lut, nbits, n, x, y)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The launches are back to back on the context's stream (torch's current one), so one HIP event
    # pair around the region gives the kernel's average duration; a pair around each 10-40 us launch
    # would add to it.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    us = 1e6 * elapsed / (args.steps * copies)
    avg_ms = ev0.elapsed_time(ev1) / (args.steps * copies)
    algo_bytes = stored + 2 * n + 4 * m
    achieved = algo_bytes / (avg_ms * 1e-3) / 1e9

    # the same product on fp16 weights by the vendor library, for context (Table 6 compares with FP16)
    Wd = [torch.randn(m, n, device=dev, dtype=torch.float16) for _ in range(max(2, int(768e6 // (2 * m * n))))]
    for Wk in Wd:
        torch.mv(Wk, x)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        for Wk in Wd:
            torch.mv(Wk, x)
    torch.cuda.synchronize()
    dense_us = 1e6 * (time.perf_counter() - t1) / (args.steps * len(Wd))

    out = {
        "metric": "microseconds per look-up-table product (batch 1) of one stored layer",
        "value": us, "unit": "us/product", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x f16 -> f32", "data": "synthetic",
        "config": {"workload": "%s-shaped layer %dx%d stored at %d bits + fp16 tables, x fp16, %d distinct "
                               "layers per step" % (cfg.name, m, n, nbits, copies)},
        "roofline": {"kernel": "lut_gemv", "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "traffic": TRAFFIC_DECODE_BYTES.get((cfg.name, nbits)),
                     "avg_launch_ms": avg_ms},
        "fp16_dense_mv_us": dense_us,
    }
    if not args.no_cpu_baseline:
        from oracle import ganq_ref as ref
        rows = 256
        packed, lut = layers[0]
        Qs = torch.from_numpy(ref.unpack_codes(packed[:rows].cpu().numpy()[:, :ref.packed_row_bytes(n, nbits)],
                                               n, nbits))
        t2 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t2 < 10.0:
            ref.lut_matvec(lut[:rows].cpu().numpy(), Qs.numpy(), x.cpu().numpy())
            reps += 1
        dt = (time.perf_counter() - t2) / reps
        out["cpu_baseline"] = {"value": 1e6 * dt * m / rows, "unit": "us/product", "cores": 1, "kind": "oracle",
                               "sample": "%d of %d rows, scaled by rows" % (rows, m)}
    print(json.dumps(out))


def stacked_main(args):
    """Layers that see the same activations (q/k/v, gate/up) share H and its factor, and rows are
    independent (Section 3.1): their weights stacked row-wise go through ONE ganq_quantize_layer call.
    Times three 4096 x 4096 layers (config c3's recipe, three seeds) solved by three calls against one
    stacked call, H given and factored inside each call as the benchmark step does."""
    import torch
    from paper_2501_12956_amd import binding, synth

    cfg = synth.CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    Ws = [synth.make_weight(cfg, sd, dev) for sd in (0, 1, 2)]
    X = synth.make_activations(cfg, 0, dev)
    ctx = binding.Context(0)
    ctx.reserve(3 * cfg.m, cfg.n, cfg.p, cfg.nbits)
    H = ctx.build_hessian(X)
    del X
    Wall = torch.cat(Ws, 0).contiguous()

    def three():
        return [ctx.quantize_layer(W, H, cfg.nbits, cfg.iters) for W in Ws]

    def one():
        return ctx.quantize_layer(Wall, H, cfg.nbits, cfg.iters)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / args.steps, out

    t3, outs = timed(three)
    t1, (Tall, Qall) = timed(one)
    # rows are independent: the stacked call reproduces the separate calls up to near ties
    same = [float((Qall[k * cfg.m:(k + 1) * cfg.m] == outs[k][1]).all(dim=1).float().mean()) for k in range(3)]
    print(json.dumps({
        "metric": "ms for three %dx%d layers sharing H (%d-bit, %d iters): three calls vs one stacked call"
                  % (cfg.m, cfg.n, cfg.nbits, cfg.iters),
        "three_calls_ms": t3, "stacked_call_ms": t1, "ratio": t3 / t1, "steps": args.steps, "warmup": args.warmup,
        "identical_rows_fraction": same, "n_gpus": 1, "data": "synthetic",
        "config": {"workload": "%s recipe, seeds 0-2 for W, one X" % cfg.name}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="c3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peak-probe", action="store_true",
                    help="skip the on-box peak measurement (fractions of measured peaks are then null)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed region: under "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE its reading gives the scale of the counter")
    ap.add_argument("--decode", action="store_true",
                    help="time the deployment-side look-up-table product instead of the solver")
    ap.add_argument("--nbits", type=int, default=4, help="--decode only: bits per stored code")
    ap.add_argument("--stacked", action="store_true",
                    help="time three layers that share their activations: three calls against one stacked call")
    ap.add_argument("--token-major", action="store_true",
                    help="hand the activations over as tokens x features (H = Xt^T Xt, read in place) instead "
                         "of features x tokens; everything else as in the default step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the solver has no multi-GPU path); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.decode:
        return decode_main(args)
    if args.stacked:
        return stacked_main(args)

    import torch
    from paper_2501_12956_amd import binding, synth

    cfg = synth.CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    W = synth.make_weight(cfg, 0, dev)
    X = synth.make_activations(cfg, 0, dev)
    Wf = W.float()                      # the objective is evaluated on the fp32 upcast
    m, n, p = cfg.m, cfg.n, cfg.p
    ctx = binding.Context(0)
    ctx.reserve(m, n, p, cfg.nbits)
    H = torch.empty(n, n, dtype=torch.float32, device=dev)
    Q = torch.empty(m, n, dtype=torch.uint8, device=dev)
    state = {}
    Xt = X.t().contiguous() if args.token_major else None

    def step():
        if Xt is not None:
            ctx.build_hessian_tokens(Xt, H=H)
        else:
            ctx.build_hessian(X, H=H)
        # Cholesky, T^0 and the alternations in one call: the library factors H itself and runs what
        # does not need L (W to fp32, T^0, G = W H, the split of H) beside the factorisation
        T, _ = ctx.quantize_layer(W, H, cfg.nbits, cfg.iters, Q=Q)
        state["loss"] = ctx.layer_loss(Wf, H, T, Q, cfg.nbits)
        state["T"] = T

    if args.calibrate_copy:
        calib = torch.zeros(2, 1 << 28, dtype=torch.float32, device=dev)    # 2 x 1 GiB
        torch.cuda.synchronize()
        calib[1].copy_(calib[0])                                            # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del calib
    peaks = {}
    if not args.no_peak_probe:
        peaks = ctx.measure_peaks()         # bare MFMA loops and a device copy, about 0.1 s
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step = 1e3 * elapsed / args.steps

    traffic = load_traffic(cfg.name)
    # peak the same silicon sustains on a bare loop, by the unit and arithmetic of each class
    def measured_peak(cls, unit, bound):
        if not peaks:
            return None
        if unit == "GB/s":
            return peaks["copy_gbs"]
        if cls in ("hessian", "gemm_wh", "loss"):
            return peaks["f16_mfma_tflops"]
        if cls in ("t_accum", "t_delta"):
            # additions that run as int8 one-hot products: 2 C digits operations issued per addition
            return peaks["i8_mfma_tops"] / (2.0 * (1 << cfg.nbits) * 2) if cls == "t_accum" else peaks["copy_gbs"]
        return peaks["f32_mfma_tflops"]

    log = ctx.sweep_log()
    upd = [t for (u, _, t) in log if u]
    npad = (n + 127) // 128 * 128
    kernels = {}
    for cls, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        bound, work, unit, peak = kernel_work(cls, m, n, p, cfg.nbits, cfg.iters)
        if cls == "t_delta" and upd:
            work = 2.0 * npad * sum(upd) / len(upd)      # bytes gathered per updating sweep
        avg_ms = ms / cnt
        rate = work / (avg_ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9) if avg_ms > 0 else 0.0
        mp = measured_peak(cls, unit, bound)
        kernels[cls] = {"ms_per_step": ms / args.steps, "launches_per_step": cnt / args.steps,
                        "avg_ms": avg_ms, "bound": bound, "achieved": rate, "peak": peak, "unit": unit,
                        "frac": rate / peak,
                        "measured_peak": mp, "frac_of_measured_peak": (rate / mp) if mp else None,
                        "traffic": traffic.get(cls)}
        if cls == "t_delta":
            # the gathered rows of the 32 MB digit matrix come from L2 and the memory-side cache, not from
            # HBM: the rate is reported, a fraction of the HBM peak would mean nothing
            kernels[cls].update({"bound": "l2", "peak": None, "frac": None, "measured_peak": None,
                                 "frac_of_measured_peak": None})
        if cls == "t_accum":
            # what the matrix cores execute for those additions: one-hot int8 products, C columns per
            # row and two base-256 digits per entry (three or four on strongly correlated H)
            issued = 2.0 * (1 << cfg.nbits) * 2 * work
            kernels[cls]["issued"] = {"int8_ops_per_launch": issued,
                                      "rate_tops": issued / (avg_ms * 1e-3) / 1e12, "peak_tops": PEAK_I8_TOPS,
                                      "frac": issued / (avg_ms * 1e-3) / 1e12 / PEAK_I8_TOPS,
                                      "note": "two-digit tiles assumed; bound \"alu\" above counts the additions"}
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    kd = kernels[dominant]
    roofline = {"kernel": dominant, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"], "traffic": kd["traffic"],
                "avg_launch_ms": kd["avg_ms"], "measured_peak": kd["measured_peak"],
                "frac_of_measured_peak": kd["frac_of_measured_peak"]}

    if cfg.m == 4096 and cfg.n == 4096 and cfg.nbits == 4 and cfg.iters == 10:
        metric = "sec per 4096x4096 layer (4-bit, 10 iters) on 1 GPU; % MFMA/HBM roofline"
    else:
        metric = ("sec per %dx%d layer (%d-bit, %d iters) on 1 GPU; %% MFMA/HBM roofline"
                  % (m, n, cfg.nbits, cfg.iters))
    out = {
        "metric": metric,
        "value": ms_per_step / 1e3, "unit": "s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None,
        # storage and the S-update are fp32; what else runs is listed, not hidden behind "f32"
        "dtype": "f32 (H build: f16 x f16 -> f32; T-update sums: exact int32 over base-256 int8 digits of H; "
                 "G = W H and the loss product: two-piece f16 splits, f32 accumulate; per-row solve: f64)",
        "data": "synthetic",
        "config": {"workload": "%s: W %dx%d %s, X %dx%d %s%s, N=%d bits, %d alternations; step = H build + "
                               "Cholesky + codebook init + alternations + loss"
                               % (cfg.name, m, n, str(cfg.w_dtype).replace("torch.", ""), n, p,
                                  str(cfg.x_dtype).replace("torch.", ""),
                                  " (handed over as tokens x features)" if args.token_major else "",
                                  cfg.nbits, cfg.iters)},
        "final_loss": state["loss"],
        "roofline": roofline,
        "kernels": kernels,
        "measured_peaks": peaks or None,
        # per sweep of the last step: did it update S_i H S_i^T from the changed columns (1) or sum it
        # again (0); the most changed indices in a row; their total
        "sweeps": log,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, X, W)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
