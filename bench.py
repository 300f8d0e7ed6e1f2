#!/usr/bin/env python3
"""Benchmark of the DAT worker step on one MI355X.

A "step" is one pass of the whole hot path over one resident synthetic batch:
dat_attack (K-step PGD) -> dat_step (outer gradient) -> dat_quantize -> dat_dequantize (8 bit).
Default workload = the configuration the headline metric is quoted on: ResNet-50, 224x224,
batch 256, bf16, PGD-10 (eps 2/255, alpha 0.5/255, uniform random init).

Prints ONE JSON line.  `value` = examples/s through the whole step; `roofline` describes the
dominant kernel (the implicit-GEMM convolution) from hipEvent pairs recorded around every
launch during the timed steps; `cpu_baseline` times the CPU reference on a bounded sample."""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
WORKLOADS = {
    # name: arch, H, W, classes, B, K, eps, alpha, normalise, config id for seeds
    "resnet50_224_b256_pgd10": (3, 224, 224, 1000, 256, 10, 2 / 255, 0.5 / 255, True, 6),
    "resnet50_224_b256_fgsm": (3, 224, 224, 1000, 256, 1, 2 / 255, 2.5 / 255, True, 4),
    "resnet50_224_b256_pgd3": (3, 224, 224, 1000, 256, 3, 4 / 255, 1 / 255, True, 5),
    "resnet18_cifar_b512_pgd10": (1, 32, 32, 10, 512, 10, 8 / 255, 2 / 255, False, 2),
    "wrn34_10_b256_pgd10": (2, 32, 32, 10, 256, 10, 8 / 255, 2 / 255, False, 3),
    # the models and shapes of the paper's own runs (Sec. "Experiment setup", "Training setting"):
    # pre-activation ResNet-18 and WRN-28-10 on 32x32, ResNet-50 with 85 images per GPU and PGD-4
    # (alpha = 2.5 eps / K, the convention of the configurations above; the paper gives no PGD step size)
    "preact_resnet18_cifar_b512_pgd10": (4, 32, 32, 10, 512, 10, 8 / 255, 2 / 255, False, 7),
    "wrn28_10_b256_pgd10": (5, 32, 32, 10, 256, 10, 8 / 255, 2 / 255, False, 8),
    "resnet50_224_b85_pgd4": (3, 224, 224, 1000, 85, 4, 2 / 255, 1.25 / 255, True, 9),
}
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def cpu_baseline(arch, H, W, classes, K, eps, alpha, norm, bits):
    """CPU reference, as it stands, on a bounded sample of the same workload: the whole step (all K attack
    iterations, the outer gradient, quantize + dequantize) for B=8 images of the configured shape."""
    import oracle
    import synth_inputs as syn
    B = 8
    m = oracle.Model(arch, 1, H, W, classes, MEAN if norm else None, STD if norm else None)
    m.set_params(syn.he_normal_params(0, m.offsets, m.fan_in, m.kind))
    x, y = syn.images(0, B, H, W), syn.labels(0, B, classes)
    t0 = time.time()
    d = m.attack(x, y, eps, alpha, K, oracle.INIT_UNIFORM, seed=1)
    t1 = time.time()
    g, _ = m.step(oracle.make_xadv(x, d), y)
    t2 = time.time()
    S = oracle.levels(bits)
    codes, scales = oracle.quantize(g, m.offsets, S, 1)
    oracle.dequantize(codes, scales, m.offsets, S)
    t3 = time.time()
    return {"value": B / (t3 - t0), "unit": "examples/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "the whole step for B=%d images of the same shape (BN batch statistics over 8 instead of 256 images): "
                      "%d attack iterations %.1f s, outer gradient %.1f s, quantize + dequantize %.1f s" % (B, K, t1 - t0, t2 - t1, t3 - t2)}


def source_hash():
    """Hash of the kernel sources: ties stored profiler figures to the code they were measured on."""
    from paper_2206_06257_amd.profile_summary import source_hash as h
    return h()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50_224_b256_pgd10", choices=sorted(WORKLOADS))
    ap.add_argument("--bits", type=int, default=8)
    ap.add_argument("--phi", default="ce", choices=["ce", "trades"],
                    help="robustness regulariser of the worker objective: adversarial cross-entropy (the headline path) or the TRADES KL term")
    ap.add_argument("--lam", type=float, default=0.0, help="weight of the clean-loss term of the worker objective")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-launch-events", action="store_true", help="do not bracket launches with events")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy 5 times and exit (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--stream-rates", action="store_true",
                    help="time plain device fill / copy / add passes over a 411 MB tensor (the size of ResNet-50's widest stage-1 "
                         "activation at batch 256) and exit: what the box streams, as context for the HBM-bound kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "ms": ms,
                          "GBs_read_plus_write": 2 * src.numel() * 4 / (ms * 1e-3) / 1e9}))
        return
    if args.stream_rates:
        n = 256 * 56 * 56 * 256
        a = torch.ones(n, dtype=torch.bfloat16, device="cuda"); b = torch.ones_like(a); c = torch.empty_like(a)
        out = {"bytes_per_tensor": 2 * n, "note": "library elementwise passes (not this package's kernels); median of 20"}
        for name, f, moved in (("fill", lambda: c.zero_(), 1), ("copy", lambda: c.copy_(a), 2), ("add_2r1w", lambda: torch.add(a, b, out=c), 3)):
            for _ in range(3):
                f()
            ts = []
            for _ in range(20):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); f(); e1.record(); torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            ms = sorted(ts)[len(ts) // 2]
            out[name] = {"ms": ms, "TBs": moved * 2 * n / (ms * 1e-3) / 1e12}
        print(json.dumps(out))
        return
    import paper_2206_06257_amd as dat
    import synth_inputs as syn

    arch, H, W, classes, B, K, eps, alpha, norm, cfg = WORKLOADS[args.workload]
    blocked_stem = arch == 3 and H % 2 == 0 and W % 2 == 0     # 7x7/2 stem: the network input is stored as 2x2 pixel blocks
    torch.cuda.set_device(0)
    model = dat.Model(arch, dat.BF16, B, H, W, classes, MEAN if norm else None, STD if norm else None)
    model.set_params(syn.he_normal_params(cfg, model.offsets, model.fan_in, model.kind))
    x = torch.from_numpy(syn.images(cfg, B, H, W)).cuda()
    y = torch.from_numpy(syn.labels(cfg, B, classes)).cuda()
    delta = torch.empty_like(x)
    xadv = torch.empty_like(x)
    grads = torch.empty(model.d, dtype=torch.float32, device="cuda")
    q = torch.empty(dat.quantized_bytes(model.d, args.bits), dtype=torch.uint8, device="cuda")
    scales = torch.empty(model.num_tensors, dtype=torch.float32, device="cuda")
    deq = torch.empty(model.d, dtype=torch.float32, device="cuda")
    offs = (model.offsets_device(), model.num_tensors)
    seed_init, seed_q = syn.seed_for(cfg, "attack_init"), syn.seed_for(cfg, "quantizer")

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]

    general = args.phi != "ce" or args.lam != 0.0     # the general objective lambda*l + phi (two or three passes per step)

    def one_step(i, marks=None):
        if args.phi == "trades":
            model.attack_kl(x, eps, alpha, K, dat.INIT_UNIFORM, seed=seed_init + i, delta=delta)
        else:
            model.attack(x, y, eps, alpha, K, dat.INIT_UNIFORM, seed=seed_init + i, delta=delta)
        if marks:
            marks[0].record()
        dat.make_xadv(x, delta, out=xadv)      # clip(x + delta, 0, 1): the batch the outer step sees
        if general:
            model.step_reg(x, xadv, y, args.lam, dat.PHI_TRADES_KL if args.phi == "trades" else dat.PHI_CE, grads=grads)
        else:
            model.step(xadv, y, grads=grads)
        if marks:
            marks[1].record()
        if general:    # two passes: the sum's abs-max is not a by-product, the quantizer finds it itself
            dat.quantize(grads, offs, args.bits, seed_q + i, q=q, scales=scales)
        else:          # the gradient writers of dat_step left the per-tensor abs-max behind: only the encoder runs
            dat.quantize_scaled(grads, offs, args.bits, seed_q + i, model.grad_scales(), q=q)
        if marks:
            marks[2].record()
        dat.dequantize(q, scales if general else model.grad_scales(), offs, model.d, args.bits, out=deq)
        if marks:
            marks[3].record()

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    # ---- timed region: exactly `steps` steps, nothing else on the stream
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record()
        one_step(args.warmup + i, ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_step = [starts[i].elapsed_time(ev[i][3]) for i in range(args.steps)]   # event time of every timed step
    # ---- the same steps once more with a hipEvent pair around every launch (per-kernel-class times
    # for the roofline); kept out of the timed region because ~2700 event pairs per step cost ~7 %
    prof = None
    if not args.no_launch_events:
        model.profile_enable(True)
        tp0 = time.perf_counter()
        for i in range(args.steps):
            one_step(args.warmup + args.steps + i)
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - tp0) * 1e3 / args.steps
        prof = model.profile_read()
        model.profile_enable(False)

    t_attack = float(np.median([starts[i].elapsed_time(ev[i][0]) for i in range(args.steps)]))
    t_step = float(np.median([ev[i][0].elapsed_time(ev[i][1]) for i in range(args.steps)]))
    t_quant = float(np.median([ev[i][1].elapsed_time(ev[i][2]) for i in range(args.steps)]))
    t_deq = float(np.median([ev[i][2].elapsed_time(ev[i][3]) for i in range(args.steps)]))

    out = {
        "metric": "PGD-10 adv examples/s + train imgs/s (ResNet-50 224, 1 GPU); % MFMA/HBM peak",
        "value": B / (ms_per_step * 1e-3), "unit": "examples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": float(np.median(per_step)), "ms_per_step_min": float(np.min(per_step)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "image": [H, W, 3], "pgd_steps": K, "eps": eps, "alpha": alpha,
                   "quantizer_bits": args.bits, "params": model.d, "phi": args.phi, "lambda": args.lam},
        "adv_examples_per_s": B / (t_attack * 1e-3), "train_images_per_s": B / (t_step * 1e-3),
        "phase_ms": {"attack": t_attack, "step": t_step, "quantize": t_quant, "dequantize": t_deq},
    }
    d = model.d
    # the stand-alone quantizer (abs-max pass of its own: three launches), timed on the same gradient outside the steps
    qe = [torch.cuda.Event(enable_timing=True) for _ in range(41)]
    qe[0].record()
    for i in range(40):
        dat.quantize(grads, offs, args.bits, seed_q + i, q=q, scales=scales)
        qe[i + 1].record()
    torch.cuda.synchronize()
    t_quant_alone = float(np.median([qe[i].elapsed_time(qe[i + 1]) for i in range(40)]))
    out["quantizer"] = {
        "quantize_GBs": d * (8 + args.bits / 8) / (t_quant * 1e-3) / 1e9, "dequantize_GBs": d * (4 + args.bits / 8) / (t_deq * 1e-3) / 1e9,
        "frac_hbm_quantize": d * (8 + args.bits / 8) / (t_quant * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "frac_hbm_quantize_moved": d * ((4 if not general else 8) + args.bits / 8) / (t_quant * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "frac_hbm_dequantize": d * (4 + args.bits / 8) / (t_deq * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "standalone_quantize_ms": t_quant_alone,
        "frac_hbm_standalone_quantize": d * (8 + args.bits / 8) / (t_quant_alone * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "note": ("frac_hbm_quantize: the 8+b/8 algorithmic bytes per element of abs-max + encode over the event time of the step's quantizer "
                 "call; in the step the per-tensor abs-max is a by-product of the kernels that write the gradient (dat_model_grad_scales), so that "
                 "call is the encoder alone and moves 4+b/8 bytes per element (frac_hbm_quantize_moved).  standalone_*: dat_quantize with its own "
                 "abs-max pass (reset + abs-max + encode launches) on the same gradient.  Dequantize: 4+b/8 bytes per element.")}
    if prof:
        ms = prof["conv_fwd"][0] + prof["conv_bwd_data"][0]
        n = prof["conv_fwd"][1] + prof["conv_bwd_data"][1]
        flops = prof["conv_fwd"][2] + prof["conv_bwd_data"][2]
        ach = flops / (ms * 1e-3) / 1e12
        # HBM bytes per launch cannot be counted from inside this process: the figure comes from the two rocprofv3 --pmc
        # runs summarised under profiles/, and is reported only while the kernel sources are the ones it was measured on
        traffic, traffic_note = None, "no stored FETCH_SIZE / WRITE_SIZE figure for this workload"
        tpath = os.path.join(ROOT, "profiles", "traffic_igemm_" + args.workload + ".json")
        if os.path.exists(tpath):
            stored = json.load(open(tpath))
            if stored.get("source_hash") == source_hash():
                traffic = stored.get("hbm_bytes_per_launch")
                traffic_note = "from profiles/%s (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of this workload; kernel sources unchanged since)" % os.path.basename(tpath)
            else:
                traffic_note = "profiles/%s was measured on other kernel sources (hash %s, now %s): not reported" % (
                    os.path.basename(tpath), stored.get("source_hash"), source_hash())
        out["roofline"] = {"bound": "mfma", "kernel": "igemm_dma_kernel + igemm_ring_kernel + igemm_kernel (conv forward + backward-data launches; the few backward-data "
                                                      "launches that also form a batch-norm input gradient from three operand streams are "
                                                      "listed as kernel_classes.conv_bwd_data_bn)", "achieved": ach,
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic,
                           "traffic_source": traffic_note,
                           "launches": n, "avg_launch_ms": ms / max(n, 1), "flops_per_launch": flops / max(n, 1),
                           "achieved_forward": prof["conv_fwd"][2] / (prof["conv_fwd"][0] * 1e-3) / 1e12,
                           "achieved_backward_data": prof["conv_bwd_data"][2] / (prof["conv_bwd_data"][0] * 1e-3) / 1e12,
                           "note": "launch times include the fused epilogue work: the batch statistics of the next BN (forward), the "
                                   "residual gradient and the two BN backward sums of the producing BN, which re-read its input and "
                                   "ReLU mask (backward-data)"}
        if traffic:   # the same launches against the HBM roofline: measured bytes per launch / measured time per launch
            gbs = traffic / (ms / max(n, 1) * 1e-3) / 1e9
            out["roofline"]["traffic_GBs"] = gbs
            out["roofline"]["traffic_frac_hbm"] = gbs / PEAK_HBM_GBS
        out["kernel_classes"] = {k: {"ms_per_step": v[0] / args.steps, "launches_per_step": v[1] / args.steps,
                                     "work_per_step": v[2] / args.steps} for k, v in prof.items()}
        pg = prof["pgd"]
        if pg[0] > 0:
            out["pgd_update"] = {"GBs": pg[2] / (pg[0] * 1e-3) / 1e9, "frac_hbm": pg[2] / (pg[0] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                 "bytes_per_element": 18,
                                 "moved_GBs": pg[2] / 18.0 * ((52.0 if blocked_stem else 68.0) / 3.0) / (pg[0] * 1e-3) / 1e9,
                                 "note": "one launch per iteration; algorithmic bytes per element: x, delta, G read (12), delta written (4), "
                                         "bf16 network input written (2).  It reads the bf16 input gradient and writes the bf16 network input "
                                         + ("as 2x2 pixel blocks of 4 channels (8 bytes per pixel, 3 of 4 channels used): 52 bytes moved per pixel "
                                            "for the 54 algorithmic ones (G is read as bf16)" if blocked_stem else
                                            "as 16-byte vectors per pixel (3 of 8 channels used): 68 bytes moved per pixel for the 54 algorithmic ones")}
        total_flops = sum(prof[k][2] for k in ("conv_fwd", "conv_bwd_data", "conv_bwd_data_bn", "conv_wgrad")) / args.steps
        out["roofline"]["measured_over"] = "%d further steps of the same work with a hipEvent pair around every launch (%.1f ms/step with events)" % (args.steps, ms_per_step_events)
        out["step_conv_TFLOPs"] = total_flops / 1e12
        out["step_frac_mfma_peak"] = total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(arch, H, W, classes, K, eps, alpha, norm, args.bits)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
