#!/usr/bin/env python3
"""Benchmark of the pre-attention expert-prediction path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input shaped
like a paper workload: predict for all L layers (one launch set), then
group_by_expert and score for all layers.  Inputs are resident in HBM before
the timed region; weights rotate over several independently generated banks so
that a step never finds its weights in the 256 MB Infinity Cache.  With
--pipeline consecutive steps overlap on two streams (grouping and scoring of
one step beside the predict of the next); every step still does all its work.

Prints ONE JSON line: throughput in predicted tokens*layers per second, the
roofline of the dominant kernel (measured live with HIP events around the
predict launches of the timed steps), and the CPU oracle timed on a bounded
sample of the same workload (a baseline, not a target).

The default run reports the workload's prefill size as the headline and, under
"also", its decode sizes (each with its own HBM roofline) and the prefill size
again with the over-provisioned prediction width the paper evaluates
(section 5.2), all on the same weight banks.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--T tokens] [--k-pred K'] [--no-cpu]
                    [--only] [--counted] [--pipeline] [--copy-probe-mib N]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published
MALL_BYTES = 256 << 20

# Bytes that crossed the L2 <-> fabric boundary per predict launch set, from two
# rocprofv3 --pmc passes over this script (FETCH_SIZE, then WRITE_SIZE, KiB per
# dispatch, summed over the predict kernels), each scaled by what the counter
# reads for the 1 GiB device copy of --copy-probe-mib in the same run (FETCH_SIZE
# reads half the copied bytes: factor 2.0; WRITE_SIZE reads them exactly: 1.0).
# Keyed by a hash of the kernel sources (comments and blank space excluded):
# once a kernel's code changes, the figure no longer describes it and the
# report says null.
TRAFFIC_BYTES = {
    ("prefill", "be865277bf0be11a"): {("deepseek_v2_lite", 4096): 3.891e+09,
                                      ("qwen3_30b_a3b", 8192): 1.457e+10,
                                      ("phi_mini_moe", 8192): 4.91e+09,
                                      ("stress", 32768): 2.41e+11},
    ("decode", "d527a095cb363a51"): {("deepseek_v2_lite", 1): 2.259e+08,
                                     ("deepseek_v2_lite", 64): 2.588e+08},
}


def _code_hash(path):
    """Hash of the kernel's source with // comments and blank space removed, so that
    rewording a comment does not retire a measurement but any change to code does."""
    import hashlib
    import re
    m = hashlib.sha256()
    for f in ("predict_%s.hip" % path, "paep_device.h"):
        try:
            with open(os.path.join(ROOT, "paper_2511_10676_amd", "csrc", f), "r") as fh:
                text = fh.read()
        except OSError:
            return None
        text = re.sub(r"//[^\n]*", "", text)
        m.update("".join(text.split()).encode())
    return m.hexdigest()[:16]


def measured_traffic(path, workload, T):
    return TRAFFIC_BYTES.get((path, _code_hash(path)), {}).get((workload, T))


def algorithmic_work(w, T, k=None):
    """Per layer call: flops and bytes the method itself must do/move
    (two weight matrices, x in, idx + probs out; h and the scores stay on chip)."""
    flops = 2.0 * w.r * (w.d + w.E) * T
    wbytes = 2.0 * w.r * (w.d + w.E)
    nbytes = wbytes + 2.0 * T * w.d + 8.0 * T * (k or w.k) + (2.0 * w.E if w.zipf_bias else 0.0)
    return flops, nbytes


class Banks:
    """The workload's predictor weights on the device: several independently generated banks (a step uses
    one and the next step the next, so that no step finds its weights in the Infinity Cache), the router
    the labels are drawn from (bank 0's), and the biases.  Shared by every token count that is timed."""

    def __init__(self, w, n_banks=None):
        import numpy as np
        import torch
        from paper_2511_10676_amd import datagen
        L = w.L
        bank_bytes = 2 * L * w.r * (w.d + w.E)
        if n_banks is None:
            n_banks = max(2, -(-2 * MALL_BYTES // bank_bytes) + 1)
        self.n_banks = n_banks
        self.to_dev = to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).cuda()
        self.W1, self.W2, self.routers, b2s = [], [], [], []
        W1_0, W2_0 = [], []
        for l in range(L):
            W1_0.append(datagen.make_w1(w, l)); W2_0.append(datagen.make_w2(w, l))
            self.routers.append(datagen.make_router(w, l, W1_0[-1], W2_0[-1]))
            b2 = datagen.make_b2(w, l)
            if b2 is not None:
                b2s.append(b2)
        self.b2_host = b2s
        self.b2 = to_dev(np.stack(b2s)) if b2s else None
        self.W1.append(to_dev(np.stack(W1_0))); self.W2.append(to_dev(np.stack(W2_0)))
        del W1_0, W2_0
        for bank in range(1, n_banks):
            self.W1.append(to_dev(np.stack([datagen.make_w1(w, l, bank) for l in range(L)])))
            self.W2.append(to_dev(np.stack([datagen.make_w2(w, l, bank) for l in range(L)])))


class Runner:
    """Device buffers for one workload at one token count, and the step."""

    def __init__(self, w, T, banks, k_pred=None, pipelined=False, counted=False):
        import numpy as np
        import torch
        from paper_2511_10676_amd import binding as B
        from paper_2511_10676_amd import datagen
        self.B, self.torch, self.w, self.T = B, torch, w, T
        self.k_pred = kp = k_pred or w.k            # experts predicted per token (> w.k: over-provisioning, section 4.1)
        L = w.L
        self.n_banks = n_banks = banks.n_banks
        self.W1, self.W2, self.b2 = banks.W1, banks.W2, banks.b2
        xs, refs = [], []
        for l in range(L):
            x = datagen.make_x(w, l, T)
            refs.append(datagen.router_labels(banks.routers[l], x, banks.b2_host[l] if banks.b2_host else None, w.k))
            xs.append(x)
        self.x = banks.to_dev(np.stack(xs))
        self.ref = torch.from_numpy(np.stack(refs)).cuda()
        del xs
        dev = self.x.device
        desc = B.make_desc(T, w.d, w.r, w.E, kp, L, B.BF16)
        self.path = B.resolve_path(desc)
        self.plan = B.predict_plan(desc)
        ws = B.predict_workspace_bytes(desc)
        self.ws = torch.empty(max(ws, 16), dtype=torch.uint8, device=dev)
        # Pipelined mode: two sets of result buffers and two streams, predict of step i+1 (stream A)
        # beside group_by_expert + score of step i (stream B).  Every step still does all of its work; a
        # buffer set is reused only after the step that read it has finished (events).
        self.pipelined = pipelined
        nset = 2 if pipelined else 1
        self.outs = [B.Prediction(torch.empty((L, T, kp), dtype=torch.int32, device=dev),
                                  torch.empty((L, T, kp), dtype=torch.float32, device=dev), None, self.path)
                     for _ in range(nset)]
        self.grps = [B.alloc_grouping(L, T, kp, w.E, dev) for _ in range(nset)]
        self.gwss = [torch.empty(max(B.group_workspace_bytes(L, T, kp, w.E), 16), dtype=torch.uint8, device=dev)
                     for _ in range(nset)]
        self.cnts = [torch.empty((L, 4), dtype=torch.int64, device=dev) for _ in range(nset)]
        self.sA = torch.cuda.Stream() if pipelined else torch.cuda.current_stream()
        self.sB = torch.cuda.Stream() if pipelined else self.sA
        self.ready = [torch.cuda.Event() for _ in range(nset)]
        self.done = [torch.cuda.Event() for _ in range(nset)]
        # every call of a step is checked and marshalled once; the timed loop only enqueues
        # --counted: the predict call also accumulates the activation counts of its selections (paep_predict_counted)
        self.counts = torch.zeros((L, w.E), dtype=torch.int32, device=dev) if counted else None
        self.p_predict = [[B.prepare_predict(self.x, self.W1[b], self.W2[b], kp, b2=self.b2, out=self.outs[k],
                                             workspace=self.ws, counts=self.counts) for k in range(nset)]
                          for b in range(n_banks)]
        self.p_group = [B.prepare_group_by_expert(self.outs[k].idx, w.E, out=self.grps[k], workspace=self.gwss[k])
                        for k in range(nset)]
        self.p_score = [B.prepare_score(self.outs[k].idx, self.ref, w.E, out=self.cnts[k]) for k in range(nset)]
        self.i = 0
        self.last = 0

    def step(self, ev=None):
        B, w, torch = self.B, self.w, self.torch
        bank = self.i % self.n_banks
        k = self.i % len(self.outs)
        self.i += 1
        self.last = k
        with torch.cuda.stream(self.sA):
            if self.pipelined:
                self.sA.wait_event(self.done[k])          # the step that last used this buffer set is through
            if ev is not None:
                ev[0].record()
            self.p_predict[bank][k]()
            if ev is not None:
                ev[1].record()
            self.ready[k].record()
        with torch.cuda.stream(self.sB):
            if self.pipelined:
                self.sB.wait_event(self.ready[k])
            self.p_group[k]()
            self.p_score[k]()
            self.done[k].record()
            if ev is not None:
                ev[2].record()

    def timed(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        evs = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            self.step(evs[s])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        predict = sorted(a.elapsed_time(b) for a, b, _ in evs)
        whole = sorted(a.elapsed_time(c) for a, _, c in evs)
        mean = lambda v: sum(v) / len(v)
        std = lambda v: (sum((t - mean(v)) ** 2 for t in v) / len(v)) ** 0.5
        self.stats = {"predict_ms_median": round(predict[len(predict) // 2], 4), "predict_ms_std": round(std(predict), 4),
                      "step_gpu_ms_median": round(whole[len(whole) // 2], 4), "step_gpu_ms_std": round(std(whole), 4)}
        return wall / steps * 1e3, mean(predict)

    def report(self, steps, warmup):
        w, T = self.w, self.T
        ms_step, predict_ms = self.timed(steps, warmup)
        flops, nbytes = algorithmic_work(w, T, self.k_pred)
        if self.path == "prefill":
            ach = flops * w.L / (predict_ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": measured_traffic("prefill", w.name, T),
                    "kernel": "prefill_kernel", "kernel_ms": round(predict_ms, 4)}
        else:
            ach = nbytes * w.L / (predict_ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": measured_traffic("decode", w.name, T),
                    "kernel": ("decode_rows_kernel" if w.r % 128 == 0 else "decode_partial_kernel") + "+decode_finalize_kernel",
                    "kernel_ms": round(predict_ms, 4)}
        self.i = 0                       # one untimed step on bank 0, whose weights the labels were drawn for
        self.step()
        self.torch.cuda.synchronize()
        prof = self.B.activation_profile(self.grps[self.last].counts)   # untimed: popularity skew of what was just predicted
        self.torch.cuda.synchronize()
        self.entropy0 = round(float(prof.entropy[0]), 4)
        return {"T": T, "k_pred": self.k_pred, "path": self.path,
                "launch": (f"{self.plan.tile} tiles, {self.plan.groups} workgroup(s) per token tile"
                           if self.path == "prefill" else
                           f"r in slices of {128 if w.r % 128 == 0 else 64} per workgroup + finalize"),
                "ms_per_step": round(ms_step, 4),
                "value": round(T * w.L / (ms_step * 1e-3), 1), "roofline": roof,
                "score_layer0": self.cnts[self.last][0].cpu().numpy().tolist(), "weight_banks": self.n_banks,
                "timing": self.stats}


def device_ceilings(torch, B):
    """What this device sustains for the two bounding resources, measured with the library's probes:
    a coalesced streaming read of 1 GiB (fresh every launch: larger than the Infinity Cache) and of a
    225 MB buffer (the size of one DeepSeek-shaped bank), and a register-only bf16 MFMA loop on every CU."""
    out = {}
    sink = torch.zeros(1 << 18, dtype=torch.uint8, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for name, nbytes, reps in (("read_1GiB_GBps", 1 << 30, 5), ("read_225MB_GBps", 225 << 20, 8)):
        bufs = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(i + 1) for i in range(3)]
        for b in bufs:
            B.probe_read(b, sink)
        torch.cuda.synchronize()
        times = []
        for i in range(reps * len(bufs)):
            a, z = ev(), ev()
            a.record(); B.probe_read(bufs[i % len(bufs)], sink); z.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(z))
        times.sort()
        out[name] = round(nbytes / (times[len(times) // 2] * 1e-3) / 1e9, 1)
        del bufs
        torch.cuda.empty_cache()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    B.probe_mfma(cus, 2000, sink)
    torch.cuda.synchronize()
    a, z = ev(), ev()
    a.record(); flops = B.probe_mfma(cus, 40000, sink); z.record()
    torch.cuda.synchronize()
    out["mfma_bf16_loop_TFLOPs"] = round(flops / (a.elapsed_time(z) * 1e-3) / 1e12, 1)
    out["note"] = "measured on this device by paep_probe_read / paep_probe_mfma (registers only, all CUs busy)"
    return out


def _oracle_pass(w, inputs):
    import oracle
    t0 = time.perf_counter()
    for lay in inputs:
        idx, probs, _ = oracle.predict(lay.x, lay.W1, lay.W2, w.k, b2=lay.b2, want_logits=False)
        oracle.group_by_expert(idx, w.E)
        oracle.score(idx, lay.ref, w.E)
    return time.perf_counter() - t0


def cpu_baseline(w, T, budget_s=16.0, budget_1t_s=5.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: with every host thread
    OpenMP gives it, and on one thread (a smaller sample of the same rows)."""
    import ctypes
    import oracle
    from paper_2511_10676_amd import datagen
    mac_per_token = w.r * (w.d + w.E)
    threads = oracle.num_threads()
    est_rate = 1.5e9 * threads                              # MAC/s guess used only to size the sample
    tokens = int(max(1, min(T * w.L, budget_s * est_rate / mac_per_token)))
    layers = max(1, min(w.L, tokens // T)) if T <= tokens else 1
    Ts = min(T, tokens // layers)
    inputs = [datagen.make_layer(w, l, Ts) for l in range(layers)]
    dt = _oracle_pass(w, inputs)
    out = {"value": round(layers * Ts / dt, 1), "unit": "tokens*layers/s", "cores": threads,
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"layers 0..{layers - 1} of {w.L}, first {Ts} of {T} tokens each: predict + group + score"}
    # one thread: the OpenMP runtime the oracle was built against is told to use one (the oracle is not changed)
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        T1 = int(max(1, min(Ts, budget_1t_s * 1.5e9 / mac_per_token)))
        lay1 = [datagen.make_layer(w, 0, T1)]
        omp.omp_set_num_threads(1)
        try:
            dt1 = _oracle_pass(w, lay1)
        finally:
            omp.omp_set_num_threads(threads)
        out["single_thread"] = {"value": round(T1 / dt1, 1), "unit": "tokens*layers/s", "cores": 1,
                                "seconds": round(dt1, 2), "sample": f"layer 0, first {T1} of {T} tokens"}
    except OSError:
        out["single_thread"] = None
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="deepseek_v2_lite")
    ap.add_argument("--T", type=int, default=0, help="tokens per layer (default: the workload's prefill size)")
    ap.add_argument("--k-pred", type=int, default=0,
                    help="experts predicted per token (default: the workload's k; larger = over-provisioned "
                         "prediction scored against the router's k labels)")
    ap.add_argument("--pipeline", action="store_true",
                    help="two streams: a step's grouping/scoring runs beside the next step's predict (+2%% steps/s "
                         "at prefill sizes, slower at decode sizes, and the predict kernel is then timed under "
                         "contention)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--counted", action="store_true",
                    help="predict through paep_predict_counted: activation counts accumulated in the predictor's "
                         "epilogue (for pricing that option; the step still runs group_by_expert)")
    ap.add_argument("--only", action="store_true",
                    help="time only the chosen token count (skip the workload's other token counts and the "
                         "over-provisioned width)")
    ap.add_argument("--sweep", action="store_true", help="accepted for compatibility: the sweep is the default")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="first run one plain device copy of this many MiB (a kernel of known traffic, for "
                         "scaling hardware byte counters collected over the same run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; --gpus must be 1 (the path shards by tokens or layers "
                 "with no communication in predict)")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2511_10676_amd import configs
    w = configs.get(args.workload)
    if w.dtype != "bf16":
        sys.exit("bench.py: choose a bf16 workload")
    T = args.T or w.prefill_T[0]
    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    from paper_2511_10676_amd import binding as B
    ceilings = device_ceilings(torch, B)
    banks = Banks(w)
    run = Runner(w, T, banks, k_pred=args.k_pred or None, pipelined=args.pipeline, counted=args.counted)
    main_rep = run.report(args.steps, args.warmup)
    line = {
        "metric": "predicted tokens*layers per second",
        "value": main_rep["value"], "unit": "tokens*layers/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_rep["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped: L={w.L} d={w.d} r={w.r} E={w.E} k={w.k}, T={T} tokens/layer "
                               f"({main_rep['path']} path, {main_rep['launch']}), step = predict + group_by_expert "
                               f"+ score, all layers",
                   "k_pred": run.k_pred, "counted_predict": bool(args.counted),
                   "streams": ("2: group_by_expert + score of step i run beside predict of step i+1"
                               if run.pipelined else "1"),
                   "weight_banks": main_rep["weight_banks"],
                   "score_layer0": main_rep["score_layer0"], "activation_entropy_layer0": run.entropy0,
                   "score_layer0_meaning": "exact-match rows, correctly predicted experts, rows whose labels are all predicted, top-1 hits, out of T rows"},
        "timing": main_rep["timing"],
        "roofline": main_rep["roofline"],
        "achievable": ceilings,
    }
    del run
    torch.cuda.empty_cache()
    if not args.only:
        # the rest of the metric: the workload's other token counts (decode sizes: HBM roofline), then the
        # headline size again predicting the over-provisioned width and scored against the router's k labels
        also = []
        kp0 = args.k_pred or None
        cases = [(T2, kp0) for T2 in list(w.decode_T) + list(w.prefill_T) if T2 != T]
        if w.k_over and not args.k_pred:
            cases.append((T, w.k_over))
        for T2, kp in cases:
            r2 = Runner(w, T2, banks, k_pred=kp, pipelined=args.pipeline)
            rep = r2.report(max(args.steps, 50) if T2 <= 64 else args.steps, args.warmup)
            if kp == kp0:
                rep.pop("score_layer0")
            else:
                rep["score_layer0_meaning"] = (f"k_pred={kp} predicted against k={w.k} labels: exact-match rows (0 by "
                                               "definition when the widths differ), correctly predicted experts, "
                                               "rows whose labels are all predicted, top-1 hits")
            also.append(rep)
            del r2
            torch.cuda.empty_cache()
        line["also"] = also
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w, T)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
