#!/usr/bin/env python3
"""Benchmark of one tree-verification step (s4c_tree_attn + s4c_accept_path + s4c_kv_compact)
on one MI355X, on seeded synthetic inputs already resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--warm] [--graph] [--no-cpu-baseline]

Prints ONE JSON line: steps/s for the whole step on the headline workload (config 5), the roofline
object of the dominant kernel (tree attention) and of the acceptance scan, the KV-read rate, a
`configs` array with the same figures for configs 1-4, and the CPU oracle timed on the host cores
on a bounded sample of the headline workload (a reported baseline, not a target).

Cache state: the inputs of configs 1-4 fit (or nearly fit) in the 256 MB last-level cache, so by
default the timed steps rotate through distinct copies of all inputs such that about 1 GB is
touched between two uses of the same copy ("cold"); --warm re-uses one copy.  Config 5 streams
2.7 GB per step and needs no rotation.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
FP32_VALU_PEAK_TFLOPS = 157.3


def workload_name(cfg):
    return ("cfg%d %s: B%d Hq%d/Hkv%d D%d %s prefix%d tree%d(levels %d) vocab%d %s + compaction"
            % (cfg.index, cfg.name, cfg.B, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype, cfg.P, cfg.N, cfg.levels, cfg.V, cfg.mode))


def cpu_baseline(cfg, par, at, ac, budget_s=15.0):
    """Time the oracle (as it stands) on the host cores on a bounded sample and scale to a step."""
    import numpy as np
    from oracle import s4c_oracle as O
    rng = np.random.default_rng(1)
    total_rows = cfg.B * cfg.N * cfg.Hq
    threads = O.num_threads()
    # calibrate attention cost on a few rows, then size the sample for ~budget_s
    def rows(n):
        return np.stack([rng.integers(0, cfg.B, n), rng.integers(0, cfg.N, n), rng.integers(0, cfg.Hq, n)], 1).astype(np.int32)
    n0 = max(threads * 2, 8)
    t0 = time.perf_counter()
    O.tree_attn_sampled(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par, rows(n0))
    dt0 = time.perf_counter() - t0
    n = int(min(total_rows, max(n0, n0 * (0.6 * budget_s) / max(dt0, 1e-6))))
    t0 = time.perf_counter()
    O.tree_attn_sampled(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par, rows(n))
    t_attn = (time.perf_counter() - t0) * total_rows / n
    # acceptance + compaction: the whole batch (cheap next to attention)
    nb = cfg.B
    t0 = time.perf_counter()
    r = O.accept_path(ac.logits[:nb], par[:nb], ac.tokens[:nb], cfg.mode, cfg.levels, ac.p_draft[:nb], ac.uniforms[:nb],
                      cfg.temperature)
    t_acc = (time.perf_counter() - t0) * cfg.B / nb
    kc, vc, cl = at.k_cache[:nb].copy(), at.v_cache[:nb].copy(), at.cache_len[:nb].copy()
    t0 = time.perf_counter()
    O.kv_compact(at.k_tree[:nb], at.v_tree[:nb], kc, vc, cl, r["path"], r["accept_len"])
    t_cmp = (time.perf_counter() - t0) * cfg.B / nb
    t_step = t_attn + t_acc + t_cmp
    return {"value": 1.0 / t_step, "unit": "steps/s", "cores": threads, "kind": "oracle",
            "sample": "attention oracle on %d of %d (sequence,node,head) rows scaled x%.1f; acceptance+compaction "
                      "oracle on %d of %d sequences scaled; est. %.1f s per full step" % (n, total_rows, total_rows / n, nb, cfg.B, t_step)}


def _timed_ms(torch, fn, reps=10):
    """Mean time of `reps` back-to-back calls, by events on the current stream."""
    fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


ATTN_SOURCES = ("tree_attn_mfma.hip", "tree_attn_mfma_smallm.hip", "tree_attn_generic.hip", "mfma_common.h")


def csrc_digest(names=None):
    """Digest of the library's sources (all of them with the public header, or the named files of csrc/): a
    committed HBM-traffic figure is only quoted for the kernels it was measured on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2506_14158_amd", "csrc")
    files = sorted(glob.glob(os.path.join(csrc, "*.h*"))) if names is None else [os.path.join(csrc, n) for n in names]
    for f in files + ([os.path.join(ROOT, "include", "s4c.h")] if names is None else []):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def committed_traffic(cfg_index, kv_splits):
    """HBM bytes per s4c_tree_attn call from the committed rocprofv3 --pmc summary (profiles/traffic.json), or
    None if there is none for this config or it was taken on other sources of the attention kernels or with another
    number of KV splits (the planner's choice)."""
    try:
        tr = json.load(open(os.path.join(ROOT, "profiles", "traffic.json"))).get("cfg%d" % cfg_index)
    except (OSError, ValueError):
        return None
    if not tr or tr.get("attn_src_sha16") != csrc_digest(ATTN_SOURCES) or tr.get("kv_splits") != kv_splits:
        return None
    return tr


class Workload:
    """One config's seeded inputs on the device (rotating copies unless warm), outputs and workspaces."""

    def __init__(self, cfg, warm, resample=False):
        import torch
        from paper_2506_14158_amd import binding as B, synth
        from paper_2506_14158_amd.verify import TreeVerifier
        from paper_2506_14158_amd.device import to_device
        self.cfg = cfg
        self.par = synth.make_parent(cfg)
        self.at = synth.make_attn_inputs(cfg, threads=16)
        self.ac = synth.make_accept_inputs(cfg, self.par, threads=16, full_draft=resample)
        d0 = to_device(cfg, self.par, self.at, self.ac)
        self.in_bytes = sum(v.numel() * v.element_size() for v in d0.values())
        self.ncopy = 1 if warm else int(max(1, min(64, -(-(1 << 30) // self.in_bytes))))
        self.copies = [d0] + [{k: v.clone() for k, v in d0.items()} for _ in range(self.ncopy - 1)]
        self.tv = TreeVerifier(cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, cfg.S_cap, cfg.V, d0["q"].dtype, cfg.levels, cfg.P)
        self.mode = B.S4C_GREEDY if cfg.mode == "greedy" else B.S4C_STOCHASTIC
        self.cache_len0 = d0["cache_len"].clone()
        self.warm = warm

    def step(self, ev=None, k=0):
        d, tv, cfg = self.copies[k % self.ncopy], self.tv, self.cfg
        # compaction advances cache_len; put it back so every step verifies the same tree
        d["cache_len"].copy_(self.cache_len0)
        if ev:
            ev[0].record()
        tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
        if ev:
            ev[1].record()
        tv.accept_path(d["logits"], d["parent"], d["tokens"], self.mode, d["p_draft"], d["uniforms"], cfg.temperature)
        if ev:
            ev[2].record()
        tv.kv_compact(d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"])
        if ev:
            ev[3].record()

    def cache_note(self):
        return ("warm: one input copy re-used" if self.warm else
                "cold: %d rotating input copies, %.0f MB touched between reuses" % (self.ncopy, self.ncopy * self.in_bytes / 1e6))


def time_steps(w, steps, warmup):
    """W untimed steps, then K timed ones: wall clock around all of them, HIP events (on the launch stream)
    around every call."""
    import numpy as np
    import torch
    for k in range(warmup):
        w.step(None, k)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        w.step(events[k], warmup + k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = lambda a, b: np.array([e[a].elapsed_time(e[b]) for e in events])
    return {"wall_s": dt, "attn": ms(0, 1), "accept": ms(1, 2), "compact": ms(2, 3), "step": ms(0, 3)}


def rooflines(w, t):
    """Roofline objects of s4c_tree_attn (the dominant call) and s4c_accept_path from the event times."""
    import numpy as np
    cfg, tv = w.cfg, w.tv
    es = cfg.es
    t_attn, t_acc = float(t["attn"].mean()) * 1e-3, float(t["accept"].mean()) * 1e-3
    kv_bytes = cfg.B * cfg.Hkv * (cfg.P + cfg.N) * cfg.D * 2 * es
    qo_bytes = 2 * cfg.B * cfg.N * cfg.Hq * cfg.D * es
    flops = 4.0 * cfg.B * cfg.Hq * cfg.N * (cfg.P + cfg.N) * cfg.D
    hbm_frac = kv_bytes / t_attn / 1e9 / HBM_PEAK_GBPS
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9)
    if cfg.dtype in ("bf16", "f16"):
        mfma_frac = flops / t_attn / 1e12 / MFMA_BF16_PEAK_TFLOPS
        if flops / kv_bytes > ridge:
            roof = {"bound": "mfma", "achieved": flops / t_attn / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
        else:
            roof = {"bound": "hbm", "achieved": kv_bytes / t_attn / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
    else:
        mfma_frac = None        # fp32 data runs on the vector ALUs; config 1 is launch-latency bound
        roof = {"bound": "hbm", "achieved": kv_bytes / t_attn / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["frac_of_hbm_peak_kv_read"] = hbm_frac
    roof["frac_of_mfma_peak"] = mfma_frac
    tr = committed_traffic(cfg.index, tv.num_splits)
    roof["traffic"] = (tr["fetch_bytes"] + tr["write_bytes"]) if tr else None
    roof["traffic_source"] = ("%s, commit %s" % (tr["source"], tr["taken_at_commit"])) if tr else None
    roof["traffic_over_algorithmic"] = (roof["traffic"] / float(kv_bytes + qo_bytes)) if tr else None
    roof["kernel"] = "s4c_tree_attn (%d KV split%s)" % (tv.num_splits, "" if tv.num_splits == 1 else "s")
    roof["ms"] = t_attn * 1e3
    roof["ms_median"] = float(np.median(t["attn"]))
    roof["ms_min"] = float(t["attn"].min())
    # the acceptance scan reads every logits row in greedy mode (the bonus token may come from any row) and
    # only the rows of nodes with children in stochastic mode (a leaf's row verifies nobody)
    rows = cfg.B * cfg.N if cfg.mode == "greedy" else int(sum((np.bincount(p[1:], minlength=cfg.N) > 0).sum() for p in w.par))
    logits_bytes = rows * cfg.V * es
    acc = {"bound": "hbm", "achieved": logits_bytes / t_acc / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
           "frac": logits_bytes / t_acc / 1e9 / HBM_PEAK_GBPS, "kernel": "s4c_accept_path", "rows_scanned": rows,
           "bytes": logits_bytes, "ms": t_acc * 1e3, "ms_median": float(np.median(t["accept"])), "ms_min": float(t["accept"].min())}
    return roof, acc, kv_bytes, flops


def config_summary(w, t):
    """The per-config object of the `configs` array (configs other than the headline one)."""
    import numpy as np
    roof, acc, kv_bytes, flops = rooflines(w, t)
    return {"workload": workload_name(w.cfg), "kv_splits": w.tv.num_splits, "cache": w.cache_note(),
            "ms_per_step": float(t["step"].mean()), "ms_median": float(np.median(t["step"])), "ms_min": float(t["step"].min()),
            "steps_per_s_wall": len(t["step"]) / t["wall_s"],
            "phases_ms": {"tree_attn": float(t["attn"].mean()), "accept_path": float(t["accept"].mean()),
                          "kv_compact": float(t["compact"].mean())},
            "roofline": roof, "accept_roofline": acc}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="1..5 (the five benchmark configs); 5 is the headline workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="only the selected config's step: skip the `configs` array (the other four configs timed the same "
                         "way, a few seconds each) and the legs of the other entry points that a plain run adds "
                         "(accept_resample, build_tree, draft_linear, multi_layer with 2 layers)")
    ap.add_argument("--no-probes", action="store_true", help="skip the measured-ceiling probes (measured_peaks)")
    ap.add_argument("--warm", action="store_true", help="re-use one input copy every step (cache-warm numbers)")
    ap.add_argument("--resample", action="store_true",
                    help="also time s4c_accept_resample (sequential rule with the correction token; stochastic "
                         "configs only; reported as accept_resample, not part of the step)")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE",
                    help="also time s4c_tree_attn_paged with this page size (power of two >= 64) through a shuffled "
                         "block table (reported as paged_attn)")
    ap.add_argument("--draft-linear", action="store_true",
                    help="also time s4c_draft_linear (Eq. 3) on the config's B*N tokens with hidden size Hq*D "
                         "(bf16 configs; reported as draft_linear, not part of the step)")
    ap.add_argument("--build-tree", action="store_true",
                    help="also time s4c_build_tree on bf16 draft logits of the config's shape (reported as "
                         "build_tree, not part of the step)")
    ap.add_argument("--layers", type=int, default=0,
                    help="also time a whole-model verify: this many layers of tree attention (each with its own KV "
                         "cache), one acceptance, one s4c_commit_path over all layers + feature rows (reported as "
                         "multi_layer, not part of the step)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph (reported as graph_ms_per_step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 3 plain 1 GiB device-to-device copies (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--dtype", choices=("config", "bf16", "f16"), default="config",
                    help="storage type of Q/K/V/cache/logits: the config's own (bf16 for configs 2-5), or fp16, the "
                         "precision of the paper's experiments (Sec. 4.1); a non-default choice is named in config.workload")
    ap.add_argument("--constant-data", action="store_true",
                    help="also time s4c_tree_attn with every Q/K/V element set to 0.5 (same launches, same instruction "
                         "stream; reported as attn_constant_data: shows how much of the time is the data-dependent clock)")
    args = ap.parse_args()
    if not args.no_other_configs:
        # the full line also times the entry points outside the three-call step, on the selected config
        args.resample = args.build_tree = args.draft_linear = True
        args.layers = args.layers or 2
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the step has no cross-GPU part); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_14158_amd import binding as B, synth
    from paper_2506_14158_amd.verify import TreeVerifier

    B.lib()   # fail loudly if the HIP library is not built
    cfg = synth.CONFIGS[args.config]
    if args.dtype != "config" and args.dtype != cfg.dtype:
        if cfg.dtype == "f32":
            print("bench.py: config %d is an fp32 workload" % args.config, file=sys.stderr)
            sys.exit(2)
        cfg = synth.scaled(cfg, dtype=args.dtype)
    resample = args.resample and cfg.mode == "stochastic"
    w = Workload(cfg, args.warm, resample)
    par, at, ac, tv, copies, ncopy, mode, cache_len0 = w.par, w.at, w.ac, w.tv, w.copies, w.ncopy, w.mode, w.cache_len0
    d0 = copies[0]
    step = w.step

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    t = time_steps(w, args.steps, args.warmup)
    dt = t["wall_s"]
    ms_step = dt * 1e3 / args.steps
    t_attn = float(t["attn"].mean()) * 1e-3
    t_acc = float(t["accept"].mean()) * 1e-3
    t_cmp = float(t["compact"].mean()) * 1e-3
    roof, acc_roof, kv_bytes, flops = rooflines(w, t)

    rec = {
        "metric": "tree-verify steps/s and achieved KV-read HBM GB/s (fraction of MI355X peak)",
        "value": args.steps / dt, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_median": float(np.median(t["step"])), "ms_min": float(t["step"].min()),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic (seeded; stands in for Spec-Bench / Vicuna runs)",
        "config": {"workload": workload_name(cfg), "kv_splits": tv.num_splits, "cache": w.cache_note()},
        "roofline": roof,
        "accept_roofline": acc_roof,
        "kv_read": {"GBps": kv_bytes / t_attn / 1e9, "frac_of_hbm_peak": kv_bytes / t_attn / 1e9 / HBM_PEAK_GBPS,
                    "attn_TFLOPs": flops / t_attn / 1e12, "frac_of_mfma_peak": flops / t_attn / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "flop_per_kv_byte": flops / kv_bytes},
        "phases_ms": {"tree_attn": t_attn * 1e3, "accept_path": t_acc * 1e3, "kv_compact": t_cmp * 1e3},
        "accept_path_GBps": acc_roof["achieved"], "accept_rows_scanned": acc_roof["rows_scanned"],
        "csrc_sha16": csrc_digest(),
        "attn_src_sha16": csrc_digest(ATTN_SOURCES),
        "timing_note": "ms_per_step and value: wall clock around the K timed steps; ms_median / ms_min and every phase: "
                       "HIP events on the launch stream",
        "paper_context": "paper reports 2.26x-2.60x end-to-end vs autoregressive decoding (A100-40GB / 4xRTX4090, fp16, batch 1)",
    }
    if not args.no_other_configs:
        # configs 1-4 (short steps: at least 100 timed ones each), timed the same way; each frees its inputs
        # before the next is drawn
        others = []
        for idx in (1, 2, 3, 4):
            if idx == args.config:
                continue
            ocfg = synth.CONFIGS[idx]
            if args.dtype != "config" and ocfg.dtype != "f32":
                ocfg = synth.scaled(ocfg, dtype=args.dtype)
            ow = Workload(ocfg, args.warm)
            others.append(config_summary(ow, time_steps(ow, max(args.steps, 100), max(args.warmup, 10))))
            del ow
            torch.cuda.empty_cache()
        rec["configs"] = others
    if not args.no_probes:
        # what plain kernels reach on this GPU (context for the published peaks above)
        from paper_2506_14158_amd import probe
        sink = probe.mfma_sink()
        big = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(1)

        def timed(fn, reps=3):
            best = 1e30
            for _ in range(reps + 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                out = fn()
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e-3)
            return best, out

        t_rd, _ = timed(lambda: probe.stream_read(big, sink))
        t_c, fl = timed(lambda: probe.mfma_bf16(False, 16000, sink))
        t_r, _ = timed(lambda: probe.mfma_bf16(True, 16000, sink))
        t_r16, _ = timed(lambda: probe.mfma_bf16(True, 16000, sink, shape=1))
        del big
        meas = {"hbm_stream_read_GBps": (1 << 31) / t_rd / 1e9, "mfma_bf16_TFLOPs_constant_operands": fl / t_c / 1e12,
                "mfma_bf16_TFLOPs_normal_operands": fl / t_r / 1e12,
                "mfma_bf16_16x16x32_TFLOPs_normal_operands": fl / t_r16 / 1e12,
                "note": "plain probe kernels on this GPU (32x32x16 unless named); the matrix-core clock drops with random operand data"}
        rec["measured_peaks"] = meas
        roof["frac_of_measured"] = roof["achieved"] / (meas["mfma_bf16_TFLOPs_normal_operands"] if roof["bound"] == "mfma"
                                                       else meas["hbm_stream_read_GBps"])
    if resample:
        d = copies[0]
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for k in range(args.warmup + args.steps):
            e = evs[k - args.warmup] if k >= args.warmup else None
            if e:
                e[0].record()
            tv.accept_resample(d["logits"], d["draft_probs"], d["parent"], d["tokens"], d["uniforms"], d["u_resample"],
                               cfg.temperature)
            if e:
                e[1].record()
        torch.cuda.synchronize()
        ms = np.array([a.elapsed_time(b) for a, b in evs])
        L = tv.accept_len.cpu().numpy()
        rec["accept_resample"] = {"ms": float(ms.mean()), "ms_min": float(ms.min()), "dtype": "f64",
                                  "accept_len_mean": float(L.mean()), "accept_len_max": int(L.max())}
    if args.paged:
        d, page = copies[0], args.paged
        max_blocks = -(-cfg.S_cap // page)
        S_log = max_blocks * page
        num_pages = cfg.B * max_blocks
        perm = torch.randperm(num_pages, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3))
        bt = perm.view(cfg.B, max_blocks).to(torch.int32).contiguous()

        def to_pool(c):      # [B][Hkv][S_cap][D] -> [num_pages][Hkv][page][D] in block-table order
            pad = torch.zeros(cfg.B, cfg.Hkv, S_log, cfg.D, dtype=c.dtype, device="cuda")
            pad[:, :, :cfg.S_cap] = c
            pages = pad.view(cfg.B, cfg.Hkv, max_blocks, page, cfg.D).permute(0, 2, 1, 3, 4).reshape(num_pages, cfg.Hkv, page, cfg.D)
            pool = torch.empty_like(pages)
            pool[perm.long()] = pages
            return pool

        kp, vp = to_pool(d["k_cache"]), to_pool(d["v_cache"])
        tvp = TreeVerifier(cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, S_log, cfg.V, d["q"].dtype, cfg.levels, cfg.P)
        d["cache_len"].copy_(cache_len0)
        run_p = lambda: B.s4c_tree_attn_paged(d["q"], d["k_tree"], d["v_tree"], kp, vp, bt, d["cache_len"], d["parent"], cfg.P,
                                              tvp.out, 0.0, tvp.attn_status, tvp.attn_ws)
        t_p = min(_timed_ms(torch, run_p, reps=max(3, args.steps // 2)) for _ in range(3))
        tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
        torch.cuda.synchronize()
        rec["paged_attn"] = {"page_size": page, "ms": t_p, "contiguous_ms": t_attn * 1e3,
                             "same_bits_as_contiguous": bool(torch.equal(tvp.out.view(torch.int16), tv.out.view(torch.int16)))
                             if cfg.dtype != "f32" else None}
        del kp, vp
    if args.draft_linear and cfg.dtype != "f32":
        dt_ = d0["q"].dtype
        Hd = cfg.Hq * cfg.D
        g = torch.Generator(device="cuda").manual_seed(1)
        rn = lambda *s_: torch.randn(*s_, device="cuda", generator=g)
        W_ = (rn(Hd, 2 * Hd) / (2 * Hd) ** 0.5).to(dt_)
        b_ = rn(Hd).to(dt_)
        best = lambda fn: min(_timed_ms(torch, fn) for _ in range(5))
        rec["draft_linear"] = []
        # the batch's B*N tree tokens (a dense contraction), and one tree's N tokens (<= 128: a stream over W)
        for Tn in (cfg.B * cfg.N, cfg.N):
            e_, f_ = rn(Tn, Hd).to(dt_), rn(Tn, Hd).to(dt_)
            o_ = torch.empty(Tn, Hd, dtype=dt_, device="cuda")
            ws_ = B.alloc_workspace(B.s4c_draft_linear_workspace_size(Tn, Hd, Hd))
            t_dl = best(lambda: B.s4c_draft_linear(e_, f_, W_, o_, b_, ws_))
            t_lib = best(lambda: torch.addmm(b_, torch.cat([e_, f_], 1), W_.t()))
            fl = 2.0 * Tn * 2 * Hd * Hd
            w_bytes = 2.0 * Hd * Hd * W_.element_size()
            rec["draft_linear"].append({"tokens": Tn, "hidden": Hd, "ms": t_dl, "TFLOPs": fl / t_dl / 1e9,
                                        "frac_of_mfma_peak": fl / t_dl / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                        "W_GBps": w_bytes / t_dl / 1e6, "W_frac_of_hbm_peak": w_bytes / t_dl / 1e6 / HBM_PEAK_GBPS,
                                        "torch_cat_addmm_ms": t_lib, "torch_TFLOPs": fl / t_lib / 1e9})
            del e_, f_, o_, ws_
        del W_
    if args.build_tree:
        d = copies[0]
        nchild = torch.zeros(cfg.B, cfg.N, dtype=torch.int32, device="cuda")
        nchild.scatter_add_(1, d["parent"][:, 1:].long(), torch.ones(cfg.B, cfg.N - 1, dtype=torch.int32, device="cuda"))
        dl = d["logits"] if d["logits"].dtype == torch.bfloat16 else d["logits"].clone()   # any rows of the right shape
        ws = B.alloc_workspace(B.s4c_build_tree_workspace_size(cfg.B, cfg.N, cfg.V))
        o_par, o_tok = torch.empty_like(d["parent"]), torch.empty_like(d["parent"])
        o_pd = torch.empty(cfg.B, cfg.N, dtype=torch.float32, device="cuda")
        root = d["tokens"][:, 0].contiguous()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for k in range(args.warmup + args.steps):
            e = evs[k - args.warmup] if k >= args.warmup else None
            if e:
                e[0].record()
            B.s4c_build_tree(dl, nchild, root, 8, o_par, o_tok, o_pd, ws, cfg.temperature)
            if e:
                e[1].record()
        torch.cuda.synchronize()
        assert torch.equal(o_par, d["parent"])
        ms = np.array([a.elapsed_time(b) for a, b in evs])
        rows = int((nchild > 0).sum())
        rec["build_tree"] = {"ms": float(ms.mean()), "ms_min": float(ms.min()), "rows_scanned": rows,
                             "GBps": rows * cfg.V * dl.element_size() / (float(ms.mean()) * 1e-3) / 1e9}
    if args.layers > 0:
        # every layer gets its own K/V cache and tree K/V (device copies of the same synthetic layer)
        Ly, d = args.layers, copies[0]
        rep = lambda t: t.unsqueeze(0).repeat(Ly, *([1] * t.dim())).contiguous()
        kcL, vcL, ktL, vtL = rep(d["k_cache"]), rep(d["v_cache"]), rep(d["k_tree"]), rep(d["v_tree"])
        hidden = cfg.Hq * cfg.D
        feats = torch.randn(cfg.B, cfg.N, hidden, device="cuda").to(d["q"].dtype)
        fout = torch.zeros(cfg.B, cfg.levels, hidden, device="cuda", dtype=d["q"].dtype)

        def model_step():
            d["cache_len"].copy_(cache_len0)
            for l in range(Ly):
                tv.tree_attn(d["q"], ktL[l], vtL[l], kcL[l], vcL[l], d["cache_len"], d["parent"])
            tv.accept_path(d["logits"], d["parent"], d["tokens"], mode, d["p_draft"], d["uniforms"], cfg.temperature)
            tv.commit_path(ktL, vtL, kcL, vcL, d["cache_len"], feats, fout)

        nsteps = max(2, min(args.steps, 10))
        model_step()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        t0 = time.perf_counter()
        for k in range(nsteps):
            model_step()
        torch.cuda.synchronize()
        ms_model = (time.perf_counter() - t0) * 1e3 / nsteps
        d["cache_len"].copy_(cache_len0)
        ev[0].record()
        tv.commit_path(ktL, vtL, kcL, vcL, d["cache_len"], feats, fout)
        ev[1].record()
        torch.cuda.synchronize()
        rec["multi_layer"] = {"layers": Ly, "ms_per_step": ms_model, "steps_per_s": 1e3 / ms_model,
                              "commit_path_ms": ev[0].elapsed_time(ev[1]),
                              "kv_cache_GB": 2 * kcL.numel() * kcL.element_size() / 1e9}
        if args.graph:
            # the same whole-model step replayed from one captured HIP graph (no per-launch host work)
            side = torch.cuda.Stream()
            gm = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                with torch.cuda.graph(gm, stream=side):
                    model_step()
            gm.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(nsteps):
                gm.replay()
            torch.cuda.synchronize()
            rec["multi_layer"]["graph_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / nsteps
            del gm
        del kcL, vcL, ktL, vtL
    if args.graph:
        # launch-bound configs: one graph launch instead of six kernel launches per step
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for k in range(ncopy):
                    step(None, k)
        reps = max(1, args.steps // ncopy)
        for _ in range(max(1, args.warmup // ncopy)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        rec["graph_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / (reps * ncopy)
    if args.constant_data:
        # last GPU leg: it overwrites the inputs of copy 0
        d = copies[0]
        d["cache_len"].copy_(cache_len0)
        for name in ("q", "k_tree", "v_tree", "k_cache", "v_cache"):
            d[name].fill_(0.5)
        run = lambda: tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
        for _ in range(max(1, args.warmup)):
            run()
        ms = _timed_ms(torch, run, reps=max(3, min(args.steps, 20)))
        rec["attn_constant_data"] = {"ms": ms, "TFLOPs": flops / ms / 1e9, "GBps": kv_bytes / ms / 1e6,
                                     "note": "every Q/K/V element 0.5; compare phases_ms.tree_attn (seeded N(0,1) data)"}
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(cfg, par, at, ac)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
