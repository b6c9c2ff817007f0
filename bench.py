#!/usr/bin/env python3
"""Benchmark of the DSA attention forward on one MI355X.

Workload: the long-sequence configuration the headline metric is quoted on (B=2, H=8, L=4096,
d=64, bf16, k=32 int8 projections, keep 5% = 205 keys), run fine-grained and vector-wise (8x1)
side by side on the same seeded synthetic tensors.  One step = one fine-grained forward plus
one vector-wise forward through dsa_attention_fwd (mask prediction, SDDMM, softmax over kept
entries, SpMM), inputs resident in HBM.  value = heads*sequences processed per second over
both passes.

Prints ONE JSON line with the throughput, the roofline entry of the dominant kernel of the step
(the fine-grained mask predictor: bound by plain vector-ALU work on the N*L*L approximate scores,
with its int8 matrix-core rate beside it), a second entry for the fine-grained attention kernel
against a gather roof measured in the same run (its K / V rows come from L2, so the HBM peak is not
its roof), per-stage times of every workload configuration, and the CPU oracle timed on the host
cores on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
# plain vector ALU: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = one 32-bit lane operation each
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9

PMC_COPY_BYTES = 256 << 20   # size of the calibration copy in --pmc-mode
# HBM bytes per launch come from two rocprofv3 --pmc runs of `bench.py --pmc-mode` (FETCH_SIZE, then
# WRITE_SIZE), each scaled by what the same counter reads for the calibration copy.  Their summary is a
# tracked file; this run does not measure them, it quotes the row of the kernel it names (or null).
TRAFFIC_SUMMARY = ROOT / "profiles" / "bench_C4_hbm_traffic.md"


COUNTER_SUMMARY = ROOT / "profiles" / "bench_C4_pmc_counters.md"


def profiled_ratio(row_prefix: str, kernel_prefix: str):
    """A cell of the derived-ratio table in the tracked counter summary (row by the start of its label,
    column by the start of the kernel's name); None if the file, the row or the column is missing."""
    try:
        header = None
        for line in COUNTER_SUMMARY.read_text().splitlines():
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if cells and cells[0] == "ratio":
                header = [c.strip("`") for c in cells]
            elif header and cells[0].startswith(row_prefix):
                for name, cell in zip(header[1:], cells[1:]):
                    if name.startswith(kernel_prefix):
                        return float(cell)
    except (OSError, ValueError):
        pass
    return None


def profiled_traffic_bytes(kernel_prefix: str):
    """Total HBM bytes per launch of the first kernel whose name starts with kernel_prefix in the
    tracked FETCH_SIZE / WRITE_SIZE summary; None if the file or the row is missing."""
    try:
        for line in TRAFFIC_SUMMARY.read_text().splitlines():
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 6 and cells[0].strip("`").startswith(kernel_prefix):
                return float(cells[5]) * 1e6
    except (OSError, ValueError):
        pass
    return None


def gather_bytes(cfg) -> int:
    """Algorithmic bytes of SDDMM + softmax + SpMM: every kept K row and V row is read once per
    selection unit, Q read once, O written once (fp32), the index lists read once."""
    e = 4 if cfg.dtype == "f32" else 2
    G = cfg.units
    rows = cfg.N * cfg.L
    return 2 * G * cfg.keep * cfg.d * e + rows * cfg.d * e + rows * cfg.d * 4 + G * cfg.keep * 4


def compulsory_bytes(cfg) -> int:
    """Q, K, V and the index lists read once, O written once: what must cross the HBM interface."""
    e = 4 if cfg.dtype == "f32" else 2
    rows = cfg.N * cfg.L
    return 3 * rows * cfg.d * e + rows * cfg.d * 4 + cfg.units * cfg.keep * 4


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip timing every stage on the other workload configs ('all_configs' is then null)")
    ap.add_argument("--no-low-precision", action="store_true",
                    help="skip the INT4 / INT2 predictor (for a kernel trace in which the dominant kernel is launched "
                         "on the int8 workload only; 'low_precision_predict' is then empty)")
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for rocprofv3 --pmc runs: a few steps plus one plain device copy of known size "
                         "(calibrates FETCH_SIZE / WRITE_SIZE), no other output")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every head*sequence is an independent problem and "
              "would shard over GPUs with no exchange step, but no multi-GPU path is built); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import dsa_inputs as di
    import paper_2110_11299_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    pkg.binding.lib()   # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)

    cf, cv = di.CONFIGS["C4f"], di.CONFIGS["C4v"]
    x = di.make_inputs(cf)

    def dev(name):
        return torch.from_numpy(x.storage(name).view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V = dev("Q"), dev("K"), dev("V")
    Qt, Kt = torch.from_numpy(x.Qt).cuda(), torch.from_numpy(x.Kt).cuda()
    passes = []
    for cfg in (cf, cv):
        sh = pkg.make_shape(cfg.B, cfg.H, cfg.L, cfg.d, cfg.k, cfg.keep, cfg.vec, pkg.DSA_BF16, float(cfg.scale))
        passes.append(dict(cfg=cfg, sh=sh,
                           O=torch.empty((cfg.B, cfg.H, cfg.L, cfg.d), dtype=torch.float32, device="cuda"),
                           idx=torch.empty((cfg.B, cfg.H, cfg.L // cfg.vec, cfg.keep), dtype=torch.int32, device="cuda"),
                           ws=pkg.binding.alloc_workspace(sh)))

    def step():
        for p in passes:
            pkg.dsa_attention_fwd(p["sh"], Q, K, V, Qt, Kt, O=p["O"], idx_out=p["idx"], ws=p["ws"])

    if args.pmc_mode:
        for _ in range(3):
            step()
        rm = torch.empty((cf.B, cf.H, cf.L), dtype=torch.int32, device="cuda")
        for _ in range(3):
            pkg.dsa_approx_rowmax(passes[0]["sh"], Qt, Kt, rowmax=rm)
        pkg.binding.dsa_gather_roof(passes[0]["sh"], K, V, passes[0]["idx"])
        # nothing but int8 matrix instructions: what the matrix-core busy counter reads when the cores are full
        pkg.dsa_mfma_i8_sustained(2048, 512, torch.empty(2048 * 256, dtype=torch.int32, device="cuda"))
        src = torch.empty(PMC_COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads and writes PMC_COPY_BYTES each
        torch.cuda.synchronize()
        print(json.dumps({"pmc_mode": True, "copy_bytes": PMC_COPY_BYTES}))
        return 0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    heads_seqs = sum(p["cfg"].N for p in passes)
    value = heads_seqs / (ms_per_step * 1e-3)

    # Per-kernel durations, same kernels and launch shapes, HIP events on the launch stream.
    def timed(fn, reps):
        """Average duration of one call in a run of reps back-to-back calls on the launch stream (one pair of
        HIP events around the run: an event between two launches would add its own gap to each)."""
        fn()
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        first.record()
        for _ in range(reps):
            fn()
        last.record()
        torch.cuda.synchronize()
        return first.elapsed_time(last) / reps   # ms

    reps = max(args.steps, 5)

    def stage_times(cfg, shc, q, kk, v, qt, kt, o, ix, wsc):
        """Every kernel of one configuration: the fused path and the staged entry points."""
        S = torch.empty((cfg.B, cfg.H, cfg.L, cfg.keep), dtype=torch.float32, device="cuda")
        st = dict(
            predict_ms=timed(lambda: pkg.dsa_predict_mask(shc, qt, kt, idx=ix, ws=wsc), reps),
            attention_ms=timed(lambda: pkg.dsa_masked_attention(shc, q, kk, v, ix, O=o), reps),
            fwd_ms=timed(lambda: pkg.dsa_attention_fwd(shc, q, kk, v, qt, kt, O=o, idx_out=ix, ws=wsc), reps),
            staged_sddmm_ms=timed(lambda: pkg.dsa_sddmm(shc, q, kk, ix, S=S), reps),
            staged_softmax_ms=timed(lambda: pkg.dsa_sparse_softmax(shc, S, P=S), reps),
            staged_spmm_ms=timed(lambda: pkg.dsa_spmm(shc, S, ix, v, O=o), reps))
        st["heads_seqs_per_s"] = cfg.N / (st["fwd_ms"] * 1e-3)
        # gathered (algorithmic) bytes are served by L2, not by HBM: a rate, not a fraction of the HBM peak
        st["attention_gather_GBs"] = gather_bytes(cfg) / (st["attention_ms"] * 1e-3) / 1e9
        st["attention_compulsory_GBs"] = compulsory_bytes(cfg) / (st["attention_ms"] * 1e-3) / 1e9
        st["attention_frac_hbm_compulsory"] = st["attention_compulsory_GBs"] / HBM_PEAK_GBS
        ops = 2.0 * cfg.N * cfg.L * cfg.L * cfg.k
        st["predict_int8_TOPS"] = ops / (st["predict_ms"] * 1e-3) / 1e12
        st["predict_frac_int8"] = st["predict_int8_TOPS"] / INT8_PEAK_TOPS
        # the predictor is bound by the selection: one inspection of every (unit, key) score at least
        scores = float(cfg.N) * (cfg.L // cfg.vec) * cfg.L
        st["predict_Gscores_per_s"] = scores / (st["predict_ms"] * 1e-3) / 1e9
        st["predict_frac_alu"] = st["predict_Gscores_per_s"] * 1e9 / ALU_PEAK_LANE_OPS
        return st

    stages = {}
    for p in passes:
        stages[p["cfg"].name] = stage_times(p["cfg"], p["sh"], Q, K, V, Qt, Kt, p["O"], p["idx"], p["ws"])
    sh_f = passes[0]["sh"]
    # the step in front of the path (not part of the timed step: Q~, K~ are inputs of the path)
    Rd = torch.from_numpy(x.R.astype(np.float32)).cuda()
    pws = torch.empty(pkg.binding.project_workspace_bytes(sh_f), dtype=torch.uint8, device="cuda")
    Qt2, Kt2 = torch.empty_like(Qt), torch.empty_like(Kt)

    def project_both():
        pkg.dsa_project_quantize(sh_f, Q, Rd, Xt=Qt2, ws=pws, want_amax=False)
        pkg.dsa_project_quantize(sh_f, K, Rd, Xt=Kt2, ws=pws, want_amax=False)

    project_ms = timed(project_both, reps)
    # the predictor at the paper's lower precisions (packed INT4 / INT2 codes made on the GPU)
    low_precision = {}
    for bits in (() if args.no_low_precision else (4, 2)):
        q_lp, _ = pkg.dsa_project_quantize_bits(sh_f, bits, Q, Rd, ws=pws, want_amax=False)
        k_lp, _ = pkg.dsa_project_quantize_bits(sh_f, bits, K, Rd, ws=pws, want_amax=False)
        ws_lp = torch.empty(pkg.binding.predict_workspace_bytes_bits(sh_f, bits), dtype=torch.uint8, device="cuda")
        idx_lp = torch.empty_like(passes[0]["idx"])
        ws_fwd = torch.empty(pkg.binding.workspace_bytes_bits(sh_f, bits), dtype=torch.uint8, device="cuda")
        low_precision[f"int{bits}"] = dict(
            predict_ms=timed(lambda: pkg.dsa_predict_mask_bits(sh_f, bits, q_lp, k_lp, idx=idx_lp, ws=ws_lp), reps),
            fwd_ms=timed(lambda: pkg.dsa_attention_fwd_bits(sh_f, bits, Q, K, V, q_lp, k_lp, O=passes[0]["O"],
                                                            idx_out=idx_lp, ws=ws_fwd), reps))
        del q_lp, k_lp, ws_lp, idx_lp, ws_fwd
    rowmax = torch.empty((cf.B, cf.H, cf.L), dtype=torch.int32, device="cuda")
    contraction_ms = timed(lambda: pkg.dsa_approx_rowmax(sh_f, Qt, Kt, rowmax=rowmax), reps)

    int8_ops = 2.0 * cf.N * cf.L * cf.L * cf.k
    contraction = dict(kernel="dsa_approx_rowmax", workload="C4: N=16 heads*seqs, L=4096, k=32", ms=contraction_ms,
                       int8_TOPS=int8_ops / (contraction_ms * 1e-3) / 1e12)
    contraction["frac_int8"] = contraction["int8_TOPS"] / INT8_PEAK_TOPS
    # the same contraction at L=4096 with 8x the heads*seqs (the C4 projections tiled): the launch and
    # pipeline-fill cost of a 12 us kernel no longer dominates
    rep = 8
    Qt8, Kt8 = Qt.repeat(rep, 1, 1, 1), Kt.repeat(rep, 1, 1, 1)
    sh8 = pkg.make_shape(cf.B * rep, cf.H, cf.L, cf.d, cf.k, cf.keep, 1, pkg.DSA_BF16, float(cf.scale))
    rowmax8 = torch.empty((cf.B * rep, cf.H, cf.L), dtype=torch.int32, device="cuda")
    ms8 = timed(lambda: pkg.dsa_approx_rowmax(sh8, Qt8, Kt8, rowmax=rowmax8), reps)
    contraction["batched"] = dict(workload=f"N={cf.N * rep} heads*seqs, L=4096, k=32", ms=ms8,
                                  int8_TOPS=rep * int8_ops / (ms8 * 1e-3) / 1e12,
                                  frac_int8=rep * int8_ops / (ms8 * 1e-3) / 1e12 / INT8_PEAK_TOPS)
    del Qt8, Kt8, rowmax8
    # what the matrix cores sustain on this chip with nothing but int8 MFMAs in flight
    sink = torch.empty(2048 * 256, dtype=torch.int32, device="cuda")
    pkg.dsa_mfma_i8_sustained(2048, 64, sink)
    mfma_ops = 4 * 2048 * 4 * 2048 * 65536
    mfma_ms = timed(lambda: pkg.dsa_mfma_i8_sustained(2048, 2048, sink), 3)
    contraction["mfma_i8_sustained_TOPS"] = mfma_ops / (mfma_ms * 1e-3) / 1e12

    # what a plain device copy reaches on this chip (bytes read + bytes written per second)
    csrc = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    copy_ms = timed(lambda: cdst.copy_(csrc), 5)
    copy_GBs = 2.0 * csrc.numel() / (copy_ms * 1e-3) / 1e9
    del csrc, cdst

    # The dominant kernel of the step is the fine-grained predictor.  It is bound by plain vector-ALU
    # work: every one of the N*L*L approximate scores has to be looked at once at least (the int8
    # contraction that produces them is a small part of its time), so `achieved` counts one lane
    # operation per score against the chip's 32-bit lane rate; the int8 rate is given beside it.
    dom = stages["C4f"]
    scores_per_launch = float(cf.N) * cf.L * cf.L
    achieved_alu = scores_per_launch / (dom["predict_ms"] * 1e-3) / 1e12
    roofline = dict(kernel="predict_stream<32, 1, 128> (fine-grained dsa_predict_mask at C4: a1 + b)", bound="alu",
                    achieved=achieved_alu, peak=ALU_PEAK_LANE_OPS / 1e12, unit="Tlane-op/s",
                    frac=achieved_alu / (ALU_PEAK_LANE_OPS / 1e12),
                    traffic=profiled_traffic_bytes("predict_stream<32, 1, 128>"),
                    traffic_source="profiles/bench_C4_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not measured in this run)",
                    valu_busy=profiled_ratio("vector ALU busy", "predict_stream<32, 1, 128>"),
                    mfma_busy=profiled_ratio("matrix-core busy", "predict_stream<32, 1, 128>"),
                    busy_source="profiles/bench_C4_pmc_counters.md (share of the launch in which the vector ALUs / the matrix cores issue; not measured in this run)",
                    algorithmic_ops=scores_per_launch, algorithmic_unit="score inspections (N*L*L), one lane operation each",
                    avg_launch_ms=dom["predict_ms"], int8_TOPS=dom["predict_int8_TOPS"],
                    frac_int8=dom["predict_frac_int8"], share_of_step=dom["predict_ms"] / ms_per_step)
    # The fine-grained attention kernel gathers K / V rows that live in L2: its roof is the rate at which the
    # memory hierarchy serves that access pattern, measured here with the gather-only twin of the kernel.
    sink = torch.empty(cf.N * cf.L * 64, dtype=torch.int32, device="cuda")
    gathered = pkg.binding.dsa_gather_roof(sh_f, K, V, passes[0]["idx"], sink)
    gather_ms = timed(lambda: pkg.binding.dsa_gather_roof(sh_f, K, V, passes[0]["idx"], sink), reps)
    roof_GBs = gathered / (gather_ms * 1e-3) / 1e9
    kv_GBs = gathered / (dom["attention_ms"] * 1e-3) / 1e9
    roofline_attention = dict(kernel="attention_rows<bf16, 64, fused> (fine-grained SDDMM+softmax+SpMM at C4: c1-c3)",
                              bound="l2-gather", achieved=kv_GBs, peak=roof_GBs, unit="GB/s", frac=kv_GBs / roof_GBs,
                              peak_source="dsa_gather_roof timed in this run: same launch shape and 16-byte gathers, no arithmetic",
                              gathered_kv_bytes=gathered, gather_probe_ms=gather_ms, avg_launch_ms=dom["attention_ms"],
                              algorithmic_bytes=gather_bytes(cf), compulsory_bytes=compulsory_bytes(cf),
                              compulsory_GBs=dom["attention_compulsory_GBs"],
                              frac_hbm_compulsory=dom["attention_compulsory_GBs"] / HBM_PEAK_GBS,
                              traffic=profiled_traffic_bytes("attention_rows<unsigned short, 64, 0>"),
                              device_copy_GBs=copy_GBs)
    del sink

    all_configs = None
    if not args.no_all_configs:
        all_configs = {}
        for name in ("C1", "C2", "C3", "C5"):
            cfg = di.CONFIGS[name]
            y = di.make_inputs(cfg)
            if cfg.dtype == "bf16":
                q, kk, v = (torch.from_numpy(y.storage(t).view(np.int16)).cuda().view(torch.bfloat16) for t in "QKV")
            else:
                q, kk, v = (torch.from_numpy(y.storage(t)).cuda() for t in "QKV")
            qt, kt = torch.from_numpy(y.Qt).cuda(), torch.from_numpy(y.Kt).cuda()
            shc = pkg.make_shape(cfg.B, cfg.H, cfg.L, cfg.d, cfg.k, cfg.keep, cfg.vec,
                                 pkg.DSA_F32 if cfg.dtype == "f32" else pkg.DSA_BF16, float(cfg.scale))
            o = torch.empty((cfg.B, cfg.H, cfg.L, cfg.d), dtype=torch.float32, device="cuda")
            ix = torch.empty((cfg.B, cfg.H, cfg.L // cfg.vec, cfg.keep), dtype=torch.int32, device="cuda")
            wsc = pkg.binding.alloc_workspace(shc)
            pkg.dsa_attention_fwd(shc, q, kk, v, qt, kt, O=o, idx_out=ix, ws=wsc)
            st = stage_times(cfg, shc, q, kk, v, qt, kt, o, ix, wsc)
            all_configs[name] = st
            del q, kk, v, qt, kt, o, ix, wsc

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import dsa_oracle
        heads = cf.N
        sl = slice(0, heads)
        Qf, Kf, Vf = (a.reshape(cf.N, cf.L, cf.d)[sl] for a in (x.Q, x.K, x.V))
        Qtf, Ktf = (a.reshape(cf.N, cf.L, cf.k)[sl] for a in (x.Qt, x.Kt))
        dsa_oracle.predict_mask(Qtf[:1, :64], Ktf[:1, :64], 4, 1)   # load the library outside the timing
        t0 = time.perf_counter()
        for cfg in (cf, cv):
            dsa_oracle.attention_fwd(Qf, Kf, Vf, Qtf, Ktf, cfg.keep, cfg.scale, cfg.vec)
        t_cpu = time.perf_counter() - t0
        cpu_baseline = dict(value=2 * heads / t_cpu, unit="heads*seqs/s", cores=dsa_oracle.num_threads(),
                            kind="oracle", seconds=t_cpu,
                            sample=f"all {heads} heads*seqs of the same tensors, one fine-grained pass then one "
                                   f"vector-wise pass (= one step), plain C oracle with OpenMP over units")

    out = dict(metric="DSA attn fwd heads*seqs/sec at L=4096, keep 5%", value=value, unit="heads*seqs/s",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="bf16",
               data="synthetic",
               config=dict(workload="C4 long-sequence DSA: B=2 H=8 L=4096 d=64 bf16, k=32 int8, keep 205 (5%), "
                                    "one fine-grained pass + one vector-wise 8x1 pass per step",
                           storage="Q,K,V bf16; Q~,K~ int8; idx int32; O fp32",
                           arithmetic="int8 x int8 -> int32 approximate scores (exact); bf16 products with fp32 "
                                      "accumulation for q.k and p.v (softmax weights rounded to bf16 for p.v); "
                                      "softmax statistics in fp32",
                           heads_seqs_per_step=heads_seqs, seed=cf.seed),
               roofline=roofline, roofline_attention=roofline_attention, cpu_baseline=cpu_baseline, stages=stages, contraction=contraction,
               all_configs=all_configs,
               low_precision_predict=dict(what="dsa_predict_mask_bits / dsa_attention_fwd_bits at C4 fine-grained",
                                          **low_precision),
               project_quantize=dict(what="Q~ and K~ from Q, K and R on the GPU (dsa_project_quantize twice), C4",
                                     ms=project_ms),
               host_cores=len(os.sched_getaffinity(0)), device=torch.cuda.get_device_name(0))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
