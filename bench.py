"""Benchmark of the whole per-layer quantisation pass (all seven entry points, a1 .. a9) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C3] [--no-cpu-baseline] [--also C2,C4,C5]

A step is one complete pass over one synthetic layer: Hessian accumulation over all calibration
tokens, damped inverse + Cholesky factor, salience, SBA, SQC + GPTQ sweep, packing.  Inputs (W, X)
are resident in HBM before the timed region.  Prints ONE JSON line.

The default workload is the target of the build: the LLaMA-7B down_proj shaped layer (4096 x 11008, 128 x 2048
calibration tokens, 2 bits on average).  The other full-size configurations are timed briefly afterwards and
reported beside the metric under `other_configs` (a few steps each, no per-kernel figures).
"""
from __future__ import annotations

import argparse
import concurrent.futures
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2405_14917_amd import binding, pipeline, synth

PEAK = {"mfma_f16": 2.5e15, "mfma_f64": 78.6e12, "alu_f64": 78.6e12, "hbm": 8.0e12}
# HBM bytes per launch of the dominant kernel function, from two `rocprofv3 --pmc` runs of this command (FETCH_SIZE,
# then WRITE_SIZE, in KiB per dispatch), each scaled by what the same counter reads for the 64 MiB copy that this
# program issues for that purpose; the files under profiles/ that are named here give the commands and the readings.
# Keyed by (config, kernel function), in bytes per pass; the line reports them per launch, like `achieved`.  A
# configuration without such a run reports null.
TRAFFIC_BYTES = {
    # profiles/gram_C3_hbm_traffic.md, per PASS (the launches of a pass together): FETCH_SIZE 3.973e7 KiB x 2.0 (the
    # yardstick's 65536 KiB read as 32778), WRITE_SIZE 5.566e5 KiB x 1.0 (its 65536 KiB written read as 65536)
    ("C3", "gram_kernel_ring<false>"): 2.0 * 3.973e7 * 1024 + 1.0 * 5.566e5 * 1024,
}
SHAPE_NAMES = {"C1": "tiny layer", "C2": "LLaMA-7B q_proj shaped layer", "C3": "LLaMA-7B down_proj shaped layer",
               "C4": "LLaMA-13B up_proj shaped layer", "C5": "LLaMA-70B-shaped MLP layer"}
T_SBA = 2048
INV_GRP = 8          # diagonal blocks of 64 columns per group of the factorisation (csrc/inverse.hip)


def resident_inputs(cfg):
    """W and X of `cfg` as device tensors (X assembled chunk by chunk from the seeded generator)."""
    W = torch.from_numpy(synth.make_weights(cfg)).cuda()
    X = torch.empty((cfg.m, cfg.t), dtype=torch.float16, device="cuda")
    nchunks = synth.n_chunks(cfg)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 8)) as pool:
        for c, xc in enumerate(pool.map(lambda i: synth.activation_chunk(cfg, i), range(nchunks))):
            t0 = c * synth.CHUNK_TOKENS
            X[:, t0:t0 + xc.shape[1]] = torch.from_numpy(xc).cuda()
    return W, X


class Pass(pipeline.LayerPass):
    """The hot path over one resident layer of a benchmark configuration; all buffers are allocated once, outside
    the timed region (the order of the entry points and the two-stream overlap are the package's LayerPass)."""

    def __init__(self, cfg, W, X, shared):
        # `shared` = (context, second stream, second context): one pair of contexts for every configuration of the
        # run, both working in caller memory sized by slim_workspace_query (no entry point allocates)
        slim, side, slim_sba = shared
        super().__init__(slim, cfg.m, cfg.beta, cfg.N, cfg.percdamp, T_SBA, second=(side, slim_sba))
        self.cfg, self.W, self.X = cfg, W, X

    def step(self):
        r = self.run(self.W, self.X)
        self.stored = (r["packed"], r["gbits"], r["row_off"], r["scale"], r["zero"])
        return r["p_star"], r["m_star"]      # 0-dim device tensors: reading them is the caller's synchronisation

    def phases(self, reps=2):
        """Not part of the step: the same pass with the host waiting between its phases, so that each phase's own
        duration can be read (the timed pass runs them back to back and overlaps nothing across these borders except
        the host's enqueueing).  Returns milliseconds per phase, averaged over `reps` passes."""
        s, s2, W, X = self.slim, self.slim_sba, self.W, self.X
        Xs = X[:, : min(self.t_sba, X.shape[1])]
        acc = {}

        def lap(name, t0):
            torch.cuda.synchronize()
            acc[name] = acc.get(name, 0.0) + (time.perf_counter() - t0) * 1e3
            return time.perf_counter()

        for _ in range(reps):
            self.G.zero_()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            nt = s.hessian_accumulate(X, self.G, 0)
            t0 = lap("hessian", t0)
            self.side.wait_stream(self.main)
            s2.sba_prepare(W, self.beta, self.N, Xs)
            s.hessian_inverse(self.G, nt, self.percdamp, U=self.U, hinv_diag=self.d)
            t0 = lap("inverse_with_sba_outputs_beside", t0)
            _, grp, _ = s.salience(W, self.d, self.beta)
            t0 = lap("salience", t0)
            with torch.cuda.stream(self.side):
                bits, _, _ = s2.sba_allocate(W, grp, self.beta, self.N, Xs, host_outputs=False)
            t0 = lap("sba_rank_and_search", t0)
            out = s.gptq_quantize(W, self.U, bits, self.beta)
            t0 = lap("sqc_and_gptq_sweep", t0)
            s.pack(out["codes"], bits, self.beta, packed_rows=self.m * (self.N + 1) // 32, host_outputs=False,
                   bit_base=self.bit_base)
            t0 = lap("pack", t0)
        return {k: v / reps for k, v in acc.items()}

    def inference(self, tokens=1, reps=100):
        """Not part of the step: the linear layer on the stored form of the last pass (App. B.2), `tokens`
        activations at a time; returns microseconds per call and the bytes of the stored form it streams."""
        packed, gbits, row_off, scale, zero = self.stored
        x = self.X[:, :tokens].t().contiguous()
        y = torch.empty((tokens, self.cfg.n), dtype=torch.float32, device="cuda")
        for _ in range(5):
            self.slim.dequant_matmul(packed, gbits, row_off, scale, zero, self.cfg.beta, x, Y=y)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            self.slim.dequant_matmul(packed, gbits, row_off, scale, zero, self.cfg.beta, x, Y=y)
        e1.record()
        torch.cuda.synchronize()
        m_star = int(row_off[-1])                     # packed holds the rows of its capacity; the layer fills m_star
        nbytes = m_star * packed.shape[1] * 4 + gbits.numel() * 4 + row_off.numel() * 4 + scale.numel() * 8 + zero.numel() * 8
        return e0.elapsed_time(e1) * 1e3 / reps, nbytes

def algorithmic_work(name, cfg, launches_per_step):
    """(bound, peak key, work per launch) for every step of the path.  Work is ALGORITHMIC: distinct results
    only (the Gram matrix is credited with its triangle), bytes that have to move at least once.  `bound` is the
    roof that binds the step: "mfma" (flops), "alu" (flops of plain vector arithmetic), "hbm" (bytes), or
    "latency" for the serial chain of diagonal blocks, which is rated as microseconds per link x links."""
    n, m, t, beta = cfg.n, cfg.m, cfg.t, cfg.beta
    k = m // beta
    ts = min(T_SBA, t)
    L = max(launches_per_step, 1)
    if name.startswith("gram_mfma"):
        return "mfma", "mfma_f16", float(m) * (m + 1) * t / L
    if name == "sba_output_dgemm":
        # two products per step (reference outputs, outputs of the all-N-bit weights), in one launch or several
        return "mfma", "mfma_f64", 2.0 * (2.0 * n * m * ts) / L
    if name == "sba_update_dgemm":
        return "mfma", "mfma_f64", 4.0 * n * beta * ts
    if name == "sba_search":
        # the k/2 rank-2beta updates of the search, in one kernel
        return "mfma", "mfma_f64", (k // 2) * 4.0 * n * beta * ts / L
    if name == "gptq_trailing_dgemm":
        # rank-512 update of the columns behind each window of 512 columns
        tot = sum(2.0 * n * (min(m, w0 + 512) - w0) * (m - min(m, w0 + 512)) for w0 in range(0, m, 512))
        return "mfma", "mfma_f64", tot / L
    if name == "gptq_window_dgemm":
        sb = min(beta, 128)
        tot = sum(2.0 * n * sb * (min(m, (b0 // 512) * 512 + 512) - b0 - sb) for b0 in range(0, m, sb))
        return "mfma", "mfma_f64", tot / L
    if name.startswith("inv_") and name.endswith("_dgemm"):
        # The factorisation and the triangular inverse together are (2/3) m^3 flops; the launch sites share them
        # as follows (each formula counts what that site's products compute, triangles once).
        w = INV_GRP * 64
        groups = [(g0, min(m, g0 + w)) for g0 in range(0, m, w)]
        if name == "inv_trtri_dgemm":          # inside the groups, beyond the diagonal blocks' own inverses
            tot = sum(((g1 - g0) ** 3 - (g1 - g0) * 64.0 ** 2) / 3.0 for g0, g1 in groups)
        elif name == "inv_trtri_rows_dgemm":   # U[g, S] = -U[g, g] T[g, S], U[g, g] triangular
            tot = sum(float(g1 - g0) ** 2 * (m - g1) for g0, g1 in groups)
        elif name == "inv_trtri_terms_dgemm":  # T[0:g0, g0:m] (+)= R[0:g0, g] U[g, g0:m], U[g, g] triangular
            tot = sum(float(g0) * (g1 - g0) ** 2 + 2.0 * g0 * (g1 - g0) * (m - g1) for g0, g1 in groups)
        elif name == "inv_panel_dgemm":
            tot = sum(2.0 * j0 * 64 * 64 / 2 for j0 in range(64, m, 64))
        elif name == "inv_window_dgemm":
            tot = sum(2.0 * (j0 - 64) * (j0 - ((j0 // 64 - 1) // INV_GRP) * INV_GRP * 64) * min(64, m - j0)
                      for j0 in range(128, m, 64))
        elif name == "inv_group_next_dgemm":
            w = INV_GRP * 64
            tot = sum(2.0 * g0 * w * (min(m, g0 + w) - g0 - 64) for g0 in range(w, m, w) if min(m, g0 + w) - g0 > 64)
        elif name == "inv_syrk_dgemm":
            w = INV_GRP * 64
            tot = sum(float(g0 - w) * (g0 - w + 1) * (min(m, g0 + w) - g0) for g0 in range(2 * w, m, w))
        else:
            tot = 0.0
        return "mfma", "mfma_f64", tot / L
    if name == "inv_chol_diag":
        return "latency", None, 0.0                                   # m / 64 dependent diagonal blocks
    if name == "sqc_search":
        return "alu", "alu_f64", 9.0 * cfg.ncand * n * beta          # ~9 fp64 operations per weight and candidate
    if name == "gptq_sweep":
        return "alu", "alu_f64", float(n) * beta * beta              # rank-1 updates inside the group
    hbm = {
        "sba_kl_step": 2.0 * 8 * n * ts,                 # one pass over P and the candidate's outputs
        "salience_colsumsq": 2.0 * n * m,                # W once (16-bit)
        "pack_codes": n * m * (1.0 + cfg.N / 8.0),       # codes in, words out
        "gram_reduce": 10.0 * m * m,                     # G read and written (4 B each), one partial per upper tile in
        "inv_widen": 10.0 * m * m,                       # upper half of G in (4 B), upper A and lower U out (8 B each)
        "inv_diag_colsumsq": 4.0 * m * m,                # upper triangle of U (8 B) once
        "gptq_widen": 10.0 * n * m / L,                  # W (16-bit) in, fp64 working copy out
        "sba_widen_w": 10.0 * n * m,
        "sba_widen_x": 10.0 * m * ts,
        "sba_fakequant": 16.0 * n * m,                   # fp64 weights in, fake-quantised fp64 weights out
        "sba_gather_x": 16.0 * (k // 2) * 2 * beta * ts,
        "sba_kl_ref": 4.0 * 8 * n * ts / L,              # the reference outputs: read twice, written once, read once
        "sqc_block_stats": 8.0 * n * beta,
    }
    if name in hbm:
        return "hbm", "hbm", hbm[name]
    return "hbm", "hbm", 0.0


def cpu_baseline(cfg):
    """The oracle as it stands, timed on this host on a bounded sample of the same layer (about 20 s of host work)
    and scaled to the full layer by each stage's own size dependence."""
    from oracle import slim_oracle as orc
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    # sample sizes: rows of W, tokens for the Gram matrix, leading block of G for the inverse (cubic scaling)
    n_s = min(cfg.n, 2048 if cfg.m <= 4096 else (512 if cfg.m <= 8192 else 256))
    t_gram = min(cfg.t, (4 if cfg.m <= 4096 else 1) * synth.CHUNK_TOKENS)
    m_inv = min(cfg.m, 4096)
    W = synth.make_weights(cfg)[:n_s].astype(np.float64)
    X0 = np.concatenate([synth.activation_chunk(cfg, c) for c in range(t_gram // synth.CHUNK_TOKENS or 1)], axis=1)
    tm = {}
    t0 = time.perf_counter()
    G = np.zeros((cfg.m, cfg.m))
    orc.gram_accumulate(G, X0[:, :t_gram])
    tm["gram"] = (time.perf_counter() - t0) * (cfg.t / t_gram)
    t0 = time.perf_counter()
    orc.hessian_inverse(G[:m_inv, :m_inv], t_gram, cfg.percdamp)
    tm["inverse"] = (time.perf_counter() - t0) * (cfg.m / m_inv) ** 3
    # second-order information for the later stages: exact for the sampled leading block, a damped diagonal beyond
    # it (the later stages' cost does not depend on the values)
    if m_inv < cfg.m:
        Hd = 2.0 / t_gram * np.diag(G) + cfg.percdamp * 2.0 / t_gram * np.mean(np.diag(G))
        U, d = np.diag(Hd ** -0.5), 1.0 / Hd
    else:
        U, d, _ = orc.hessian_inverse(G, t_gram, cfg.percdamp)
    rows = cfg.n / n_s
    t0 = time.perf_counter()
    _, grp, _ = orc.salience(W, d, cfg.beta)
    tm["salience"] = (time.perf_counter() - t0) * rows
    t0 = time.perf_counter()
    bits, _, _, _ = orc.sba_allocate(W, grp, cfg.beta, cfg.N, X0[:, : min(T_SBA, cfg.t)].astype(np.float64))
    tm["sba"] = (time.perf_counter() - t0) * rows
    t0 = time.perf_counter()
    out = orc.gptq_quantize(W, U, bits, cfg.beta, orc.tau_grid())
    tm["gptq"] = (time.perf_counter() - t0) * rows
    t0 = time.perf_counter()
    orc.pack_fast(out["codes"], bits, cfg.beta)
    tm["pack"] = (time.perf_counter() - t0) * rows
    total = sum(tm.values())
    return {
        "value": cfg.n * cfg.m / total, "unit": "weights/s", "cores": cores, "kind": "oracle",
        "sample": "Gram on %d of %d tokens (x%.0f), inverse of the leading %d x %d block (x%.1f, cubic), "
                  "salience/SBA/SQC+GPTQ/pack on %d of %d rows (x%.0f); scaled seconds per stage: %s" % (
                      t_gram, cfg.t, cfg.t / t_gram, m_inv, m_inv, (cfg.m / m_inv) ** 3, n_s, cfg.n, rows,
                      ", ".join("%s %.1f" % kv for kv in tm.items())),
    }


def workload_text(cfg):
    return ("%s: %s W %dx%d %s, X %dx%d f16 (%d calibration tokens), group %d, %d-bit average, 1%% damping, "
            "%d SQC candidates, SBA objective on %d tokens" % (
                cfg.name, SHAPE_NAMES.get(cfg.name, "layer"), cfg.n, cfg.m, cfg.w_dtype, cfg.m, cfg.t, cfg.t, cfg.beta,
                cfg.N, cfg.ncand, min(T_SBA, cfg.t)))


def timed_steps(job, steps, warmup):
    for _ in range(warmup):
        job.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        p_star, m_star = job.step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, int(p_star), int(m_star)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C3", choices=sorted(synth.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=2)
    ap.add_argument("--no-shared-input", action="store_true", help="skip the three-layer figure beside the metric")
    ap.add_argument("--also", default="C2,C4,C5",
                    help="other configurations to time briefly beside the metric (comma separated, '' for none)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the pass is a single-GPU job); run with --gpus 1")

    cfg = synth.CONFIGS[args.config]
    also_cfgs = [c for c in args.also.split(",") if c and c != cfg.name]
    for name in also_cfgs:
        if name not in synth.CONFIGS:
            sys.exit("bench.py: unknown configuration %r in --also" % name)
    # one pair of contexts (and streams) for all configurations, each with a workspace for the largest of them
    run_cfgs = [cfg] + [synth.CONFIGS[c] for c in also_cfgs]
    ws_main = max(binding.workspace_query(c.n, c.m, c.beta, c.t, min(T_SBA, c.t), 1) for c in run_cfgs)
    ws_sba = max(binding.workspace_query(c.n, c.m, c.beta, 0, min(T_SBA, c.t)) for c in run_cfgs)
    slim = binding.Slim("cuda:0", ws_main)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        slim_sba = binding.Slim("cuda:0", ws_sba)
    shared = (slim, side, slim_sba)
    W, X = resident_inputs(cfg)
    job = Pass(cfg, W, X, shared)

    # A plain streaming kernel of known size (64 MiB read, 64 MiB written: the negation of 32 Mi fp16 values, the only
    # launch of torch's neg kernel in this program): the yardstick that the HBM traffic counters of a
    # rocprofv3 --pmc run of this command are scaled by.
    calib_src = torch.ones(32 << 20, dtype=torch.float16, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    torch.neg(calib_src, out=calib_dst)
    del calib_src, calib_dst

    ms_per_step, p_star, m_star = timed_steps(job, args.steps, args.warmup)

    # per-kernel durations with HIP events on the library's stream, in extra steps of the same job
    for c in job.contexts():
        c.profile_enable(True)
        c.profile_reset()
    for _ in range(args.profile_steps):
        job.step()
    prof = {}
    for c in job.contexts():
        for full, (ms, cnt) in c.profile_collect().items():
            a = prof.get(full, (0.0, 0))
            prof[full] = (a[0] + ms, a[1] + cnt)
        c.profile_enable(False)
    # A profiling entry is named "<step>" or "<step>@<kernel function>" (launch sites that choose among several
    # kernel functions say which one ran), with "#side" appended for launches on the library's side streams.
    # `kernels` is keyed by step.  The roofline is given for the kernel FUNCTION with the largest share of the GPU
    # time among ALL functions (side streams and the persistent reserved forms included), under the name rocprofv3
    # lists it by, so that its average duration can be compared with the rocprofv3 summary of the same command.
    kernels, functions = {}, {}
    for full, (ms, cnt) in prof.items():
        full, _, side = full.partition("#")
        step, _, fn = full.partition("@")
        k = kernels.setdefault(step, {"ms": 0.0, "cnt": 0, "parts": []})
        k["ms"] += ms
        k["cnt"] += cnt
        k["parts"].append(((fn or step) + ("#side" if side else ""), ms, cnt))
    for step, k in kernels.items():
        k["ms_per_step"] = k["ms"] / args.profile_steps
        k["launches_per_step"] = k["cnt"] / args.profile_steps
        k["avg_us"] = 1e3 * k["ms"] / k["cnt"]
        bound, peak_key, work = algorithmic_work(step, cfg, k["launches_per_step"])
        k["bound"], k["peak_key"], k["work_per_step"] = bound, peak_key, work * k["launches_per_step"]
        for fn, ms, cnt in k["parts"]:
            f = functions.setdefault(fn, {"ms": 0.0, "cnt": 0, "work": 0.0, "bound": bound, "peak_key": peak_key})
            f["ms"] += ms
            f["cnt"] += cnt
            # a step that ran on several kernel functions is credited to them in proportion to their time
            f["work"] += k["work_per_step"] * args.profile_steps * (ms / k["ms"] if k["ms"] > 0 else 0.0)
    roofline = None
    if functions:
        dom = max(functions, key=lambda fn: functions[fn]["ms"])
        f = functions[dom]
        if f["bound"] == "latency":
            roofline = {"kernel": dom, "bound": "latency", "achieved": None, "peak": None, "unit": "us per link",
                        "frac": None, "traffic": None, "avg_us": 1e3 * f["ms"] / f["cnt"],
                        "launches_per_step": f["cnt"] / args.profile_steps, "ms_per_step": f["ms"] / args.profile_steps}
        else:
            achieved = f["work"] / (f["ms"] * 1e-3)
            unit = {"mfma": "TFLOP/s", "alu": "TFLOP/s", "hbm": "GB/s"}[f["bound"]]
            div = 1e9 if f["bound"] == "hbm" else 1e12
            roofline = {"kernel": dom.partition("#")[0], "bound": f["bound"], "achieved": achieved / div,
                        "peak": PEAK[f["peak_key"]] / div, "unit": unit, "frac": achieved / PEAK[f["peak_key"]],
                        "traffic": (TRAFFIC_BYTES[(cfg.name, dom.partition("#")[0])] / (f["cnt"] / args.profile_steps)
                                    if (cfg.name, dom.partition("#")[0]) in TRAFFIC_BYTES else None),
                        "avg_us": 1e3 * f["ms"] / f["cnt"], "launches_per_step": f["cnt"] / args.profile_steps,
                        "ms_per_step": f["ms"] / args.profile_steps}
    # every step of the path for the record: time, the roof that binds it, the fraction of that roof, and the time
    # the step would take at the roof (its floor).  The chain of diagonal blocks is rated by its latency.
    others, floor_ms = {}, 0.0
    for name, k in kernels.items():
        entry = {"ms_per_step": round(k["ms_per_step"], 4), "launches_per_step": k["launches_per_step"],
                 "bound": k["bound"]}
        if k["bound"] == "latency":
            entry["latency"] = {"us_per_link": round(k["avg_us"], 2), "links": k["launches_per_step"]}
        elif k["work_per_step"] > 0:
            floor = k["work_per_step"] / PEAK[k["peak_key"]] * 1e3
            floor_ms += floor
            entry["floor_ms"] = round(floor, 4)
            entry["frac"] = round(floor / k["ms_per_step"], 4)
        others[name] = entry
    whole_pass = {"sum_of_floors_ms": floor_ms, "frac": floor_ms / ms_per_step,
                  "note": "sum over the steps of (algorithmic work / peak of the roof that binds the step) against "
                          "the measured ms_per_step; the alu entries count an FMA as two operations"}

    line = {
        "metric": "weights_quantized_per_s", "value": cfg.n * cfg.m / (ms_per_step * 1e-3), "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 x f16 -> f32 (Gram MFMA), f64 (inverse, salience, SBA, SQC, GPTQ sweep), u8/u32 (pack)",
        "data": "synthetic",
        "config": {"workload": workload_text(cfg), "p_star": p_star, "m_star": m_star},
        "roofline": roofline,
        "whole_pass": whole_pass,
        "kernels": others,
        "kernel_notes": {
            "sqc_search": "alu peak counts an FMA as two operations; the search loop is mostly single-operation "
                          "instructions (multiply, round, two clamps), so its fraction of the issue bound is about "
                          "twice the frac given",
            "inv_syrk_dgemm, inv_panel_dgemm, inv_window_dgemm, inv_trtri_*_dgemm, sba_output_dgemm": "run beside other "
                          "streams' work by design (the factorisation's chains, its far updates and the triangular "
                          "inverse on four streams, beside the SBA outputs on part of the chip): their durations "
                          "overlap and their frac is not a fraction of the chip",
            "hbm entries": "yardsticks on the same chip (plain PyTorch kernels, 1 to 4 GB): fill 6.9 TB/s, copy 4.9 to 5.3 TB/s "
                           "read plus written (0.61 to 0.66 of the peak), read-only sum 4.0 TB/s, fp16 -> fp64 conversion 3.2 TB/s",
            "gram_mfma_f16": "power-limited: the same kernel runs at 0.71 of the nominal peak on constant data and at "
                             "0.49 to 0.51 on random data when Gram launches follow one another",
        },
    }
    # beside the metric: the phases of a pass with the host waiting between them, and what the fp64 phase
    # (inverse with the two SBA output products beside it) achieves as a whole
    ph = job.phases()
    ts = min(T_SBA, cfg.t)
    fp64_flops = (2.0 / 3.0) * float(cfg.m) ** 3 + 2.0 * (2.0 * cfg.n * cfg.m * ts)
    line["phases_ms"] = {k: round(v, 3) for k, v in ph.items()}
    line["phases_ms"]["note"] = ("one pass with the host waiting at the borders of the phases (extra passes after the timed "
                                 "region); inverse_with_sba_outputs_beside: (2/3) m^3 + 4 n m t_s fp64 flops = %.3g, i.e. "
                                 "%.2f of the fp64 matrix peak over the phase" % (
                                     fp64_flops, fp64_flops / (ph["inverse_with_sba_outputs_beside"] * 1e-3) / PEAK["mfma_f64"]))
    # beside the metric: the inference kernel of the stored form (next step of the path, not part of `value`)
    us, nbytes = job.inference(tokens=1)
    line["inference"] = {"kernel": "dequant_matmul", "tokens": 1, "us_per_call": us, "stored_bytes": nbytes,
                         "GB_per_s": nbytes / us / 1e3, "frac_hbm": nbytes / (us * 1e-6) / PEAK["hbm"]}
    # beside the metric too: three layers that read the same input (q/k/v of a block) with one Hessian and one
    # inverse between them; the three layers are this layer's weights three times, the result per layer is the
    # step's own
    if not args.no_shared_input:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        shared_reps = 2
        for _ in range(shared_reps):
            job.run_shared_input([W, W, W], X)
        torch.cuda.synchronize()
        line["shared_input"] = {"layers": 3, "ms_per_layer": (time.perf_counter() - t0) * 1e3 / (3 * shared_reps),
                                "note": "one Gram matrix and one inverse for three layers of the step's shape"}
    job.close()
    del job, W, X
    torch.cuda.empty_cache()
    # the other full-size configurations, a few steps each
    other_cfgs = {}
    for name in also_cfgs:
        oc = synth.CONFIGS[name]
        Wo, Xo = resident_inputs(oc)
        ojob = Pass(oc, Wo, Xo, shared)
        ms, ps, mst = timed_steps(ojob, 10, 5)
        other_cfgs[name] = {"workload": workload_text(oc), "ms_per_step": ms, "value": oc.n * oc.m / (ms * 1e-3),
                            "unit": "weights/s", "steps": 10, "warmup": 5, "p_star": ps, "m_star": mst}
        ojob.close()
        del ojob, Wo, Xo
        torch.cuda.empty_cache()
    line["other_configs"] = other_cfgs
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg)
    else:
        line["cpu_baseline"] = None
    slim_sba.close()
    slim.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
