#!/usr/bin/env python3
"""Benchmark of the factorized hot path on one MI355X.

One *step* is one pass of the factorized multiplies over the operator micro-benchmark schema
(star join, S 1,000,000 x 20, R 100,000 x 200, uniform keys, float32, seed 1):

    T X (cx = 1 and 16) and T^T Y (cx = 1 and 16),

through the C ABI, with every input already resident in HBM.  Three copies of the source tables (and their
plans, built outside the timed region) take turns from step to step, so that the tables come from HBM and not
from the 256 MB last-level cache.  `value` is the step's algorithmic bytes (what each operator must read or
write once: the `bytes_*` functions below) divided by the step's wall time; the same steps on one warm copy
are reported beside it.  The JSON line also carries gradient-descent iterations/s factorized vs materialized
(Alg. 1), the Gram matrix and the join-gather baseline on their own, the per-kernel breakdown, the roofline
entry of the step's dominant kernel (timed with HIP events inside the timed region) and the CPU oracle timed
on a bounded sample of the same step.  `--only <operator>` runs one operator alone for a profiler.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
FP32_MFMA_PEAK = 157.3e12
BF16_MFMA_PEAK = 2.5e15


# ----------------------------------------------------------------------------- byte model
def _is_identity(s):
    """NULL row_idx, or the identity on the first r_k target rows and -1 beyond (what the plan detects)."""
    if s.row_idx is None:
        return True
    idx = s.row_idx
    return (s.rows <= idx.size and np.array_equal(idx[:s.rows], np.arange(s.rows, dtype=idx.dtype))
            and bool(np.all(idx[s.rows:] == -1)))


def shapes_of(schema):
    """(rows, cols, needs an inverse index) per source."""
    return [(s.rows, s.cols, not _is_identity(s)) for s in schema.sources]


def bytes_tables(shapes):
    return 4 * sum(r * c for r, c, _ in shapes)


def bytes_lmm(shapes, r_T, c_T, c):
    ni = [(r, k) for r, k, has in shapes if has]
    return bytes_tables(shapes) + 4 * r_T * len(ni) + 8 * c * sum(r for r, _ in ni) + 4 * r_T * c + 4 * c_T * c


def bytes_tmm(shapes, r_T, c_T, c):
    ni = [(r, k) for r, k, has in shapes if has]
    return (bytes_tables(shapes) + 4 * r_T * c + sum(4 * r_T + 4 * (r + 1) + 8 * c * r for r, _ in ni)
            + 4 * c_T * c)


def bytes_gd(shapes, r_T, c_T):
    ident = sum(r * c for r, c, has in shapes if not has)
    ni = [(r, c) for r, c, has in shapes if has]
    return (4 * ident + 8 * sum(r * c for r, c in ni) + 4 * r_T * (2 * len(ni) + 3)
            + 16 * sum(r for r, _ in ni) + 8 * c_T)


def bytes_gd_clustered(shapes, r_T, c_T):
    """One model's iteration over a two-table star join whose entity table and labels are kept in join order: both
    tables once, the key and the label of every row, weights in and out."""
    return bytes_tables(shapes) + 8 * r_T + 8 * c_T


def bytes_gd_rows_joined(schema):
    """One model's iteration that fetches every source's row per target row and uses it twice (stacked tables):
    every reached table row once, row indices, labels, weights in and out."""
    b = 0
    for s in schema.sources:
        reached = s.rows if _is_identity(s) else int(np.count_nonzero(s.row_idx >= 0))
        b += 4 * reached * s.cols + (0 if _is_identity(s) else 4 * schema.r_T)
    return b + 4 * schema.r_T + 8 * schema.c_T


def bytes_materialize(shapes, r_T, c_T):
    ni = sum(1 for _, _, has in shapes if has)
    return bytes_tables(shapes) + 4 * r_T * ni + 4 * r_T * c_T


def bytes_crossprod(shapes, r_T, c_T):
    ni = [(r, c) for r, c, has in shapes if has]
    return bytes_tables(shapes) + sum(4 * r_T + 4 * (r + 1) for r, _ in ni) + 4 * c_T * c_T


def complexity_ratio_lr(shapes, r_T, c_T):
    """Eq. (1) for linear regression with dense operands (Sec. 3.1): O_materialized / O_factorized."""
    m_T = r_T * c_T
    o_mat = 1 * m_T + r_T * c_T + m_T + c_T * r_T
    o_fact = sum(1 * r * c + r * c_T for r, c, _ in shapes) + sum(r * c + c * r_T for r, c, _ in shapes)
    return o_mat / o_fact


# ----------------------------------------------------------------------------- helpers
def time_loop(torch, fn, reps, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def graph_time(torch, fn, iters, replays=10):
    """Seconds per call of `fn` when `iters` calls are captured in a HIP graph and the graph is replayed."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(iters):
            fn()
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (replays * iters)


STEP_OPS = ("lmm_c1", "tmm_c1", "lmm_c16", "tmm_c16")     # the step: T X and T^T Y, one and sixteen operand columns
OTHER_OPS = ("gd_step", "crossprod", "materialize")          # timed on their own, outside `value`
CLUSTERED_OP = "gd_clustered"    # gd_step on plans that keep the entity table in join order (ilargi_plan_cluster)
CLUSTERED_GATHER_OP = "gd_clustered_gathered_labels"   # ... without the labels in the copy (--only, for the profiler)


class Workload:
    """Operands of the operator micro-benchmark and `copies` independent copies of the source tables with
    their plans.  The copies take turns (3 x 168 MB on the config-1 centre schema against a 256 MB last-level
    cache), so that no launch finds its tables cached from the previous one; copy 0 alone is the warm case."""

    def __init__(self, il, torch, sch, srcs, dev, copies=3):
        self.il, self.torch, self.sch = il, torch, sch
        r_T, c_T = sch.r_T, sch.c_T
        self.shp = shapes_of(sch)
        self.tables = [srcs] + [[(D.clone(), None if idx is None else idx.clone(), cm) for D, idx, cm in srcs]
                                for _ in range(copies - 1)]
        self.plans = [il.ilargi_plan_create(t, r_T, c_T, max_cx=16) for t in self.tables]
        self.X = {c: dev(sch.extras[f"X{c}"]) for c in (1, 16)}
        self.Y = {c: dev(sch.extras[f"Y{c}"]) for c in (1, 16)}
        self.out_l = {c: torch.empty((r_T, c), device="cuda") for c in (1, 16)}
        self.out_t = {c: torch.empty((c_T, c), device="cuda") for c in (1, 16)}
        self.G = torch.empty((c_T, c_T), device="cuda")
        self.Tm = None                      # allocated on first use (880 MB)
        self.W = torch.zeros((c_T, 1), device="cuda")
        self.lr = torch.full((1,), 0.1, device="cuda")
        self.loss = torch.zeros(1, device="cuda")
        # labels for the regression: y = T w* + noise, the product taken on the device
        rng = np.random.Generator(np.random.PCG64(101))
        w_star = dev(rng.standard_normal((c_T, 1)).astype(np.float32))
        self.y = (il.ilargi_lmm(self.plans[0], w_star).reshape(-1) + 0.01 * torch.randn(r_T, device="cuda")).contiguous()
        self.nbytes = {"lmm_c1": bytes_lmm(self.shp, r_T, c_T, 1), "tmm_c1": bytes_tmm(self.shp, r_T, c_T, 1),
                       "lmm_c16": bytes_lmm(self.shp, r_T, c_T, 16), "tmm_c16": bytes_tmm(self.shp, r_T, c_T, 16),
                       "gd_step": bytes_gd(self.shp, r_T, c_T), CLUSTERED_OP: bytes_gd_clustered(self.shp, r_T, c_T),
                       CLUSTERED_GATHER_OP: bytes_gd_clustered(self.shp, r_T, c_T) + 4 * r_T,
                       "crossprod": bytes_crossprod(self.shp, r_T, c_T),
                       "materialize": bytes_materialize(self.shp, r_T, c_T)}

    def call(self, name, plan):
        il = self.il
        if name.startswith("lmm_c"):
            c = int(name[5:])
            return il.ilargi_lmm(plan, self.X[c], self.out_l[c])
        if name.startswith("tmm_c"):
            c = int(name[5:])
            return il.ilargi_tmm(plan, self.Y[c], self.out_t[c])
        if name in ("gd_step", CLUSTERED_OP, CLUSTERED_GATHER_OP):
            return il.ilargi_gd_step(plan, il.LINEAR, self.W, self.y, self.lr, self.loss)
        if name == "crossprod":
            return il.ilargi_crossprod(plan, self.G)
        if name == "materialize":
            if self.Tm is None:
                self.Tm = self.torch.empty((self.sch.r_T, self.sch.c_T), device="cuda")
            return il.ilargi_materialize(plan, self.Tm)
        raise KeyError(name)

    def cluster(self, on, labels=True):
        """Every copy of the tables gets (or drops) the join-ordered copy of its entity table."""
        for plan in self.plans:
            if on:
                self.il.ilargi_plan_cluster(plan, y=self.y if labels else None)
            else:
                self.il.ilargi_plan_cluster(plan, None)
        self.torch.cuda.synchronize()

    def step(self, i, rotate=True, label=False):
        """One step: the four multiplies on copy i of the tables (copy 0 when not rotating)."""
        plan = self.plans[i % len(self.plans)] if rotate else self.plans[0]
        for name in STEP_OPS:
            if label:
                self.il.ilargi_plan_trace_label(plan, name)
            self.call(name, plan)

    def time_op(self, name, rotate, reps=30, batches=5):
        """Median over `batches` of the mean time of `reps` launches between two events on the launch stream."""
        torch = self.torch
        n = len(self.plans)
        for i in range(n):
            self.call(name, self.plans[i if rotate else 0])
        torch.cuda.synchronize()
        ts = []
        for _ in range(batches):
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                self.call(name, self.plans[i % n if rotate else 0])
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3 / reps)
        return float(np.median(ts))

    def op_record(self, name, t):
        b = self.nbytes[name]
        return {"us": round(t * 1e6, 1), "GBps": round(b / t / 1e9, 1), "hbm_frac": round(b / t / 1e9 / HBM_PEAK_GBPS, 4),
                "MB": round(b / 1e6, 1)}


def cpu_baseline(sch, sample_rows, budget_s=20.0):
    """The oracle, as it stands, on the first `sample_rows` target rows of the same step (the four multiplies,
    which it computes on the joined table it builds first)."""
    import datagen
    import oracle
    srcs = []
    for s in sch.sources:
        if s.row_idx is None:
            srcs.append(datagen.Source(s.D[:sample_rows], None, s.col_map))
        else:
            srcs.append(datagen.Source(s.D, s.row_idx[:sample_rows], s.col_map))
    sub = datagen.Schema(srcs, sample_rows, sch.c_T)
    shp = shapes_of(sub)
    nbytes = (bytes_lmm(shp, sub.r_T, sub.c_T, 1) + bytes_tmm(shp, sub.r_T, sub.c_T, 1)
              + bytes_lmm(shp, sub.r_T, sub.c_T, 16) + bytes_tmm(shp, sub.r_T, sub.c_T, 16))
    reps, t_total = 0, 0.0
    while t_total < budget_s and reps < 100:
        t0 = time.perf_counter()
        tg = oracle.Target(sub)                                        # materialize (join-gather)
        oracle.lmm(tg, sch.extras["X1"]); oracle.tmm(tg, sch.extras["Y1"][:sample_rows])
        oracle.lmm(tg, sch.extras["X16"]); oracle.tmm(tg, sch.extras["Y16"][:sample_rows])
        t_total += time.perf_counter() - t0
        reps += 1
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = 1
    cores = min(len(os.sched_getaffinity(0)), blas_threads) if blas_threads else len(os.sched_getaffinity(0))
    return {
        "value": round(nbytes * reps / t_total / 1e9, 3), "unit": "GB/s", "cores": int(cores),
        "kind": "oracle",
        "sample": f"first {sample_rows} of {sch.r_T} target rows, same step (join, then T X and T^T Y with 1 and 16 "
                  f"operand columns), {reps} repetition(s), {t_total:.1f} s; the byte count is the factorized step's "
                  f"on the sample; host has {len(os.sched_getaffinity(0))} usable cores, BLAS threads {blas_threads}",
        "ms_per_step_scaled_to_full": round(t_total / reps * 1e3 * sch.r_T / sample_rows, 1),
    }


def run_sweep(il, torch, datagen, dev, path, records=None):
    """Factorized vs materialized over the tuple-ratio / feature-ratio grid of the micro-benchmark."""
    rows = []
    for r_R, c_R in datagen.CONFIG1_GRID:
        sch = datagen.config1(r_R=r_R, c_R=c_R)
        shp = shapes_of(sch)
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=16)
        Tm = il.ilargi_materialize(plan)
        mplan = il.ilargi_plan_create([(Tm, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=16)
        rec = {"r_R": r_R, "c_R": c_R, "TR": sch.r_T / r_R, "FR": c_R / 20,
               "complexity_ratio": round(complexity_ratio_lr(shp, sch.r_T, sch.c_T), 3)}
        rec["materialize_us"] = round(time_loop(torch, lambda: il.ilargi_materialize(plan, Tm), 5) * 1e6, 1)
        for c in (1, 16):
            X, Y = dev(sch.extras[f"X{c}"]), dev(sch.extras[f"Y{c}"])
            o1 = torch.empty((sch.r_T, c), device="cuda"); o2 = torch.empty((sch.c_T, c), device="cuda")
            for name, fn_f, fn_m, b in (
                ("lmm", lambda: il.ilargi_lmm(plan, X, o1), lambda: il.ilargi_lmm(mplan, X, o1), bytes_lmm(shp, sch.r_T, sch.c_T, c)),
                ("tmm", lambda: il.ilargi_tmm(plan, Y, o2), lambda: il.ilargi_tmm(mplan, Y, o2), bytes_tmm(shp, sch.r_T, sch.c_T, c)),
            ):
                tf, tm = time_loop(torch, fn_f, 20), time_loop(torch, fn_m, 20)
                rec[f"{name}_c{c}"] = {"fact_us": round(tf * 1e6, 1), "mat_us": round(tm * 1e6, 1),
                                       "speedup": round(tm / tf, 3), "fact_GBps": round(b / tf / 1e9, 1)}
        W = torch.zeros((sch.c_T, 1), device="cuda")
        y = torch.randn(sch.r_T, device="cuda")
        lr = torch.full((1,), 0.1, device="cuda")
        loss = torch.zeros(1, device="cuda")
        tf = time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss), 20)
        tm = time_loop(torch, lambda: il.ilargi_gd_step(mplan, il.LINEAR, W, y, lr, loss), 20)
        rec["gd"] = {"fact_us": round(tf * 1e6, 1), "mat_us": round(tm * 1e6, 1), "speedup": round(tm / tf, 3)}
        # the same iteration with the entity table (and the labels) kept in join order, where the one-pass kernel
        # takes the tables (dimension tables of at most 256 columns)
        try:
            il.ilargi_plan_cluster(plan, y=y)
            tc = time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss), 20)
            rec["gd"].update({"clustered_us": round(tc * 1e6, 1), "clustered_speedup": round(tm / tc, 3)})
            il.ilargi_plan_cluster(plan, None)
        except il.IlargiError:
            pass
        rec["chooser"] = chooser_record(il, f"config1 r_R={r_R} c_R={c_R}", shp, sch.r_T, sch.c_T, tf, tm,
                                        rec["materialize_us"] * 1e-6)
        if records is not None:
            records.append(rec["chooser"])
        rows.append(rec)
        print(json.dumps(rec), file=sys.stderr, flush=True)
        del plan, mplan, Tm
        torch.cuda.empty_cache()
    with open(path, "w") as f:
        json.dump(rows, f, indent=1)
    if records is not None:
        held_out_schemas(il, torch, datagen, records)


HELD_OUT = [   # (name, r_S, c_S, [(r_R, c_R, keys), ...]): shapes that played no part in setting the byte model's constants
    ("held-out S 2000000x8 + R 20000x64", 2_000_000, 8, [(20_000, 64, "uniform")]),
    ("held-out S 500000x40 + R 250000x40", 500_000, 40, [(250_000, 40, "uniform")]),
    ("held-out S 3000000x4 + R 3000x16 + R 300000x32", 3_000_000, 4, [(3_000, 16, "uniform"), (300_000, 32, "uniform")]),
    ("held-out S 1000000x64 + R 100000x16", 1_000_000, 64, [(100_000, 16, "uniform")]),
    ("held-out S 4000000x12 + R 1000000x24", 4_000_000, 12, [(1_000_000, 24, "uniform")]),
    ("held-out S 800000x16 + R 8000x512 (Zipf keys)", 800_000, 16, [(8_000, 512, ("zipf", 1.1))]),
]


def held_out_schemas(il, torch, datagen, records):
    """More validation points for ilargi_choose: 200-iteration trainings on schemas outside the benchmark's grid."""
    for name, r_S, c_S, dims in HELD_OUT:
        sch = datagen.star_schema(datagen.rng_for(900 + len(records)), r_S, c_S, dims)
        shp = shapes_of(sch)
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
        T = il.ilargi_materialize(plan)
        t_join = time_loop(torch, lambda: il.ilargi_materialize(plan, T), 3, warm=1)
        mplan = il.ilargi_plan_create([(T, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=1)
        W = torch.zeros((sch.c_T, 1), device="cuda")
        y = torch.randn(sch.r_T, device="cuda")
        lr = torch.full((1,), 0.01, device="cuda")
        loss = torch.zeros(1, device="cuda")
        t_f = time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss), 20)
        t_m = time_loop(torch, lambda: il.ilargi_gd_step(mplan, il.LINEAR, W, y, lr, loss), 20)
        records.append(chooser_record(il, name, shp, sch.r_T, sch.c_T, t_f, t_m, t_join))
        print(json.dumps(records[-1]), file=sys.stderr, flush=True)
        del plan, mplan, T
        torch.cuda.empty_cache()


def kernel_model(shp, r_T, c_T):
    """Algorithmic bytes (and, where the matrix cores bound the kernel, flops) of one launch of each traced
    kernel on a two-table star join [S | I_R R], keyed by trace name "<operator>/<kernel family>[:source]".
    Every term is a buffer the kernel has to read or write once; gathered rows count once per use."""
    (r_S, c_S, _), (r_R, c_R, _) = shp[0], shp[1]
    m = {}
    for c in (1, 16):
        w = 4 * c
        seg = 4 * r_T + w * r_T + 4 * (r_R + 1) + w * r_R        # perm, Y rows, rowptr, Z_R written
        m[f"lmm_c{c}/lmm_rows:1"] = ("hbm", 4 * r_R * c_R + w * r_R + w * c_R)               # R once, P_R written, X_R
        m[f"lmm_c{c}/lmm_assemble"] = ("hbm", 4 * r_S * c_S + 4 * r_T + 2 * w * r_T + w * c_S)  # S once, fk, P rows, out
        m[f"tmm_c{c}/segsum:1"] = ("hbm", seg)
        m[f"tmm_c{c}/colred:0"] = ("hbm", 4 * r_S * c_S + w * r_T)                             # S once, Y
        m[f"tmm_c{c}/colred:1"] = ("hbm", 4 * r_R * c_R + w * r_R)                             # R once, Z_R
        m[f"tmm_c{c}/colred+segsum:0"] = ("hbm", 4 * r_S * c_S + w * r_T + seg)                # both of the above
        # join-order pass over R: R once, perm, rowptr, the joined rows of Y; Z_R is never written
        m[f"tmm_c{c}/tmm_join:1"] = ("hbm", 4 * r_R * c_R + 4 * r_T + 4 * (r_R + 1) + w * r_T)
        # ... sharing its launch with the column reduce of S
        m[f"tmm_c{c}/colred+join:0"] = ("hbm", 4 * r_S * c_S + w * r_T + m[f"tmm_c{c}/tmm_join:1"][1])
    m["gd_step/lmm_rows:1"] = m["lmm_c1/lmm_rows:1"]
    m["gd_step/lmm_assemble"] = ("hbm", 4 * r_S * c_S + 4 * r_T * 4 + 4 * c_S)                 # S once, fk, P, y, E written
    m["gd_step/segsum:1"] = m["tmm_c1/segsum:1"]
    m["gd_step/colred:1"] = m["tmm_c1/colred:1"]
    m["gd_step/tmm_join:1"] = m["tmm_c1/tmm_join:1"]
    # the clustered iteration: S (join-ordered copy) and R once, key and label of every row
    m["gd_clustered/gd_cluster"] = ("hbm", 4 * r_S * c_S + 4 * r_R * c_R + 8 * r_T)
    # ... with the labels gathered through the index (target row and label instead of the label alone)
    m["gd_clustered_gathered_labels/gd_cluster"] = ("hbm", 4 * r_S * c_S + 4 * r_R * c_R + 12 * r_T)
    m["materialize/materialize"] = ("hbm", bytes_materialize(shp, r_T, c_T))
    # Gram matrix: S^T S and the rows of S summed per row of R in one join-order pass; the cross block
    # Zc^T R; the diagonal block R^T diag(cnt) R (upper-triangle 16 x 16 tiles on the matrix cores)
    m["crossprod/gram_star"] = ("hbm", 4 * r_S * c_S + 4 * r_T + 4 * (r_R + 1) + 4 * r_R * c_S)
    m["crossprod/gram:1"] = ("hbm", 4 * r_R * (c_S + c_R))
    tiles = ((c_R + 15) // 16) * ((c_R + 15) // 16 + 1) // 2
    m["crossprod/gram:3"] = ("mfma", 4 * r_R * c_R + 4 * (r_R + 1), tiles * 2 * 256 * r_R)
    return m


def scalar_ops(il, torch, plan, mplan, sch):
    """Tab. 2, first four rows, on the same schema: element-wise operators, rowSum and colSum, factorized
    (on the source tables) vs the same entry points on the materialized table.  Bytes: an element-wise
    operator reads and writes every cell it touches once; rowSum is the left multiply by ones; colSum
    reads the tables once (the fan-out vectors are part of the plan)."""
    shp = shapes_of(sch)
    cells_f = sum(r * c for r, c, _ in shp)
    cells_m = sch.r_T * sch.c_T
    outs_f = [torch.empty_like(D) for D, _ in plan._borrowed]
    outs_m = [torch.empty_like(D) for D, _ in mplan._borrowed]
    rs = torch.empty(sch.r_T, device="cuda")
    cs = torch.empty(sch.c_T, device="cuda")
    out = {}
    cases = (("mul", lambda pl, o: il.ilargi_elementwise(pl, "mul", 1.5, outs=o), 8 * cells_f, 8 * cells_m),
             ("exp", lambda pl, o: il.ilargi_elementwise(pl, "exp", 0.0, outs=o), 8 * cells_f, 8 * cells_m),
             ("row_sum", lambda pl, o: il.ilargi_row_sum(pl, rs), bytes_lmm(shp, sch.r_T, sch.c_T, 1),
              4 * cells_m + 4 * sch.r_T + 4 * sch.c_T),
             ("col_sum", lambda pl, o: il.ilargi_col_sum(pl, cs), 4 * cells_f + 4 * sum(r for r, _, _ in shp) + 4 * sch.c_T,
              4 * cells_m + 4 * sch.r_T + 4 * sch.c_T))
    for name, fn, b_f, b_m in cases:
        t_f = time_loop(torch, lambda: fn(plan, outs_f), 20)
        t_m = time_loop(torch, lambda: fn(mplan, outs_m), 10)
        out[name] = {"factorized_us": round(t_f * 1e6, 1), "materialized_us": round(t_m * 1e6, 1),
                     "speedup": round(t_m / t_f, 2), "factorized_GBps": round(b_f / t_f / 1e9, 1),
                     "materialized_GBps": round(b_m / t_m / 1e9, 1)}
    out["cells"] = {"factorized": int(cells_f), "materialized": int(cells_m), "ratio_tab2": round(cells_m / cells_f, 2)}
    return out


def unsupervised(il, torch, plan, mplan, sch, k=10):
    """KMeans (one Lloyd iteration, k centroids) and Gaussian NMF (one round of multiplicative updates, rank k) on
    the same schema, factorized vs the same entry points on the materialized table, with the factorized
    iteration's kernels listed.  Timing only: the factors start from random positive values."""
    g = torch.Generator(device="cuda").manual_seed(7)
    C0 = torch.randn((sch.c_T, k), device="cuda", generator=g)
    W0 = torch.rand((sch.r_T, k), device="cuda", generator=g) + 0.05
    H0 = torch.rand((sch.c_T, k), device="cuda", generator=g) + 0.05
    assign = torch.empty(sch.r_T, dtype=torch.int32, device="cuda")
    counts = torch.empty(k, dtype=torch.int32, device="cuda")
    out = {"k": k}

    def kmeans(pl):
        C = C0.clone()
        return lambda: il.ilargi_kmeans_step(pl, C, assign, counts)

    def gnmf(pl):
        W, Ht = W0.clone(), H0.clone()
        return lambda: il.ilargi_gnmf_step(pl, W, Ht)

    for name, make in (("kmeans", kmeans), ("gnmf", gnmf)):
        t_f = time_loop(torch, make(plan), 20)
        t_m = time_loop(torch, make(mplan), 10)
        fn = make(plan)
        fn()
        il.ilargi_plan_trace_begin(plan, "*", 64)
        fn()
        ms, names = il.ilargi_plan_trace_end(plan, 64, names=True)
        out[name] = {"factorized_it_per_s": round(1.0 / t_f, 1), "materialized_it_per_s": round(1.0 / t_m, 1),
                     "factorized_us": round(t_f * 1e6, 1), "materialized_us": round(t_m * 1e6, 1),
                     "speedup": round(t_m / t_f, 2),
                     "kernels_us": {f"{i}:{n}": round(float(v) * 1e3, 1) for i, (n, v) in enumerate(zip(names, ms))}}
    return out


def sparse_tables(il, torch, datagen, dev):
    """Source tables kept in compressed sparse rows (Sec. 3.1; sparsity sweep of Tab. 3) on the config-1 centre
    schema with a fraction p of the cells set to zero: one gradient-descent iteration and the one-column
    multiplies, tables sparse vs the same tables dense (zeros stored)."""
    out = {}
    base = datagen.config1()
    for p in (0.5, 0.9, 0.99):
        sch = datagen.sparsify(base, p, seed=11)
        rec = {}
        for kind in ("dense", "sparse"):
            srcs = il.schema_to_device(sch, sparse=(kind == "sparse"))
            plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
            W = torch.zeros((sch.c_T, 1), device="cuda")
            y = torch.randn(sch.r_T, device="cuda")
            lr = torch.full((1,), 0.1, device="cuda")
            loss = torch.zeros(1, device="cuda")
            X = torch.randn(sch.c_T, 1, device="cuda"); Y = torch.randn(sch.r_T, 1, device="cuda")
            o1 = torch.empty(sch.r_T, 1, device="cuda"); o2 = torch.empty(sch.c_T, 1, device="cuda")
            rec[kind] = {"gd_us": round(time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss), 20) * 1e6, 1),
                         "lmm_c1_us": round(time_loop(torch, lambda: il.ilargi_lmm(plan, X, o1), 20) * 1e6, 1),
                         "tmm_c1_us": round(time_loop(torch, lambda: il.ilargi_tmm(plan, Y, o2), 20) * 1e6, 1)}
            if kind == "sparse":
                rec["stored_entries"] = int(sum(D.nnz for D, _, _ in srcs))
            del plan, srcs
            torch.cuda.empty_cache()
        rec["gd_speedup_sparse_over_dense"] = round(rec["dense"]["gd_us"] / rec["sparse"]["gd_us"], 2)
        out[f"p={p}"] = rec
    return out


def wide_setup(il, torch, datagen, dev):
    sch = datagen.config4()
    m = 256
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=m)
    W = torch.zeros((sch.c_T, m), device="cuda")
    y = torch.randn(sch.r_T, device="cuda")
    lr = dev(sch.extras["lr"].astype(np.float32))
    loss = torch.zeros(m, device="cuda")
    return sch, m, plan, W, y, lr, loss


def wide_only(il, torch, datagen, dev, which, reps):
    """The 256-model gradient-descent iteration alone (float32 or bfloat16 inputs), for a profiler run."""
    sch, m, plan, W, y, lr, loss = wide_setup(il, torch, datagen, dev)
    prec = il.F32 if which == "wide_f32" else il.BF16_IN_F32_ACC
    t = time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss, precision=prec), reps)
    il.ilargi_plan_trace_begin(plan, "*", 64)
    il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss, precision=prec)
    ms, names = il.ilargi_plan_trace_end(plan, 64, names=True)
    print(json.dumps({"only": which, "launches": reps + 3, "ms_per_iteration": round(t * 1e3, 3),
                      "kernels_us": {f"{i}:{n}": round(float(v) * 1e3, 1) for i, (n, v) in enumerate(zip(names, ms))}}),
          flush=True)
    return 0


def wide_batch(il, torch, datagen, dev, mfma_file):
    """The batched hyper-parameter workload (256 linear regressions at once on the same schema, seed 4):
    gradient-descent iterations/s and matrix-core utilisation, float32 and bfloat16 inputs, factorized vs
    materialized.  Flops are the algorithmic ones of Alg. 1: 2 products x 2 m (sum_k r_k c_k).  `mfma_frac` is
    algorithmic flops / time / peak; `mfma_busy_measured` is the matrix cores' busy share of each large kernel's
    cycles from the committed counter summary (rocprofv3 --pmc), when that file is present."""
    sch, m, plan, W, y, lr, loss = wide_setup(il, torch, datagen, dev)
    T = il.ilargi_materialize(plan)
    mplan = il.ilargi_plan_create([(T, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=m)
    fl_fact = 4 * m * sum(s.rows * s.cols for s in sch.sources)
    fl_mat = 4 * m * sch.r_T * sch.c_T
    peaks = {"f32": FP32_MFMA_PEAK, "bf16": BF16_MFMA_PEAK}
    out = {}
    for prec, pn in ((il.F32, "f32"), (il.BF16_IN_F32_ACC, "bf16")):
        for nm, pl, fl in (("factorized", plan, fl_fact), ("materialized", mplan, fl_mat)):
            W.zero_()
            t = time_loop(torch, lambda: il.ilargi_gd_step(pl, il.LINEAR, W, y, lr, loss, precision=prec), 10)
            rec = {"gd_it_per_s": round(1.0 / t, 1), "ms_per_iteration": round(t * 1e3, 3),
                   "TFLOPs": round(fl / t / 1e12, 2), "mfma_frac": round(fl / t / peaks[pn], 4)}
            if nm == "factorized":
                il.ilargi_plan_trace_begin(pl, "*", 64)
                il.ilargi_gd_step(pl, il.LINEAR, W, y, lr, loss, precision=prec)
                ms, names = il.ilargi_plan_trace_end(pl, 64, names=True)
                rec["kernels_us"] = {f"{i}:{n}": round(float(v) * 1e3, 1) for i, (n, v) in enumerate(zip(names, ms))}
            out[f"{pn}_{nm}"] = rec
    # the same iterations on a plan that keeps the entity table and the labels in join order: the fused pass streams
    # the copy instead of gathering rows of S (same sums, same order, same bits)
    il.ilargi_plan_cluster(plan, y=y)
    for prec, pn in ((il.F32, "f32"), (il.BF16_IN_F32_ACC, "bf16")):
        W.zero_()
        t = time_loop(torch, lambda: il.ilargi_gd_step(plan, il.LINEAR, W, y, lr, loss, precision=prec), 10)
        out[f"{pn}_factorized_clustered"] = {"gd_it_per_s": round(1.0 / t, 1), "ms_per_iteration": round(t * 1e3, 3),
                                             "TFLOPs": round(fl_fact / t / 1e12, 2),
                                             "mfma_frac": round(fl_fact / t / peaks[pn], 4)}
    il.ilargi_plan_cluster(plan, None)
    out["bf16_over_f32_factorized"] = round(out["f32_factorized"]["ms_per_iteration"] / out["bf16_factorized"]["ms_per_iteration"], 3)
    busy = {}
    for key in ("wide_f32/lmm_rows:1", "wide_f32/star_pass", "wide_f32/colred:1",
                "wide_bf16/lmm_rows:1", "wide_bf16/star_pass", "wide_bf16/colred:1"):
        v = read_profile_value(mfma_file, key, "mfma_busy_frac")
        if v is not None:
            busy[key] = v
    out["mfma_busy_measured"] = busy or None
    out["flops_per_iteration"] = {"factorized": fl_fact, "materialized": fl_mat}
    out["note"] = ("m = 256 models; the factorized step walks the target rows in join order and never stores the "
                   "r_T x m residual (R W_R, one fused pass, R^T Z, update); the materialized step writes the "
                   "1 GB residual and reads it back for T^T E")
    return out


CHOOSER_ITERATIONS = 200   # the paper's training length (Sec. 4.1)


def chooser_record(il, name, shp, r_T, c_T, t_fact, t_mat, t_join):
    """One validation point of ilargi_choose: measured winner of a 200-iteration training (join included for
    the materialized strategy) against the byte-model decision, Eq. (1) > 1 and the tuple/feature-ratio rule."""
    c = il.ilargi_choose([(r, k, has) for r, k, has in shp], r_T, c_T, iterations=CHOOSER_ITERATIONS)
    total_f = CHOOSER_ITERATIONS * t_fact
    total_m = t_join + CHOOSER_ITERATIONS * t_mat
    return {"schema": name, "measured_factorize": int(total_f <= total_m), "measured_speedup": round(total_m / total_f, 3),
            "byte_model": int(c["factorize"]), "predicted_speedup": round(c["seconds_materialized"] / c["seconds_factorized"], 3),
            "eq1_ratio": round(c["complexity_ratio"], 3), "eq1_rule": int(c["complexity_ratio"] > 1.0),
            "tuple_ratio": round(c["tuple_ratio"], 2), "feature_ratio": round(c["feature_ratio"], 2),
            "tr_fr_rule": int(c["morpheus_rule"])}


def chooser_summary(records):
    n = len(records)
    if n == 0:
        return None
    acc = {rule: round(sum(int(r[rule] == r["measured_factorize"]) for r in records) / n, 3)
           for rule in ("byte_model", "eq1_rule", "tr_fr_rule")}
    return {"iterations": CHOOSER_ITERATIONS, "points": n, "accuracy": acc, "records": records}


def other_configs(il, torch, datagen, records=None):
    """Gradient-descent iterations/s, factorized vs materialized, on the remaining single-model
    configurations (full size): 0 (tiny star join, linear), 2 (three dimensions with a Zipf key, logistic),
    3 (union with overlap, linear)."""
    out = {}
    for name, model, mname in (("config0", il.LINEAR, "linear"), ("config2", il.LOGISTIC, "logistic"),
                               ("config3", il.LINEAR, "linear")):
        sch = getattr(datagen, name)()
        shp = shapes_of(sch)
        srcs = il.schema_to_device(sch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
        torch.cuda.synchronize()
        plan_ms = (time.perf_counter() - t0) * 1e3
        T = il.ilargi_materialize(plan)
        t_mat_once = time_loop(torch, lambda: il.ilargi_materialize(plan, T), 3, warm=1)
        mplan = il.ilargi_plan_create([(T, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=1)
        W = torch.zeros((sch.c_T, 1), device="cuda")
        y = (torch.rand(sch.r_T, device="cuda") > 0.5).float()
        lr = torch.full((1,), 0.1, device="cuda")
        loss = torch.zeros(1, device="cuda")
        t_f = time_loop(torch, lambda: il.ilargi_gd_step(plan, model, W, y, lr, loss), 20)
        t_m = time_loop(torch, lambda: il.ilargi_gd_step(mplan, model, W, y, lr, loss), 20)
        eager = None
        if t_f < 30e-6:
            # iterations this short are bound by the host's launch rate when enqueued one by one from Python: time
            # them as a captured graph of 50 iterations, replayed
            eager = {"gd_factorized_it_per_s": round(1.0 / t_f, 1), "gd_materialized_it_per_s": round(1.0 / t_m, 1)}
            t_f = graph_time(torch, lambda: il.ilargi_gd_step(plan, model, W, y, lr, loss), 50)
            t_m = graph_time(torch, lambda: il.ilargi_gd_step(mplan, model, W, y, lr, loss), 50)
        il.ilargi_plan_trace_begin(plan, "*", 64)
        il.ilargi_gd_step(plan, model, W, y, lr, loss)
        _, launched = il.ilargi_plan_trace_end(plan, 64, names=True)
        joined = any(k.startswith("gd_rowjoin") for k in launched)
        b = bytes_gd_rows_joined(sch) if joined else bytes_gd(shp, sch.r_T, sch.c_T)
        out[name] = {"model": mname, "launches": launched, "gd_factorized_MB": round(b / 1e6, 1), "r_T": sch.r_T, "c_T": sch.c_T, "sources": len(sch.sources),
                     "gd_factorized_it_per_s": round(1.0 / t_f, 1), "gd_materialized_it_per_s": round(1.0 / t_m, 1),
                     "speedup": round(t_m / t_f, 3), "gd_factorized_GBps": round(b / t_f / 1e9, 1),
                     "materialize_once_us": round(t_mat_once * 1e6, 1), "plan_build_ms": round(plan_ms, 1),
                     "complexity_ratio_eq1": round(complexity_ratio_lr(shp, sch.r_T, sch.c_T), 3)}
        if name == "config3":
            # the Gram matrix this configuration asks for, factorized vs on the joined table
            G = torch.empty((sch.c_T, sch.c_T), device="cuda")
            t_cf = time_loop(torch, lambda: il.ilargi_crossprod(plan, G), 10)
            t_cm = time_loop(torch, lambda: il.ilargi_crossprod(mplan, G), 10)
            out[name]["crossprod_us"] = round(t_cf * 1e6, 1)
            out[name]["crossprod_materialized_us"] = round(t_cm * 1e6, 1)
            out[name]["crossprod_MB"] = round(4 * sum(r * c for r, c, _ in shp) / 1e6, 1)
            out[name]["crossprod_GFLOP"] = round(2.0 * sch.r_T * sch.c_T * sch.c_T / 1e9, 2)
        if eager is not None:
            out[name]["timed_as"] = "captured graph of 50 iterations (GPU time); enqueued one by one from Python: " + json.dumps(eager)
        if records is not None:
            records.append(chooser_record(il, name, shp, sch.r_T, sch.c_T, t_f, t_m, t_mat_once))
        del plan, mplan, T, W, y
        torch.cuda.empty_cache()
    return out


def stream_probe(il, torch):
    """What plain streaming kernels reach on this device (1 GiB buffers)."""
    n = 1 << 28
    src = torch.empty(n, device="cuda").normal_()
    dst = torch.empty(n, device="cuda")
    in_order = n // 1024                 # one float4 per thread, workgroups dispatched in address order
    sink = torch.empty(in_order, device="cuda")
    res = {}
    for kind, name, factor in ((1, "read", 1), (2, "write", 1), (0, "copy", 2), (4, "write_nontemporal", 1),
                               (3, "copy_nontemporal", 2)):
        d = sink if kind == 1 else dst
        t = time_loop(torch, lambda: il.ilargi_stream_probe(kind, d, src, n, 8192), 10)
        res[f"{name}_GBps"] = round(factor * n * 4 / t / 1e9, 1)
        if kind in (0, 1, 2):
            t = time_loop(torch, lambda: il.ilargi_stream_probe(kind, d, src, n, in_order), 10)
            res[f"{name}_in_order_GBps"] = round(factor * n * 4 / t / 1e9, 1)
    res["note"] = ("8192 workgroups with a grid stride, except *_in_order: one float4 per thread, workgroups "
                   "dispatched in address order")
    return res


def read_profile_value(path, key, field):
    """A number from a committed profiler summary: the line that starts with '<key> ' and holds '<field>: <N>'."""
    try:
        for line in open(path):
            if line.startswith(key + " ") and field + ":" in line:
                return float(line.split(field + ":")[1].split()[0])
    except OSError:
        pass
    return None


def trace_all(il, plans, max_launches):
    for pl in plans:
        il.ilargi_plan_trace_begin(pl, "*", max_launches)


def trace_collect(il, plans, max_launches):
    """{trace name: [ms, ...]} over the given plans."""
    per = {}
    for pl in plans:
        ms, names = il.ilargi_plan_trace_end(pl, max_launches, names=True)
        for nm, v in zip(names, ms):
            per.setdefault(nm, []).append(float(v))
    return per


def run_only(il, torch, wl, name, reps):
    """One operator alone, `reps` launches on the rotating tables, after a plain 1 GiB copy that gives a profiler
    run the scale of its byte counters.  Prints the kernels of one call in launch order and exits."""
    n = 1 << 28
    src = torch.empty(n, device="cuda").normal_()
    dst = torch.empty(n, device="cuda")
    il.ilargi_stream_probe(0, dst, src, n, n // 1024)
    torch.cuda.synchronize()
    del src, dst
    if name == CLUSTERED_OP:
        wl.cluster(True)
    if name == CLUSTERED_GATHER_OP:
        wl.cluster(True, labels=False)
    for i in range(3):
        wl.call(name, wl.plans[i % len(wl.plans)])
    torch.cuda.synchronize()
    il.ilargi_plan_trace_begin(wl.plans[0], "*", 64)
    il.ilargi_plan_trace_label(wl.plans[0], name)
    wl.call(name, wl.plans[0])
    torch.cuda.synchronize()
    ms, names = il.ilargi_plan_trace_end(wl.plans[0], 64, names=True)
    t = wl.time_op(name, rotate=True, reps=reps, batches=1)
    print(json.dumps({"only": name, "launches": reps + len(wl.plans) + 4, "us": round(t * 1e6, 1),
                      "kernels_us": {f"{i}:{nm}": round(float(v) * 1e3, 1) for i, (nm, v) in enumerate(zip(names, ms))}}),
          flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cpu-sample-rows", type=int, default=100_000)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-wide", action="store_true", help="skip the 256-model batched workload")
    ap.add_argument("--no-configs", action="store_true", help="skip the other single-model configurations")
    ap.add_argument("--no-extras", action="store_true", help="skip the scalar operators, KMeans / NMF and sparse tables")
    ap.add_argument("--only", default="", help="run one operator alone (for a profiler): " + ", ".join(STEP_OPS + OTHER_OPS + (CLUSTERED_OP, CLUSTERED_GATHER_OP))
                    + ", wide_f32, wide_bf16")
    ap.add_argument("--sweep", default="", help="also run the TR/FR sweep and write it to this JSON file")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "traffic_by_operator_and_kernel.txt"))
    ap.add_argument("--mfma-file", default=os.path.join(ROOT, "profiles", "wide_batch_mfma_counters.txt"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import datagen
    import paper_2502_01985_amd as il

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if args.only in ("wide_f32", "wide_bf16"):
        return wide_only(il, torch, datagen, dev, args.only, args.steps)

    sch = datagen.config1()                      # centre of the grid: R 100,000 x 200
    shp = shapes_of(sch)
    srcs = il.schema_to_device(sch)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=16)    # (the first call also loads the code object)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=16)    # tables resident: validation + inverse index
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    del plan
    wl = Workload(il, torch, sch, srcs, dev)
    if args.only:
        if args.only not in STEP_OPS + OTHER_OPS + (CLUSTERED_OP, CLUSTERED_GATHER_OP):
            print(f"bench.py: unknown operator {args.only}", file=sys.stderr)
            return 2
        return run_only(il, torch, wl, args.only, args.steps)
    step_bytes = sum(wl.nbytes[n] for n in STEP_OPS)
    ncopies = len(wl.plans)

    for i in range(args.warmup):
        wl.step(i)
    torch.cuda.synchronize()
    # discovery pass (untimed): every kernel launch of the step bracketed by HIP events, to find the dominant kernel
    n_disc = 2 * ncopies
    cap = 32 * n_disc
    trace_all(il, wl.plans, cap)
    for i in range(n_disc):
        wl.step(i, label=True)
    torch.cuda.synchronize()
    per_kernel = trace_collect(il, wl.plans, cap)
    model = kernel_model(shp, sch.r_T, sch.c_T)

    def kernel_records(per, n_steps):
        recs = {}
        for nm, v in per.items():
            avg = float(np.mean(v))
            rec = {"launches_per_step": round(len(v) / n_steps, 2), "avg_us": round(avg * 1e3, 2),
                   "us_per_step": round(sum(v) / n_steps * 1e3, 2)}
            if nm in model:
                rec["algorithmic_MB"] = round(model[nm][1] / 1e6, 2)
                rec["GBps"] = round(model[nm][1] / (avg * 1e-3) / 1e9, 1)
                rec["hbm_frac"] = round(rec["GBps"] / HBM_PEAK_GBPS, 4)
                if model[nm][0] == "mfma":
                    rec["TFLOPs"] = round(model[nm][2] / (avg * 1e-3) / 1e12, 2)
                    rec["mfma_frac"] = round(model[nm][2] / (avg * 1e-3) / FP32_MFMA_PEAK, 4)
            recs[nm] = rec
        return recs

    kernels = kernel_records(per_kernel, n_disc)
    # the dominant kernel of the factorized step: largest share of the step among the kernels with a byte model
    dom = max((k for k in kernels if k in model), key=lambda k: kernels[k]["us_per_step"])

    # the timed region: K steps, the tables rotating; the dominant kernel's launches are bracketed by HIP events
    # on the launch stream
    for pl in wl.plans:
        il.ilargi_plan_trace_begin(pl, dom, 2 * args.steps + 16)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        wl.step(i, label=True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom_ms = np.concatenate([il.ilargi_plan_trace_end(pl, 2 * args.steps + 16) for pl in wl.plans])
    ms_per_step = elapsed / args.steps * 1e3
    avg_ms = float(np.mean(dom_ms))
    ach = model[dom][1] / (avg_ms * 1e-3) / 1e9
    traffic = read_profile_value(args.traffic_file, dom, "traffic_bytes_per_launch")
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None if traffic is None else int(traffic),
                "avg_launch_us": round(avg_ms * 1e3, 2), "launches_timed": int(dom_ms.size),
                "algorithmic_bytes_per_launch": int(model[dom][1]),
                "share_of_step": round(float(np.sum(dom_ms)) / args.steps / ms_per_step, 4)}
    # the same K steps on one copy of the tables (warm: 168 MB of tables stay in the 256 MB last-level cache)
    for i in range(args.warmup):
        wl.step(0, rotate=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        wl.step(0, rotate=False)
    torch.cuda.synchronize()
    ms_per_step_warm = (time.perf_counter() - t0) / args.steps * 1e3
    # the rotating steps once more, one step per copy of the tables captured in a HIP graph and the graph replayed:
    # the same kernels without the host's share of every launch
    ncp = len(wl.plans)
    state = {"i": 0}

    def one_step():
        wl.step(state["i"], rotate=True)
        state["i"] += 1
    try:
        ms_per_step_graph = graph_time(torch, one_step, ncp, replays=max(args.steps // ncp, 1)) * 1e3
    except Exception as exc:                                        # (reported, never fatal: the headline is the eager loop)
        print(f"bench.py: graph replay of the step failed: {exc}", file=sys.stderr)
        ms_per_step_graph = None

    # per operator: tables rotating (headline) and one copy back to back (warm)
    ops_rot = {n: wl.op_record(n, wl.time_op(n, rotate=True)) for n in STEP_OPS + ("gd_step", "crossprod")}
    ops_warm = {n: wl.op_record(n, wl.time_op(n, rotate=False)) for n in STEP_OPS + OTHER_OPS}
    # kernels of the operators outside the step (one traced call each)
    trace_all(il, wl.plans[:1], 256)
    for n in OTHER_OPS:
        il.ilargi_plan_trace_label(wl.plans[0], n)
        for _ in range(3):
            wl.call(n, wl.plans[0])
    torch.cuda.synchronize()
    other_kernels = kernel_records(trace_collect(il, wl.plans[:1], 256), 3)
    # the same iteration on plans that keep the entity table in join order (84 MB more per copy of the tables)
    wl.cluster(True)
    clustered = {"tables_rotated": wl.op_record(CLUSTERED_OP, wl.time_op(CLUSTERED_OP, rotate=True)),
                 "warm_tables": wl.op_record(CLUSTERED_OP, wl.time_op(CLUSTERED_OP, rotate=False)),
                 "crossprod": wl.op_record("crossprod", wl.time_op("crossprod", rotate=True))}
    trace_all(il, wl.plans[:1], 64)
    il.ilargi_plan_trace_label(wl.plans[0], CLUSTERED_OP)
    for _ in range(3):
        wl.call(CLUSTERED_OP, wl.plans[0])
    torch.cuda.synchronize()
    other_kernels.update(kernel_records(trace_collect(il, wl.plans[:1], 64), 3))
    wl.cluster(False)

    # gradient descent: factorized vs materialized iterations/s (the materialized strategy = the join once, then
    # the same entry point on a one-source plan over T, 880 MB: larger than every cache)
    Tm = wl.Tm
    mplan = il.ilargi_plan_create([(Tm, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=16)
    Wm = torch.zeros((sch.c_T, 1), device="cuda")
    t_fact = ops_rot["gd_step"]["us"] * 1e-6
    t_fact_warm = ops_warm["gd_step"]["us"] * 1e-6
    t_mat = time_loop(torch, lambda: il.ilargi_gd_step(mplan, il.LINEAR, Wm, wl.y, wl.lr, wl.loss), 30)
    t_join = ops_warm["materialize"]["us"] * 1e-6
    mat_ops = {}
    for c in (1, 16):
        o1 = torch.empty((sch.r_T, c), device="cuda"); o2 = torch.empty((sch.c_T, c), device="cuda")
        tl = time_loop(torch, lambda: il.ilargi_lmm(mplan, wl.X[c], o1), 10)
        tt = time_loop(torch, lambda: il.ilargi_tmm(mplan, wl.Y[c], o2), 10)
        mat_ops[f"lmm_c{c}"] = {"us": round(tl * 1e6, 1), "speedup_factorized": round(tl * 1e6 / ops_rot[f"lmm_c{c}"]["us"], 2)}
        mat_ops[f"tmm_c{c}"] = {"us": round(tt * 1e6, 1), "speedup_factorized": round(tt * 1e6 / ops_rot[f"tmm_c{c}"]["us"], 2)}
    scalar = models = None
    if not args.no_extras:
        scalar = scalar_ops(il, torch, wl.plans[0], mplan, sch)
        models = unsupervised(il, torch, wl.plans[0], mplan, sch)
    del mplan

    probe = stream_probe(il, torch)
    records = []
    if args.sweep:
        run_sweep(il, torch, datagen, dev, args.sweep, records)
    else:
        records.append(chooser_record(il, "config1", shp, sch.r_T, sch.c_T, t_fact, t_mat, t_join))
    del wl, Tm
    torch.cuda.empty_cache()
    wide = sparse = None
    if not args.no_wide:
        wide = wide_batch(il, torch, datagen, dev, args.mfma_file)
        torch.cuda.empty_cache()
    if not args.no_extras:
        sparse = sparse_tables(il, torch, datagen, dev)
        torch.cuda.empty_cache()
    configs = None if args.no_configs else other_configs(il, torch, datagen, records)

    cpu = None if args.no_cpu else cpu_baseline(sch, args.cpu_sample_rows)

    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "factorized LMM+T^T.Y GB/s and % HBM peak; LR GD iters/sec vs materialized",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config1 centre: star join S 1000000x20 + R 100000x200, uniform fk, T 1000000x220; "
                               "step = factorized T X and T^T Y with 1 and 16 operand columns (4 calls), "
                               f"{ncopies} copies of the source tables taking turns from step to step",
                   "seed": 1, "tuple_ratio": 10, "feature_ratio": 10,
                   "complexity_ratio_eq1": round(complexity_ratio_lr(shp, sch.r_T, sch.c_T), 3)},
        "hbm_frac": round(value / HBM_PEAK_GBPS, 4),
        "hbm_frac_target": 0.60,
        "step_algorithmic_MB": round(step_bytes / 1e6, 1),
        "warm_tables": {"ms_per_step": round(ms_per_step_warm, 4),
                        "GBps": round(step_bytes / (ms_per_step_warm * 1e-3) / 1e9, 1),
                        "hbm_frac": round(step_bytes / (ms_per_step_warm * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                        "note": "the same steps on one copy of the tables: 168 MB that stay in the 256 MB last-level cache"},
        "step_as_captured_graph": None if ms_per_step_graph is None else {
            "ms_per_step": round(ms_per_step_graph, 4),
            "GBps": round(step_bytes / (ms_per_step_graph * 1e-3) / 1e9, 1),
            "hbm_frac": round(step_bytes / (ms_per_step_graph * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "note": "one step per copy of the tables captured in a HIP graph, the graph replayed (tables rotating as in `value`)"},
        "gd": {"factorized_it_per_s": round(1.0 / t_fact, 1), "materialized_it_per_s": round(1.0 / t_mat, 1),
               "speedup": round(t_mat / t_fact, 3),
               "factorized_it_per_s_warm_tables": round(1.0 / t_fact_warm, 1),
               "factorized_GBps": ops_rot["gd_step"]["GBps"], "factorized_hbm_frac": ops_rot["gd_step"]["hbm_frac"],
               "materialize_once_us": ops_warm["materialize"]["us"],
               "break_even_iterations": (round(t_join / (t_fact - t_mat), 1) if t_fact > t_mat else 0),
               "clustered_entity_table": {
                   "it_per_s": round(1e6 / clustered["tables_rotated"]["us"], 1),
                   "it_per_s_warm_tables": round(1e6 / clustered["warm_tables"]["us"], 1),
                   "speedup_over_materialized": round(t_mat * 1e6 / clustered["tables_rotated"]["us"], 3),
                   "tables_rotated": clustered["tables_rotated"], "warm_tables": clustered["warm_tables"],
                   "crossprod_tables_rotated": clustered["crossprod"],
                   "note": "ilargi_plan_cluster: the plan keeps the entity table in join order (one more copy of S); "
                           "one launch reads S and R once and stores only partial sums"}},
        "ops_tables_rotated": ops_rot,
        "ops_warm_tables": ops_warm,
        "materialized_ops": mat_ops,
        "crossprod": ops_rot["crossprod"],
        "materialize": ops_warm["materialize"],
        "plan_build_ms": round(plan_ms, 2),
        "kernels": dict(sorted(kernels.items(), key=lambda kv: -kv[1]["us_per_step"])),
        "kernels_outside_step": dict(sorted(other_kernels.items(), key=lambda kv: -kv[1]["us_per_step"])[:12]),
        "stream_probe": probe,
        "scalar_ops": scalar,
        "kmeans_gnmf": models,
        "sparse_tables": sparse,
        "chooser": chooser_summary(records),
        "wide_batch": wide,
        "other_configs": configs,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
