#!/usr/bin/env python3
"""Benchmark of the MI355X Recurrent Residual Module library.

Default run: the headline workload, an AlexNet-shaped int8 conv stack -- five conv layers with
ReLU / requantisation / max-pool between them -- over synthetic 32-frame moving-patch sequences for `--streams`
independent video streams (chunks processed in parallel, Sec. 3.2 of the paper).  One "step" is one frame of
every stream through the whole stack (rrm_stack_step: per layer the difference and change map, then the
convolution of the changed part, with the nonlinearity fused into the next layer's difference kernel).  The
steps walk cyclically through two different 32-frame sequences (64 frames); steps W .. W+K-1 are timed, so a
sequence start (a frame in which everything changes) lies in the timed region whenever that range crosses a
multiple of 32; the JSON line says how many did.  Inputs are resident in HBM before the timed region.  After
the timed loops, outside them, sampled streams of every layer's stored projection are compared with the CPU
oracle ("verified").  Then every layer of the other configurations (single int8 conv, ResNet-shaped bf16
convs, FC sparse-delta, binary conv) is timed at 5 / 10 / 25 % change, at one stream and at `--config-streams`
streams ("configs"), the device's sustained copy and matrix-core rates are measured ("peaks"), and the CPU
oracle is timed on a bounded sample.  Prints ONE JSON line; everything else goes to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--streams S] [--no-configs] [--sweep] [--lean | --lean-case C]

--sweep times the full density grids of configs 2-4 and writes sweep.jsonl into the output folder plus a
table on stderr.  --lean runs only eager steps of the headline stack (delta path, then dense path) after the
calibration copy: the run a profiler wraps.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
MFMA_PEAK = {0: 5.0e15, 1: 2.5e15}  # dense int8 OP/s, bf16 FLOP/s
VALU_LANE_PEAK = 256 * 64 * 2.4e9   # lane-instructions / s: 256 CUs x 4 SIMD16 x 16 lanes x 2.4 GHz


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def macs(shape) -> int:
    """dense multiply count of a layer (Table 1 of the paper)."""
    if shape.kind == 1:
        return shape.n * shape.c_in * shape.c_out
    return shape.n * shape.h_out * shape.w_out * (shape.c_in // shape.groups) * shape.c_out * shape.kh * shape.kw


class Timer:
    """HIP-event timing on the current torch stream."""

    def __init__(self):
        import torch
        self.t = torch
        self.a = torch.cuda.Event(enable_timing=True)
        self.b = torch.cuda.Event(enable_timing=True)

    def __enter__(self):
        self.t.cuda.synchronize()
        self.a.record()
        return self

    def __exit__(self, *exc):
        self.b.record()
        self.t.cuda.synchronize()
        self.ms = self.a.elapsed_time(self.b)


# ------------------------------------------------------------------------------------------------
# config 1: the AlexNet-shaped int8 stack
# ------------------------------------------------------------------------------------------------
class Stack:
    def __init__(self, streams: int, T: int = 32, fuse: bool = True):
        import torch
        import paper_1802_09723_amd as rrm
        import rrm_synth as S
        self.torch, self.rrm, self.S = torch, rrm, S
        self.B, self.T = streams, T
        self.fuse, self.path = fuse, 0
        seqs = [S.config1(seed=S.seed_for(1, k), n=streams, T=T) for k in range(2)]
        self.cfg = seqs[0]
        self.layers = [rrm.Layer(l["shape"], S.I8, l["weights"], l["bias"]) for l in self.cfg["layers"]]
        # frames of two different sequences back to back: 0..T-1 of A, 0..T-1 of B
        self.frames = [torch.from_numpy(f).cuda() for s in seqs for f in s["frames"]]
        self.host_frames = [f for s in seqs for f in s["frames"]]
        self.bufs, self.meta = [], []
        for l, L in zip(self.cfg["layers"], self.layers):
            sh = l["shape"]
            ho, wo = L.y_shape[1], L.y_shape[2]
            po, qo = ((ho - 3) // 2 + 1, (wo - 3) // 2 + 1) if l["pool"] else (ho, wo)
            self.bufs.append(torch.empty((sh.n, po, qo, sh.c_out), dtype=torch.int8, device="cuda"))
            self.meta.append((sh.n, ho, wo, sh.c_out, bool(l["pool"])))
        self.ysnap = [L.snapshot_ptrs()[1] for L in self.layers]
        self.shifts = self._calibrate()
        self.graph = None

    def _calibrate(self):
        """Per-layer right shift of the harness requantisation: smallest shift that brings the
        99.9th percentile of ReLU(y) on the first frame to <= 127 (fixed for the whole run)."""
        torch, rrm = self.torch, self.rrm
        shifts = []
        x = self.frames[0]
        for i, L in enumerate(self.layers):
            y = torch.empty(L.y_shape, dtype=torch.int32, device="cuda")
            L.dense(x, y)
            torch.cuda.synchronize()
            v = float(np.percentile(np.maximum(y[:1].cpu().numpy(), 0), 99.9))
            s = 0
            while (int(v) >> s) > 127:
                s += 1
            shifts.append(s)
            n, ho, wo, c, pool = self.meta[i]
            rrm.relu_requant_pool_i8(y, self.bufs[i], n, ho, wo, c, s, pool)
            x = self.bufs[i]
        torch.cuda.synchronize()
        return shifts

    def set_path(self, path: int):
        for L in self.layers:
            L.set_option("path", path)
        self.path = path
        self.graph = None

    def frame(self, x):
        """One frame of every stream through the stack.  Delta path: conv2-conv5 take their input straight
        from the stored projection of the layer before (rrm_step_from_projection: f and the difference in
        one pass, only where that projection changed); the last layer's f, and every f with --no-fuse or on
        the dense path, is the separate kernel (bufs[i] holds the previous frame's result)."""
        last = len(self.layers) - 1
        if self.fuse and self.path != 2:  # the library's stack call: Algorithm 1's loop over the layers
            self.rrm.stack_step(self.layers, self.shifts, [m[4] for m in self.meta], x, self.bufs[last])
            return
        for i, L in enumerate(self.layers):
            n, ho, wo, c, pool = self.meta[i]
            if i > 0 and self.fuse and self.path != 2:
                L.step_from_projection(self.layers[i - 1], self.shifts[i - 1], self.meta[i - 1][4])
            else:
                L.step(x)
            if i == last or not self.fuse or self.path == 2:
                L.relu_requant_pool_changed(self.bufs[i], self.shifts[i], pool)
            x = self.bufs[i]

    def capture(self):
        """One HIP graph per frame of the two sequences: a step reads its frame where it lies in HBM (a single
        graph with a static input would add a copy of every frame to every step)."""
        torch = self.torch
        self.frame(self.frames[0])  # make sure nothing lazy happens inside the captures
        torch.cuda.synchronize()
        self.graph = []
        pool = None
        for f in self.frames:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, pool=pool):
                self.frame(f)
            pool = pool or g.pool()
            self.graph.append(g)

    def run_steps(self, k0: int, K: int, use_graph: bool):
        nf = len(self.frames)
        for k in range(k0, k0 + K):
            if use_graph:
                self.graph[k % nf].replay()
            else:
                self.frame(self.frames[k % nf])

    def timed(self, K: int, W: int, use_graph: bool) -> float:
        """ms per step over exactly K steps after W warm-up steps."""
        if use_graph and self.graph is None:
            self.capture()
        self.run_steps(0, W, use_graph)
        with Timer() as t:
            self.run_steps(W, K, use_graph)
        return t.ms / K

    def verify(self, frame_index: int, streams):
        """Compare, for the given streams, every layer's stored projection with the CPU oracle's dense
        projection of frame `frame_index` through the stack (Sec. 3.2: the recurrence yields what a normal
        layer computes from the frame itself).  Returns the number of differing entries (int8 stack: exact)."""
        import oracle
        S = self.S
        self.torch.cuda.synchronize()
        got = [L.y_snapshot() for L in self.layers]
        bad = 0
        for b in streams:
            x = np.ascontiguousarray(self.host_frames[frame_index][b:b + 1])
            for i, l in enumerate(self.cfg["layers"]):
                y = oracle.dense(l["shape"].with_n(1), S.I8, l["weights"], l["bias"], x)
                bad += int(np.count_nonzero(got[i][b:b + 1].cpu().numpy() != y))
                x = oracle.relu_requant_pool(y, self.shifts[i], l["pool"])
            # f of the last layer (the stack call's output buffer)
            bad += int(np.count_nonzero(self.bufs[-1][b:b + 1].cpu().numpy() != x))
        return bad

    def profile_layers(self, K: int, W: int):
        """Eager pass with every kernel of rrm_step bracketed by HIP events (the library's
        "profile" option): per-layer average scan / compute kernel time and change statistics."""
        self.run_steps(0, W, False)
        self.torch.cuda.synchronize()
        s0 = [L.stats() for L in self.layers]
        for L in self.layers:
            L.set_option("profile", 1)
        self.run_steps(W, K, False)
        self.torch.cuda.synchronize()
        out = []
        for L, a in zip(self.layers, s0):
            scan_us, comp_us, n = L.kernel_times()
            L.set_option("profile", 0)
            b = L.stats()
            d = {k: b[k] - a[k] for k in ("changed_elems", "changed_units", "active_tiles", "total_tiles", "delta_steps")}
            out.append({"scan_us": scan_us / max(n, 1), "compute_us": comp_us / max(n, 1), "steps": n,
                        "tile_positions": b["tile_positions"], **d})
        return out


def conv_alg_bytes(shape, esize, changed_units_per_step, active_positions_per_step, terms=1):
    """Algorithmic HBM bytes of one delta step of a conv layer, split by kernel.
    scan: both copies of x are read once; changed 16-byte units write their difference (terms
          buffers) and the snapshot.
    tile: the changed difference units are read once, the weights once (if anything changed),
          and the output positions whose receptive field changed are read and written once (4-byte
          outputs).  `active_positions_per_step` counts real output positions (clipped blocks of the
          window-tile kernel are counted by the caller as what lies inside the map)."""
    xb = shape.n * shape.h * shape.w * shape.c_in * esize
    wb = shape.c_out * shape.kh * shape.kw * (shape.c_in // shape.groups) * esize
    scan = 2 * xb + changed_units_per_step * 16 * (1 + terms)
    tile = changed_units_per_step * 16 * terms + 2 * active_positions_per_step * shape.c_out * 4 + (wb if active_positions_per_step > 0 else 0)
    return scan, tile


def active_positions(shape, stats_row, tiles_per_step):
    """Output positions under the active tiles of a step: exact for the position-gather kernel; for 4x4 (8x8)
    blocks the blocks' share of the map (clipped border blocks hold fewer positions)."""
    tp = stats_row.get("tile_positions", 16) or 1
    if tp == 1:
        return tiles_per_step
    side = int(round(tp ** 0.5))
    blocks = shape.n * -(-shape.h_out // side) * -(-shape.w_out // side)
    return tiles_per_step / blocks * shape.n * shape.h_out * shape.w_out


COPY_BYTES = 64 << 20
_CAL = []  # the calibration copy's two buffers


def calibration_copy(reps: int = 4):
    """A plain copy of known size (COPY_BYTES read, COPY_BYTES written per launch: the library's copy probe), so
    that a rocprofv3 --pmc run of this script holds the reading of FETCH_SIZE / WRITE_SIZE for a known number
    of HBM bytes next to the library's kernels.  In the --lean modes it also marks, in the list of dispatches,
    where the counted steps begin and end."""
    import torch
    import paper_1802_09723_amd as rrm
    if not _CAL:
        _CAL.append(torch.arange(COPY_BYTES // 4, dtype=torch.int32, device="cuda"))
        _CAL.append(torch.empty_like(_CAL[0]))
    src, dst = _CAL
    for _ in range(reps):
        rrm.probe_copy(dst, src, COPY_BYTES)
    torch.cuda.synchronize()


def measure_peaks():
    """What this device sustains on the library's two probes: a streaming copy of 1 GiB (bytes read + written
    per second) and a register-resident matrix-core loop on every compute unit (int8 and bf16)."""
    import torch
    import paper_1802_09723_amd as rrm
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.zero_()
    rrm.probe_copy(dst, src, nbytes)
    with Timer() as t:
        for _ in range(5):
            rrm.probe_copy(dst, src, nbytes)
    copy = 2 * nbytes * 5 / (t.ms * 1e-3)
    del src, dst
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = {"copy_GBps": round(copy / 1e9, 1), "copy_frac_of_8TBps": round(copy / HBM_PEAK, 3)}
    wgs, iters = 256 * 8, 4096
    for name, dt, per in (("mfma_i8_TOPs", rrm.I8, 65536), ("mfma_bf16_TFLOPs", rrm.BF16, 32768)):
        rrm.probe_mfma(dt, sink, 64, wgs)
        with Timer() as t:
            rrm.probe_mfma(dt, sink, iters, wgs)
        rate = wgs * 4 * 4 * iters * per / (t.ms * 1e-3)
        out[name] = round(rate / 1e12, 1)
        out[name.split("_T")[0] + "_frac_of_published"] = round(rate / MFMA_PEAK[0 if dt == rrm.I8 else 1], 3)
    return out


def measured_traffic(kernel: str, streams: int):
    """HBM bytes per launch of `kernel` ("scan:conv1", "tile:conv3", ...) from the committed
    counter summary of this workload (profiles/hbm_traffic_alexnet_streams<S>.txt, rows
    `<kernel> <fetch bytes> <write bytes>`), or None when there is no such measurement."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_alexnet_streams{streams}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == kernel:
            try:
                return int(float(f[1]) + float(f[2]))
            except ValueError:
                return None
    return None


def run_stack(args):
    import torch
    calibration_copy()
    st = Stack(args.streams, fuse=not args.no_fuse)
    if args.conv_kernel:
        for L in st.layers:
            try:
                L.set_option("conv_kernel", args.conv_kernel)
            except Exception:  # (a layer the position-gather kernel does not take keeps its kernel)
                pass
            L.reset()
    B = st.B
    shapes = [l["shape"] for l in st.cfg["layers"]]
    names = [l["name"] for l in st.cfg["layers"]]
    log(f"[bench] AlexNet int8 conv stack, streams={B}, shifts={st.shifts}")

    # ---- headline: K steps of the delta path (graph replay unless --no-graph) --------------------
    st.set_path(0)
    ms_delta = st.timed(args.steps, args.warmup, not args.no_graph)
    # ---- outside the timed region: what the timed steps left behind, against the CPU oracle -----------
    nf, last = len(st.frames), args.warmup + args.steps - 1
    sample = sorted({0, B // 2, B - 1})
    verified = {"streams": sample, "what": "every layer's stored projection and f of the last layer, element by element, "
                "against the CPU oracle's dense projection of the same frame"}
    verified["after_timed_loop"] = st.verify(last % nf, sample) == 0
    # ... and on across the boundary between the two sequences, to the second frame of the next sequence
    more = (st.T + 1 - last) % st.T or st.T
    st.run_steps(last + 1, more, not args.no_graph)
    verified["after_sequence_boundary"] = st.verify((last + more) % nf, sample) == 0
    starts = sum(1 for k in range(args.warmup, args.warmup + args.steps) if k % st.T == 0)
    # ---- same steps with every layer recomputed densely (the library's own dense path) -----------
    st.set_path(2)
    ms_dense = st.timed(args.steps, args.warmup, not args.no_graph)
    verified["dense_path"] = st.verify(last % nf, sample) == 0
    verified["ok"] = bool(verified["after_timed_loop"] and verified["after_sequence_boundary"] and verified["dense_path"])
    log("[verified]", json.dumps(verified))
    st.set_path(0)
    # ---- per-kernel times and change statistics (eager, event-bracketed) -------------------------
    prof = st.profile_layers(args.steps, args.warmup)
    st.set_path(2)
    prof_dense = st.profile_layers(min(args.steps, 64), 4)
    st.set_path(0)

    frames_per_s = B * 1e3 / ms_delta
    total_macs = sum(macs(s) for s in shapes)  # for all B streams, one frame each
    layers = []
    dom = None
    prev = None  # (shape, active sub-tiles per step) of the layer before
    for nm, sh, p, pd in zip(names, shapes, prof, prof_dense):
        n = max(p["steps"], 1)
        cu = p["changed_units"] / n
        at = active_positions(sh, p, p["active_tiles"] / n)  # output positions written per step
        scan_b, tile_b = conv_alg_bytes(sh, 1, cu, at)
        if prev is not None and st.fuse:
            # fused scan: the producer's written positions are read once (int32), the stored input is read
            # only under them (about the same share of it), changed units are written twice
            psh, pat = prev
            share = pat / (psh.n * psh.h_out * psh.w_out)
            scan_b = pat * psh.c_out * 4 + share * sh.n * sh.h * sh.w * sh.c_in + cu * 32
        prev = (sh, at)
        rho_elem = p["changed_elems"] / n / (sh.n * sh.h * sh.w * sh.c_in)
        rho_tile = p["active_tiles"] / max(p["total_tiles"], 1)
        ops_alg = 2 * rho_elem * macs(sh)
        t_step = p["scan_us"] + p["compute_us"]
        t_roof_hbm = (scan_b + tile_b) / HBM_PEAK * 1e6
        t_roof_mfma = ops_alg / MFMA_PEAK[0] * 1e6
        rec = {
            "layer": nm, "rho_elem": round(rho_elem, 4), "rho_tile": round(rho_tile, 4),
            "scan_us": round(p["scan_us"], 2), "tile_us": round(p["compute_us"], 2),
            "dense_us": round(pd["compute_us"], 2),
            "frames_per_s": round(B * 1e6 / t_step, 1),
            "dense_equiv_gops": round(2 * macs(sh) / t_step * 1e-3, 1),
            "speedup_vs_dense_kernel": round((pd["compute_us"] + pd["scan_us"]) / t_step, 3),
            "alg_bytes": int(scan_b + tile_b), "roof_us": round(max(t_roof_hbm, t_roof_mfma), 3),
            "roof_bound": "hbm" if t_roof_hbm >= t_roof_mfma else "mfma",
            "roof_frac": round(max(t_roof_hbm, t_roof_mfma) / t_step, 4),
        }
        layers.append(rec)
        log("[layer]", json.dumps(rec))
        for kind, us, byts in (("scan", p["scan_us"], scan_b), ("tile", p["compute_us"], tile_b)):
            if dom is None or us > dom["us"]:
                dom = {"kernel": f"{kind}:{nm}", "us": us, "bytes": byts,
                       "ops": ops_alg if kind == "tile" else 0.0}

    # the dominant kernel is priced against whichever of its two rooflines is the larger time
    t_hbm, t_mfma = dom["bytes"] / HBM_PEAK, dom["ops"] / MFMA_PEAK[0]
    traffic = measured_traffic(dom["kernel"], B)
    if t_hbm >= t_mfma:
        achieved = dom["bytes"] / (dom["us"] * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": round(achieved * 1e9 / HBM_PEAK, 4)}
    else:
        achieved = dom["ops"] / (dom["us"] * 1e-6) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_PEAK[0] / 1e12, "unit": "TOP/s",
                    "frac": round(achieved * 1e12 / MFMA_PEAK[0], 4)}
    roofline.update({"traffic": traffic, "kernel": dom["kernel"], "avg_us": round(dom["us"], 2),
                     "alg_bytes_per_launch": int(dom["bytes"]), "alg_ops_per_launch": int(dom["ops"]),
                     "hbm_frac": round(t_hbm / (dom["us"] * 1e-6), 4), "mfma_frac": round(t_mfma / (dom["us"] * 1e-6), 5)})

    floor_us = launch_floor(st)
    cpu = None if args.skip_cpu else cpu_baseline_stack(st)
    out = {
        "metric": "frames_per_s", "value": round(frames_per_s, 1), "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_delta, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "cfg1_alexnet_conv_stack_int8", "streams": B, "frames_per_sequence": st.T,
                   "graph_replay": not args.no_graph, "fused_f": not args.no_fuse,
                   "sequence_starts_in_timed_region": starts},
        "verified": verified,
        "dense_equiv_gops": round(2 * total_macs / (ms_delta * 1e-3) * 1e-9, 1),
        "ms_per_step_dense_path": round(ms_dense, 5),
        "speedup_vs_dense_path": round(ms_dense / ms_delta, 3),
        "launch_floor_us": round(floor_us, 2),
        "layers": layers, "roofline": roofline, "cpu_baseline": cpu,
    }
    return out


def launch_floor(st) -> float:
    """us per launch of a one-thread kernel replayed back to back in a graph (the floor under
    every per-kernel time quoted here)."""
    import torch
    rrm = st.rrm
    y = torch.zeros((1, 3, 3, 1), dtype=torch.int32, device="cuda")
    o = torch.zeros((1, 1, 1, 1), dtype=torch.int8, device="cuda")
    rrm.relu_requant_pool_i8(y, o, 1, 3, 3, 1, 0, True)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(100):
            rrm.relu_requant_pool_i8(y, o, 1, 3, 3, 1, 0, True)
    g.replay()
    with Timer() as t:
        for _ in range(10):
            g.replay()
    return t.ms * 1e3 / 1000


def cpu_baseline_stack(st, budget_s: float = 8.0):
    """The CPU oracle (dense projection of every layer, its own nonlinearity in between) on this host's
    cores: whole 32-frame sequences, one stream after the other, until about `budget_s` seconds of work.
    Beside it, on shorter samples: the same on one thread, and the oracle's own recurrence (Algorithm 1 on the
    CPU: work proportional to the changed inputs) on all threads and on one."""
    import oracle
    S = st.S
    cfg = st.cfg
    layers1 = [(l["shape"].with_n(1), l) for l in cfg["layers"]]
    nthreads = oracle.threads()

    def dense_frames(budget, max_streams):
        frames_done, streams_done, t0 = 0, 0, time.perf_counter()
        while streams_done < max_streams and (time.perf_counter() - t0) < budget:
            for f in range(st.T):
                x = np.ascontiguousarray(st.host_frames[f][streams_done:streams_done + 1])
                for i, (sh, l) in enumerate(layers1):
                    y = oracle.dense(sh, S.I8, l["weights"], l["bias"], x)
                    x = oracle.relu_requant_pool(y, st.shifts[i], l["pool"])
                frames_done += 1
                if (time.perf_counter() - t0) > 2 * budget:
                    break
            streams_done += 1
        return frames_done, streams_done, time.perf_counter() - t0

    def recurrence_frames(budget):
        states = [oracle.State(sh, S.I8, l["weights"], l["bias"]) for sh, l in layers1]
        frames_done, t0, t_first = 0, time.perf_counter(), 0.0
        for f in range(st.T):
            x = np.ascontiguousarray(st.host_frames[f][0:1])
            for i, (sh, l) in enumerate(layers1):
                x = oracle.relu_requant_pool(states[i].step(x), st.shifts[i], l["pool"])
            if f == 0:
                t_first = time.perf_counter() - t0  # (the first frame changes everything: not a delta step)
            else:
                frames_done += 1
            if (time.perf_counter() - t0) > budget and frames_done >= 2:
                break
        return frames_done, time.perf_counter() - t0 - t_first

    frames_done, streams_done, dt = dense_frames(budget_s, st.B)
    out = {"value": round(frames_done / dt, 3), "unit": "frames/s", "cores": nthreads, "kind": "oracle",
           "sample": f"{frames_done} frames ({streams_done} streams x {st.T} frames) through the 5-layer stack "
                     f"(dense oracle per layer), {dt:.1f} s"}
    k, dt = recurrence_frames(4.0)
    out["oracle_step"] = {"value": round(k / dt, 3), "unit": "frames/s", "cores": nthreads,
                          "sample": f"{k} delta frames of stream 0 through the oracle's recurrence, {dt:.1f} s"}
    oracle.set_threads(1)
    try:
        k, _, dt = dense_frames(2.0, 1)
        out["single_thread"] = {"value": round(k / dt, 3), "unit": "frames/s", "cores": 1,
                                "sample": f"{k} frames of stream 0, dense oracle, {dt:.1f} s"}
        k, dt = recurrence_frames(3.0)
        out["oracle_step_single_thread"] = {"value": round(k / dt, 3), "unit": "frames/s", "cores": 1,
                                            "sample": f"{k} delta frames of stream 0, {dt:.1f} s"}
    finally:
        oracle.set_threads(nthreads)
    return out


# ------------------------------------------------------------------------------------------------
# configs 0, 2, 3, 4 (one layer at a time)
# ------------------------------------------------------------------------------------------------
def time_layer(seq, to_dev, weights, reps: int = 5, eps: float = 0.0, drift: bool = False, cold: bool = False, opts=None):
    """Per-step wall time (graph of one whole sequence, delta and dense path) and event-bracketed
    kernel times of one layer over its frame sequence.  eps: truncation threshold (bf16 layers).
    drift (bf16 conv): after the whole sequence on the delta path, max |stored projection - dense projection of
    the last frame| / max |dense projection|, with the difference carried as two bf16 terms and as one.
    cold: the delta and the dense step again with the caches flushed before each step (a 1 GiB copy)."""
    import torch
    import paper_1802_09723_amd as rrm
    L = rrm.Layer(seq.shape, seq.dtype, weights, seq.bias)
    if eps:
        L.set_threshold(eps)
    for k, v in (opts or {}).items():
        L.set_option(k, v)
    xs = [to_dev(f) for f in seq.frames]
    res = {}
    for tag, path in (("delta", 0), ("dense", 2)):
        L.set_option("path", path)
        for x in xs:  # warm-up pass, leaves the snapshot at the last frame
            L.step(x)
        torch.cuda.synchronize()
        # ping-pong through the sequence: T-2, ..., 0, 1, ..., T-1.  Every step is a genuine
        # consecutive-frame difference and the replay ends where it starts.
        order = xs[-2::-1] + xs[1:]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for x in order:
                L.step(x)
        g.replay()
        with Timer() as t:
            for _ in range(reps):
                g.replay()
        res[f"{tag}_us"] = t.ms * 1e3 / (reps * len(order))
        # event-bracketed kernels (eager)
        s0 = L.stats()
        L.set_option("profile", 1)
        for x in order:
            L.step(x)
        torch.cuda.synchronize()
        a, c, n = L.kernel_times()
        L.set_option("profile", 0)
        s1 = L.stats()
        res[f"{tag}_scan_us"], res[f"{tag}_compute_us"] = a / max(n, 1), c / max(n, 1)
        if path == 0:
            res["stats"] = {k: (s1[k] - s0[k]) / max(n, 1)
                            for k in ("changed_elems", "changed_units", "active_tiles", "total_tiles", "truncated_elems")}
            res["stats"]["tile_positions"] = s1["tile_positions"]
        if cold:
            big_a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            big_b = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in order[:12]]
            for x, (e0, e1) in zip(order, ev):
                rrm.probe_copy(big_b, big_a, 1 << 30)
                e0.record()
                L.step(x)
                e1.record()
            torch.cuda.synchronize()
            res[f"{tag}_cold_us"] = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3
            del big_a, big_b
    if drift:
        y_ref = torch.empty(L.y_shape, dtype=torch.float32, device="cuda")
        L.dense(xs[-1], y_ref)
        for terms in (2, 1):
            L.set_option("path", 1)  # (never the in-kernel switch to recomputation, which would hide the drift)
            L.set_option("bf16_terms", terms)
            L.reset()
            for x in xs:
                L.step(x)
            y = L.y_snapshot()
            res[f"drift_terms{terms}"] = float((y - y_ref).abs().max() / y_ref.abs().max())
        L.set_option("bf16_terms", 2)
    L.destroy()
    return res


CONFIG_GRID = {2: (0.05, 0.10, 0.25), 3: (0.05, 0.10, 0.25), 4: (0.05, 0.10, 0.20)}


def config_rows(stream_counts, full: bool):
    """Every layer of configurations 0, 2, 3, 4 over a density grid (full: the configurations' whole grids and
    the truncation-threshold cases; else 5 / 10 / 25 %), at each of `stream_counts` streams."""
    import torch
    import rrm_synth as S
    rows = []

    def dev_i8(f):
        return torch.from_numpy(np.ascontiguousarray(f)).cuda()

    def dev_bf16(f):
        return torch.from_numpy(np.ascontiguousarray(f).view(np.int16)).cuda()

    def dev_bin(f):
        return torch.from_numpy(S.pack_pm1(f).view(np.int32)).cuda()

    def conv_row(config, seq, r, ns, esize, terms, peak, sfx, extra=None):
        sh, stt = seq.shape, r["stats"]
        pos = active_positions(sh, stt, stt["active_tiles"])
        scan_b, tile_b = conv_alg_bytes(sh, esize, stt["changed_units"], pos, terms=terms)
        rho_elem = stt["changed_elems"] / (sh.n * sh.h * sh.w * sh.c_in)
        ops = 2 * rho_elem * macs(sh)
        kt = r["delta_scan_us"] + r["delta_compute_us"]
        t_hbm, t_mfma = (scan_b + tile_b) / HBM_PEAK * 1e6, ops / peak * 1e6
        roof = max(t_hbm, t_mfma)
        row = {"config": config, "case": seq.name + sfx, "streams": ns, "rho_elem": rho_elem,
               "rho_tile": stt["active_tiles"] / max(stt["total_tiles"], 1),
               "step_us": r["delta_us"], "dense_step_us": r["dense_us"], "scan_us": r["delta_scan_us"],
               "compute_us": r["delta_compute_us"], "dense_kernel_us": r["dense_compute_us"],
               "frames_per_s": ns * 1e6 / r["delta_us"], "dense_equiv_gops": 2 * macs(sh) / r["delta_us"] * 1e-3,
               "speedup_vs_dense": r["dense_us"] / r["delta_us"], "alg_bytes": scan_b + tile_b, "roof_us": roof,
               "roof_bound": "hbm" if t_hbm >= t_mfma else "mfma",
               "roof_frac_kernels": roof / kt, "roof_frac_wall": roof / r["delta_us"]}
        for k in ("drift_terms1", "drift_terms2"):
            if k in r:
                row[k] = r[k]
        row.update(extra or {})
        rows.append(row)
        log("[config]", json.dumps(row))

    for ns in stream_counts:
        # many streams: shorter sequences keep the synthetic data small; one stream: the configs' lengths
        Tc, Tf, Tb = (16, 64, 32) if ns == 1 else (6, 8, 6)
        sfx = "" if ns == 1 else f"_s{ns}"
        # config 0: one small int8 conv
        seq = S.config0(n=ns, T=8)
        conv_row(0, seq, time_layer(seq, dev_i8, seq.weights), ns, 1, 1, MFMA_PEAK[0], sfx)
        # config 2: ResNet-18-shaped bf16 3x3 convs
        for layer, hw, c in S.RESNET_LAYERS:
            for frac in (S.RESNET_DENSITIES if full else CONFIG_GRID[2]):
                seq = S.config2(layer, frac, n=ns, T=Tc)
                conv_row(2, seq, time_layer(seq, dev_bf16, seq.weights, drift=(ns == 1)), ns, 2, 2, MFMA_PEAK[1], sfx)
        # The truncation threshold (Sec. 3.4, "Improving sparsity"; the paper's experiments use 1e-2): the same
        # block-redraw sequences with a little noise on every entry, as a camera would add; without a
        # threshold every entry changes, with it the noise is truncated.
        if full and ns > 1:
            for layer, hw, c in S.RESNET_LAYERS[:2]:
                base = S.config2(layer, 0.05, n=ns, T=Tc)
                rng = S.rng_for(S.seed_for(2, 900) + hw)
                noisy = [base.frames[0]] + [
                    S.f32_to_bf16_bits(np.maximum(S.bf16_bits_to_f32(f) + rng.normal(0, 0.0015, size=f.shape).astype(np.float32), 0))
                    for f in base.frames[1:]]
                for eps in (0.0, 1e-2):
                    seq = S.Sequence_(base.shape, base.dtype, base.weights, base.bias, noisy, f"{base.name}_noise_eps{eps:g}")
                    r = time_layer(seq, dev_bf16, seq.weights, eps=eps)
                    conv_row(2, seq, r, ns, 2, 2, MFMA_PEAK[1], sfx,
                             {"epsilon": eps, "truncated_frac": r["stats"]["truncated_elems"] / (ns * hw * hw * c)})
        # config 3: FC sparse-delta mat-vec
        for layer, ci, co in S.FC_LAYERS:
            for dt, es in ((S.I8, 1), (S.BF16, 2)):
                for frac in (S.FC_DENSITIES if full else CONFIG_GRID[3]):
                    seq = S.config3(layer, dt, frac, n=ns, T=Tf)
                    r = time_layer(seq, dev_i8 if dt == S.I8 else dev_bf16, seq.weights, cold=(ns == 1))
                    nnz = r["stats"]["changed_elems"]  # over all streams
                    # a column of W is priced once however many streams need it (at most all of W)
                    byts = min(nnz, ci) * co * es + ns * (2 * ci * es + 2 * co * 4)
                    kt = r["delta_scan_us"] + r["delta_compute_us"]
                    roof = byts / HBM_PEAK * 1e6
                    row = {"config": 3, "case": seq.name + sfx, "streams": ns, "rho_elem": nnz / (ns * ci),
                           "step_us": r["delta_us"], "dense_step_us": r["dense_us"], "scan_us": r["delta_scan_us"],
                           "compute_us": r["delta_compute_us"], "dense_kernel_us": r["dense_compute_us"],
                           "frames_per_s": ns * 1e6 / r["delta_us"],
                           "dense_equiv_gops": 2 * ns * ci * co / r["delta_us"] * 1e-3,
                           "speedup_vs_dense": r["dense_us"] / r["delta_us"],
                           "alg_bytes": byts, "roof_us": roof, "roof_bound": "hbm",
                           "columns_GBps": nnz * co * es / (kt * 1e-6) / 1e9,
                           "dense_GBps": ns * ci * co * es / (r["dense_compute_us"] * 1e-6) / 1e9,
                           "roof_frac_kernels": roof / kt, "roof_frac_wall": roof / r["delta_us"]}
                    if "delta_cold_us" in r:
                        row["cold_step_us"], row["cold_dense_step_us"] = r["delta_cold_us"], r["dense_cold_us"]
                    rows.append(row)
                    log("[config]", json.dumps(row))
        # config 3 with pruned weights (Sec. 4.3: compressed models keep about a tenth of their FC weights): a seeded
        # random tenth of fc6's weights survives; the delta step walks the non-zeros of the changed columns
        if ns == 1:
            for dt, es in ((S.I8, 1), (S.BF16, 2)):
                for frac in (0.05, 0.25):
                    seq = S.pruned(S.config3("fc6", dt, frac, n=ns, T=Tf), 0.10, S.seed_for(3, 77))
                    r = time_layer(seq, dev_i8 if dt == S.I8 else dev_bf16, seq.weights, opts={"fc_sparse_weights": 1})
                    ci, co = 9216, 4096
                    nnz = r["stats"]["changed_elems"]
                    nzw = float(np.count_nonzero(seq.weights)) / seq.weights.size
                    # per changed column its non-zeros (value + 2-byte row) and two offsets; x twice; y read and written
                    byts = nnz * (co * nzw * (es + 2) + 8) + ns * (2 * ci * es + 2 * co * 4)
                    kt = r["delta_scan_us"] + r["delta_compute_us"]
                    roof = byts / HBM_PEAK * 1e6
                    row = {"config": 3, "case": seq.name, "streams": ns, "rho_elem": nnz / (ns * ci), "weight_density": nzw,
                           "step_us": r["delta_us"], "dense_step_us": r["dense_us"], "scan_us": r["delta_scan_us"],
                           "compute_us": r["delta_compute_us"], "dense_kernel_us": r["dense_compute_us"],
                           "frames_per_s": ns * 1e6 / r["delta_us"], "dense_equiv_gops": 2 * ns * ci * co / r["delta_us"] * 1e-3,
                           "speedup_vs_dense": r["dense_us"] / r["delta_us"], "alg_bytes": byts, "roof_us": roof,
                           "roof_bound": "hbm", "roof_frac_kernels": roof / kt, "roof_frac_wall": roof / r["delta_us"]}
                    rows.append(row)
                    log("[config]", json.dumps(row))
        # config 4: binary conv
        for layer, hw, c in S.XNOR_LAYERS:
            for frac in (S.XNOR_FLIPS if full else CONFIG_GRID[4]):
                seq = S.config4(layer, frac, n=ns, T=Tb)
                r = time_layer(seq, dev_bin, S.pack_pm1(seq.weights))
                sh, stt = seq.shape, r["stats"]
                words = stt["changed_units"] * 4  # upper bound on 32-bit words holding a flipped bit
                lane_instr = 2 * words * c * 9
                roof = max(lane_instr / VALU_LANE_PEAK,
                           (2 * ns * hw * hw * c / 8 + 2 * active_positions(sh, stt, stt["active_tiles"]) * c * 4) / HBM_PEAK) * 1e6
                kt = r["delta_scan_us"] + r["delta_compute_us"]
                row = {"config": 4, "case": seq.name + sfx, "streams": ns,
                       "rho_elem": stt["changed_elems"] / (ns * hw * hw * c),
                       "rho_tile": stt["active_tiles"] / max(stt["total_tiles"], 1), "step_us": r["delta_us"],
                       "dense_step_us": r["dense_us"], "scan_us": r["delta_scan_us"], "compute_us": r["delta_compute_us"],
                       "dense_kernel_us": r["dense_compute_us"], "frames_per_s": ns * 1e6 / r["delta_us"],
                       "dense_equiv_gops": 2 * macs(sh) / r["delta_us"] * 1e-3,
                       "speedup_vs_dense": r["dense_us"] / r["delta_us"],
                       "roof_us": roof, "roof_bound": "alu", "roof_frac_kernels": roof / kt,
                       "roof_frac_wall": roof / r["delta_us"]}
                rows.append(row)
                log("[config]", json.dumps(row))
    return rows


def compact(rows):
    """The per-configuration array of the JSON line: case, streams, change density, wall time of a delta step and
    of a dense step (graph replay), roofline time and the fraction of it reached on wall time (and on the
    kernels' own time, which leaves out launch gaps)."""
    out = []
    for r in rows:
        c = {"cfg": r["config"], "case": r["case"], "n": r["streams"], "rho": round(r["rho_elem"], 4),
             "us": round(r["step_us"], 2), "dense_us": round(r["dense_step_us"], 2), "roof_us": round(r["roof_us"], 3),
             "bound": r["roof_bound"], "frac": round(r["roof_frac_wall"], 4), "frac_kernels": round(r["roof_frac_kernels"], 4)}
        for k, name in (("cold_step_us", "cold_us"), ("cold_dense_step_us", "cold_dense_us"),
                        ("drift_terms1", "drift_terms1"), ("drift_terms2", "drift_terms2")):
            if k in r:
                c[name] = float(f"{r[k]:.3g}")
        out.append(c)
    return out


def write_sweep(rows):
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", "sweep.jsonl"), "w") as f:
        for r in rows:
            f.write(json.dumps(r) + "\n")
    log("| case | rho_elem | step us | dense us | speedup | scan us | compute us | roof us | frac (kernels) | frac (wall) |")
    log("|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        log(f"| {r['case']} | {r['rho_elem']:.3f} | {r['step_us']:.2f} | {r['dense_step_us']:.2f} | {r['speedup_vs_dense']:.2f} | "
            f"{r['scan_us']:.2f} | {r['compute_us']:.2f} | {r['roof_us']:.3f} | {r['roof_frac_kernels']:.3f} | {r['roof_frac_wall']:.3f} |")


def run_lean_case(args):
    """Eager steps of one layer of configurations 0, 2, 3, 4 and nothing else, for a profiler.  --lean-case is
    "<cfg>:<layer>:<density>:<streams>[:<dtype i8|bf16>][:path=<p>]", e.g. "3:fc6:0.25:1:i8" or "2:r14:0.05:1:path=3".
    Dispatch order: warm-up pass, copy, the counted delta steps (per step the layer's kernels in launch order),
    copy, dense warm-up pass, copy, the counted dense steps, copy."""
    import torch
    import rrm_synth as S
    import paper_1802_09723_amd as rrm
    f = args.lean_case.split(":")
    cfg, layer, frac, ns = int(f[0]), f[1], float(f[2]), int(f[3])
    opts = [x for x in f[4:] if "=" in x]
    dts = [x for x in f[4:] if "=" not in x]
    if cfg == 0:
        seq, w = S.config0(n=ns, T=8), None
    elif cfg == 2:
        seq, w = S.config2(layer, frac, n=ns, T=16 if ns == 1 else 6), None
    elif cfg == 3:
        seq, w = S.config3(layer, S.BF16 if dts and dts[0] == "bf16" else S.I8, frac, n=ns, T=64 if ns == 1 else 8), None
    elif cfg == 4:
        seq = S.config4(layer, frac, n=ns, T=32 if ns == 1 else 6)
        w = S.pack_pm1(seq.weights)
    else:
        raise SystemExit("--lean-case: configuration 0, 2, 3 or 4")
    w = seq.weights if w is None else w

    def dev(fr):
        if seq.dtype == S.BIN:
            return torch.from_numpy(S.pack_pm1(fr).view(np.int32)).cuda()
        a = np.ascontiguousarray(fr)
        return torch.from_numpy(a if seq.dtype == S.I8 else a.view(np.int16)).cuda()

    L = rrm.Layer(seq.shape, seq.dtype, w, seq.bias)
    for o in opts:
        k, v = o.split("=")
        if k != "path":
            L.set_option(k, int(v))
    xs = [dev(fr) for fr in seq.frames]
    order = xs[-2::-1] + xs[1:]
    path = int(dict(o.split("=") for o in opts).get("path", 0))
    calibration_copy(0)  # (allocates the markers' buffers)
    for p in (path, 2):
        L.set_option("path", p)
        for x in xs:
            L.step(x)
        torch.cuda.synchronize()
        calibration_copy(1)
        for x in order[:args.steps]:
            L.step(x)
        torch.cuda.synchronize()
        calibration_copy(1)
    st = L.stats()
    L.destroy()
    return {"lean_case": args.lean_case, "name": seq.name, "counted_steps": min(args.steps, len(order)),
            "changed_elems": int(st["changed_elems"]), "changed_units": int(st["changed_units"])}


def run_lean(args):
    """Eager steps of the headline stack and nothing else, for a profiler: `--steps` delta steps (frames
    warmup .. warmup+steps-1 of the cyclic pair of sequences), then as many dense-path steps, each counted run
    between two copies of known size (COPY_BYTES read and written: the counters' calibration and the markers).
    Per step the dispatches come in a fixed order: per layer its difference kernel then its convolution kernel,
    and last the nonlinearity of conv5 (dense path: the nonlinearity after every layer)."""
    import torch
    st = Stack(args.streams, fuse=not args.no_fuse)
    if args.conv_kernel:
        for L in st.layers:
            try:
                L.set_option("conv_kernel", args.conv_kernel)
            except Exception:
                pass
            L.reset()
    calibration_copy(0)  # (allocates the markers' buffers)
    for path in (0, 2):
        st.set_path(path)
        st.run_steps(0, args.warmup, False)
        torch.cuda.synchronize()
        calibration_copy(1)  # (marks the boundary between warm-up and counted steps in the dispatch list)
        st.run_steps(args.warmup, args.steps, False)
        torch.cuda.synchronize()
        calibration_copy(1)
    return {"lean": True, "steps": args.steps, "warmup": args.warmup, "streams": args.streams}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=320)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--streams", type=int, default=int(os.environ.get("RRM_BENCH_STREAMS", "512")))
    ap.add_argument("--no-graph", action="store_true", help="issue every launch from Python instead of replaying a HIP graph")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--no-fuse", action="store_true",
                    help="delta path: write every layer's input to memory (separate f kernel) instead of rrm_step_from_projection")
    ap.add_argument("--conv-kernel", type=int, default=0, help="0 automatic, 1 window-tile, 2 position-gather (where eligible)")
    ap.add_argument("--sweep", action="store_true", help="full density grids of configs 2-4 into sweep.jsonl and a table")
    ap.add_argument("--no-configs", action="store_true", help="leave out the per-configuration array")
    ap.add_argument("--config-streams", type=int, default=64,
                    help="the per-configuration array times every layer at 1 stream (the configs' batch) and at this many")
    ap.add_argument("--lean", action="store_true", help="only eager steps of the headline stack (for a profiler)")
    ap.add_argument("--lean-case", default="", help="only eager steps of one layer of configs 0/2/3/4 (for a profiler), "
                    "cfg:layer:density:streams[:i8|bf16][:path=P]")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (video streams are independent and would shard without any "
              "collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.lean_case:
        print(json.dumps(run_lean_case(args)), flush=True)
        return
    if args.lean:
        print(json.dumps(run_lean(args)), flush=True)
        return
    out = run_stack(args)
    out["peaks"] = measure_peaks()
    log("[peaks]", json.dumps(out["peaks"]))
    r = out["roofline"]
    meas = out["peaks"]["copy_GBps"] if r["bound"] == "hbm" else out["peaks"]["mfma_i8_TOPs"]
    r["frac_of_measured_peak"] = round(r["achieved"] / meas, 4)
    if not args.no_configs or args.sweep:
        rows = config_rows(sorted({1, max(1, args.config_streams)}), full=args.sweep)
        out["configs"] = compact(rows)
        if args.sweep:
            write_sweep(rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
