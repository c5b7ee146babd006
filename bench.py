#!/usr/bin/env python3
"""Benchmark of the PILC entropy-coding hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: pilc_encode (mean shift,
fixed-point CDF -> (cum,freq), rANS lanes, offset scan, pack) followed by pilc_decode of the
container it produced.  Inputs are resident in HBM before the timed region starts.  Prints one
JSON line: the headline workload (--config, default 1: the CIFAR-shaped batch) with
  roofline      dominant kernel of the step: algorithmic bytes / its HIP-event duration against
                the 8 TB/s HBM peak, and `traffic` = HBM bytes of one launch read from two
                rocprofv3 --pmc child runs (FETCH_SIZE, WRITE_SIZE), each scaled by what the same
                counter reports for a plain device copy of known size in the same child run;
                `plain_copy_GBs` is a device-to-device copy timed in the same run (read + written
                bytes per second): the achievable figure beside the published peak;
  cpu_baseline  the CPU oracle timed on the host cores on a bounded prefix of the workload;
and, under other_workloads, the same three things (rates, roofline with traffic, cpu_baseline) for
every other single-GPU workload: the tiny, ImageNet64-shaped, 1080p and entropy-extreme batches
(the last at 12 and 16 bits of precision with 64 lanes per image on all 8192 images, and at 1 and
1024 lanes per image on its first 512), the paper's own table-driven coder (Sec. 3.2 Algs. 3-4) on
the recipe of its coder measurement (Sec. 4.3) and on the stream of vector indices (Sec. 3.1), the
Three-Way AR residual transform (Sec. 3.1 eqs. (2)-(4)) on three image shapes, and the coder under
a mixture of ten logistic laws (the workload Sec. 2 names).

--workload / --config / --prec-bits / --lanes-per-image / --images pick another headline;
--no-extra leaves the other workloads out.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import shutil
import signal
import subprocess
import sys
import tempfile
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
HERE = os.path.dirname(os.path.abspath(__file__))
METRIC = "compress & decompress MB/s (raw uint8) on 1 MI355X; bits/subpixel"
METRIC_ANSAI = "coder encode & decode MB/s (uint8 symbols) on 1 MI355X; bits/symbol"
METRIC_TWAR = "residual transform forward & inverse MB/s (raw uint8) on 1 MI355X"
METRIC_MIX = "compress & decompress MB/s (raw uint8) under a logistic mixture on 1 MI355X; bits/subpixel"
MIX_IMAGES = {0: 64, 2: 2048, 3: 4}   # default number of images per base config
TWAR_WEIGHTS = ([[-16384, 16384, 16384], [8192, -8192, 16384], [8192, -8192, 16384]], [0, 0, 0])


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1,
                    help="workload 0..4 of BASELINE.json (default 1: CIFAR-shaped, 50,000 images)")
    ap.add_argument("--components", type=int, default=10,
                    help="mixture components K of --workload mix (default 10, the count Sec. 2 of the "
                         "paper names)")
    ap.add_argument("--workload", choices=("pilc", "ansai", "twar", "mix"), default="pilc",
                    help="pilc: the image path on --config; ansai: the table-driven coder on pieces; "
                         "twar: the Three-Way AR residual transform on the images of --config; "
                         "mix: the coder under a mixture of --components logistic laws on the first "
                         "2048 images of config 2 (or --config 0/3, --images)")
    ap.add_argument("--prec-bits", type=int, default=None, help="M of --config 4 (12 or 16)")
    ap.add_argument("--lanes-per-image", type=int, default=None, help="lanes per image of --config 4")
    ap.add_argument("--images", type=int, default=None,
                    help="first N images (pilc) or pieces (ansai) only (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-images", type=int, default=None)
    ap.add_argument("--no-traffic", action="store_true",
                    help="skip the two rocprofv3 --pmc child runs that measure HBM traffic")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--lane-sweep", action="store_true",
                    help="instead of the benchmark: the stress workload (config 4) on 256 random + 256 "
                         "constant images over lanes per image 1..1024 and M = 12, 16, kernels chosen "
                         "automatically and, at 8..64 lanes per image, forced either way; one JSON line")
    ap.add_argument("--piece-sweep", action="store_true",
                    help="instead of the benchmark: the table-driven coder over the number of pieces "
                         "coded in parallel (the axis of the paper's Fig. 5), 64 .. 10^6 pieces of 1000 "
                         "symbols, D = 8, M = 12; one JSON line")
    ap.add_argument("--pmc-child", action="store_true",
                    help="internal: one warm-up and one step of every workload of the run, each followed "
                         "by a plain device copy; prints nothing")
    return ap.parse_args()


# ----------------------------------------------------------------------------------------------
# HBM traffic from rocprofv3 counters (child processes, started before this process touches HIP)
# ----------------------------------------------------------------------------------------------
def _run_pmc(counters: str, argv):
    """One rocprofv3 --pmc run of `bench.py --pmc-child <argv>` with the space-separated
    `counters`.  Returns the dispatches in launch order as (kernel name, {counter: value}), or None."""
    exe = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(exe):
        return None
    out_dir = tempfile.mkdtemp(prefix="pilc_pmc_", dir="/tmp")
    cmd = [exe, "--pmc"] + counters.split() + ["-d", out_dir, "-o", "pmc", "--output-format", "csv", "--",
                                               sys.executable, os.path.join(HERE, "bench.py"), "--pmc-child"] + argv
    env = dict(os.environ, TMPDIR="/tmp")
    try:
        proc = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL,
                                stderr=subprocess.DEVNULL, start_new_session=True)
        try:
            proc.wait(timeout=420)
        except subprocess.TimeoutExpired:
            os.killpg(proc.pid, signal.SIGKILL)
            proc.wait()
            return None
        if proc.returncode != 0:
            return None
        rows = {}
        for root, _, files in os.walk(out_dir):
            for f in files:
                if f.endswith("counter_collection.csv"):
                    with open(os.path.join(root, f)) as fh:
                        for r in csv.DictReader(fh):
                            d = rows.setdefault(int(r["Dispatch_Id"]), (r["Kernel_Name"].split("(")[0], {}))
                            d[1][r["Counter_Name"]] = float(r["Counter_Value"])
        return [rows[k] for k in sorted(rows)]
    except (OSError, KeyError, ValueError):
        return None
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)


COPY_KERNEL = "bitwise_not"   # the child's plain read-all-write-all pass between two workloads
PROBE_MAX_BYTES = 1 << 30     # the pass covers at most this much: one launch (torch splits an
                              # elementwise kernel beyond 2^31 elements), counters far from any limit


def probe_copy_bytes(run):
    """Bytes read (and bytes written) by the child's plain pass after `run`."""
    return float(min(int(run.probe_bytes // 2), PROBE_MAX_BYTES))


# third pass: how busy the vector ALUs were (the thread-per-lane kernels are bound by them)
VALU_COUNTERS = "SQ_INSTS_VALU SQ_ACTIVE_INST_VALU GRBM_GUI_ACTIVE"


def measure_traffic(argv, count):
    """HBM bytes per launch of the kernels of each of the `count` workloads of this run, and their
    vector-ALU counters.  The child runs the workloads in order, each followed by a plain
    copy-like pass over a buffer of known size, so those passes cut the launch sequence into one
    segment per workload.  Returns a list of {"read": {kernel: KiB of its last launch},
    "write": {...}, "read_copy_kib", "write_copy_kib", "valu": {kernel: {counter: value}}} or None."""
    out = [dict() for _ in range(count)]
    for counters, key in (("FETCH_SIZE", "read"), ("WRITE_SIZE", "write"), (VALU_COUNTERS, "valu")):
        rows = _run_pmc(counters, argv)
        if not rows:
            if key == "valu":
                break              # the traffic figures stand without it
            return None
        seg, cur = [], {}
        for name, values in rows:
            if COPY_KERNEL in name:
                seg.append((cur, values))
                cur = {}
            else:
                cur[name] = values     # a later launch of the same kernel replaces the warm-up's
        if len(seg) != count:
            if key == "valu":
                break
            return None
        for i, (kernels, copy_values) in enumerate(seg):
            if key == "valu":
                out[i][key] = kernels
            else:
                out[i][key] = {k: v[counters] for k, v in kernels.items()}
                out[i][key + "_copy_kib"] = copy_values[counters]
    return out


def _matches(kernel, name):
    # the timing name is the kernel's, or its stem (k_twar_inverse: k_twar_inverse<..>, .._tall)
    return ("::" + kernel) in name and not name.split("::" + kernel)[1][:1].isalpha()


def valu_of(kernel, seg):
    """Vector-ALU figures of the last launch of `kernel` from a segment of measure_traffic: wavefront
    instructions issued, and the share of the chip's issue slots they took (an instruction
    occupies a SIMD for 4 cycles; 1024 SIMDs; GRBM_GUI_ACTIVE sums the busy cycles of the 8 XCDs)."""
    if not seg or "valu" not in seg:
        return None
    vals = [v for name, v in seg["valu"].items() if _matches(kernel, name)]
    if not vals or not vals[-1].get("GRBM_GUI_ACTIVE"):
        return None
    v = vals[-1]
    return {"wavefront_instructions": v.get("SQ_INSTS_VALU"),
            "issue_frac": 4.0 * v.get("SQ_ACTIVE_INST_VALU", 0.0) / (1024.0 * v["GRBM_GUI_ACTIVE"] / 8.0),
            "peak_wavefront_instructions_per_s": 256 * 4 * 2.4e9 / 4}


def traffic_of(kernel, seg, copy_bytes):
    """(bytes, detail) of one launch of `kernel` from a segment of measure_traffic: counter value x
    1024 x scale, scale = known bytes of the plain copy / what the counter read for that copy."""
    if not seg:
        return None, None
    detail = {}
    for key in ("read", "write"):
        if not seg.get(key + "_copy_kib"):
            return None, None
        scale = copy_bytes / (seg[key + "_copy_kib"] * 1024.0)
        vals = [v for name, v in seg[key].items() if _matches(kernel, name)]
        if not vals:
            return None, None
        detail[key + "_bytes"] = vals[-1] * 1024.0 * scale
        detail[key + "_scale"] = scale
    return detail["read_bytes"] + detail["write_bytes"], detail


# ----------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands
# ----------------------------------------------------------------------------------------------
def cpu_baseline(wl, sample_images):
    from oracle import pilc_oracle as orc

    n, h, w, m, mode, la, lb = wl.geom
    hw = h * w
    unit = max(1, la // hw) if mode == 0 else 1          # images per lane-aligned slab unit
    k = max(unit, (min(sample_images, n) // unit) * unit)
    cores = max(1, min(16, os.cpu_count() or 1))
    per = -(-(k // unit) // cores) * unit
    slabs = [(a, min(a + per, k)) for a in range(0, k, per)]

    def prep(a, b):
        sl = slice(a, b)
        g = orc.make_geom(b - a, h, w, m, mode, la, lb)
        return g, wl.img[sl].copy(), wl.mu[sl].copy(), wl.log_scale[sl].copy(), wl.chan_coef[sl].copy()

    jobs = [prep(a, b) for a, b in slabs]
    orc.lib()

    def enc(job):
        rc, coded = orc.encode(*job)
        assert rc == orc.OK
        return coded

    def dec(args):
        job, coded = args
        rc, img = orc.decode(job[0], coded, job[2], job[3], job[4])
        assert rc == orc.OK and np.array_equal(img, job[1])

    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        t0 = time.perf_counter()
        coded = list(pool.map(enc, jobs))
        t1 = time.perf_counter()
        list(pool.map(dec, zip(jobs, coded)))
        t2 = time.perf_counter()
    raw_mb = k * hw * 3 / 1e6
    j0 = jobs[0]  # one core, on the first slab only
    t3 = time.perf_counter()
    c0 = enc(j0)
    t4 = time.perf_counter()
    dec((j0, c0))
    t5 = time.perf_counter()
    mb0 = (slabs[0][1] - slabs[0][0]) * hw * 3 / 1e6
    return {
        "value": raw_mb / (t2 - t0), "unit": "MB/s", "cores": len(jobs), "kind": "oracle",
        "sample": "first %d images of the workload (%.1f MB raw), encode+decode, %d slabs in a thread pool"
                  % (k, raw_mb, len(jobs)),
        "compress_MB_s": raw_mb / (t1 - t0), "decompress_MB_s": raw_mb / (t2 - t1),
        "one_core": {"value": mb0 / (t5 - t3), "compress_MB_s": mb0 / (t4 - t3),
                     "decompress_MB_s": mb0 / (t5 - t4), "sample_MB": mb0},
    }


# ----------------------------------------------------------------------------------------------
# One workload on the GPU
# ----------------------------------------------------------------------------------------------
class Run:
    def __init__(self, config, images, prec_bits=None, lanes_per_image=None, workload=None):
        import torch
        from paper_2206_05279_amd import binding as pb
        from paper_2206_05279_amd import synth

        self.torch, self.pb = torch, pb
        dev = torch.device("cuda:0")
        t = time.perf_counter()
        if workload is not None:
            wl = workload          # arrays shared with another run of the same data
        elif config == 4:
            wl = synth.make_workload(4, images, prec_bits=prec_bits or 12, lanes_per_image=lanes_per_image or 64)
        else:
            wl = synth.make_workload(config, images)
        self.wl = wl
        self.config = config
        self.gen_s = time.perf_counter() - t
        self.geom = pb.make_geom(*wl.geom)
        self.img = torch.from_numpy(wl.img).to(dev)
        self.mu = torch.from_numpy(wl.mu).to(dev)
        self.ls = torch.from_numpy(wl.log_scale).to(dev)
        self.coef = torch.from_numpy(wl.chan_coef).to(dev)
        ws_bytes, max_coded = pb.pilc_workspace_size(self.geom)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.empty(max_coded, dtype=torch.uint8, device=dev)
        self.out = torch.empty_like(self.img)
        self.name = "cfg%d %s: %d x %dx%dx3 uint8, M=%d, %d lanes" % (
            config, wl.name, wl.n, wl.h, wl.w, wl.prec_bits, pb.pilc_lane_count(self.geom))
        self.raw = wl.subpixels
        self.probe_src = self.mu           # plain copy of known size: 2 bytes per subpixel
        self.probe_bytes = 4.0 * wl.subpixels
        self.step = "pilc_encode + pilc_decode of the whole batch"
        self.cpu_sample = {0: 64, 1: 21504, 2: 5376, 3: 10, 4: 336}[config]

    def cpu(self, scale=1.0):
        return cpu_baseline(self.wl, max(1, int(self.cpu_sample * scale)))

    def algo_bytes(self, nbytes):
        # either lane kernel: 1 B pixel + 2 B mu + 2 B log-scale per subpixel, plus the container
        return 5.0 * self.raw + nbytes

    def reference(self):
        return self.img

    def encode(self):
        return self.pb.pilc_encode(self.geom, self.img, self.mu, self.ls, self.coef, self.workspace,
                                   self.coded)[1]

    def decode(self, nbytes):
        self.pb.pilc_decode(self.geom, self.coded, nbytes, self.mu, self.ls, self.coef,
                            self.workspace, self.out)

    def timed(self, steps, warmup):
        torch, pb = self.torch, self.pb
        for _ in range(warmup):
            self.decode(self.encode())
        torch.cuda.synchronize()
        # timed region: exactly `steps` steps; per-kernel HIP events are recorded inside the
        # library on the stream the kernels are launched on
        pb.pilc_set_timing(True)
        kernel_ms, enc_ms, dec_ms = {}, 0.0, 0.0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            nbytes = self.encode()
            te = pb.pilc_last_timing()
            self.decode(nbytes)
            td = pb.pilc_last_timing()
            enc_ms += te[0][1]
            dec_ms += td[0][1]
            for name, ms in te[1:] + td[1:]:
                kernel_ms[name] = kernel_ms.get(name, 0.0) + ms
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        pb.pilc_set_timing(False)
        raw = self.raw
        return {
            "elapsed": elapsed, "nbytes": int(nbytes), "raw": raw,
            "kernel_ms": {k: v / steps for k, v in kernel_ms.items()},
            "compress_MB_s": raw / 1e6 / (enc_ms / steps * 1e-3),
            "decompress_MB_s": raw / 1e6 / (dec_ms / steps * 1e-3),
            "ok": bool(torch.equal(self.out, self.reference())),
        }


# ----------------------------------------------------------------------------------------------
# The table-driven coder on pieces
# ----------------------------------------------------------------------------------------------
def cpu_baseline_pieces(wl, sample_pieces):
    from oracle import ansai_oracle as ao

    k = min(sample_pieces, wl.pieces)
    cores = max(1, min(16, os.cpu_count() or 1))
    per = -(-k // cores)
    slabs = [(a, min(a + per, k)) for a in range(0, k, per)]
    jobs = [(np.ascontiguousarray(wl.sym[a:b]), np.ascontiguousarray(wl.dist[a:b])) for a, b in slabs]
    ao.lib()

    def enc(job):
        rc, coded = ao.encode(wl.prec_bits, wl.mass, job[0], job[1])
        assert rc == ao.OK
        return coded

    def dec(args):
        job, coded = args
        rc, sym = ao.decode(wl.prec_bits, wl.mass, job[1], coded)
        assert rc == ao.OK and np.array_equal(sym, job[0])

    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        t0 = time.perf_counter()
        coded = list(pool.map(enc, jobs))
        t1 = time.perf_counter()
        list(pool.map(dec, zip(jobs, coded)))
        t2 = time.perf_counter()
    raw_mb = k * wl.count / 1e6
    t3 = time.perf_counter()
    c0 = enc(jobs[0])
    t4 = time.perf_counter()
    dec((jobs[0], c0))
    t5 = time.perf_counter()
    mb0 = jobs[0][0].size / 1e6
    return {
        "value": raw_mb / (t2 - t0), "unit": "MB/s", "cores": len(jobs), "kind": "oracle",
        "sample": "first %d pieces of the workload (%.1f MB of symbols), encode+decode with the tables of "
                  "Algs. 3-4, %d slabs in a thread pool" % (k, raw_mb, len(jobs)),
        "compress_MB_s": raw_mb / (t1 - t0), "decompress_MB_s": raw_mb / (t2 - t1),
        "one_core": {"value": mb0 / (t5 - t3), "compress_MB_s": mb0 / (t4 - t3),
                     "decompress_MB_s": mb0 / (t5 - t4), "sample_MB": mb0},
    }


class PieceRun:
    """pilc_ansai_encode + pilc_ansai_decode of the whole batch; tables built once, outside."""

    def __init__(self, config, pieces):
        import torch
        from paper_2206_05279_amd import binding as pb
        from paper_2206_05279_amd import synth_pieces

        self.torch, self.pb = torch, pb
        dev = torch.device("cuda:0")
        t = time.perf_counter()
        self.wl = wl = synth_pieces.make_piece_workload(config, pieces, threads=16)
        self.gen_s = time.perf_counter() - t
        d, x = wl.mass.shape
        self.shape = pb.make_ansai_shape(wl.pieces, wl.count, wl.prec_bits, d, x)
        self.sym = torch.from_numpy(wl.sym).to(dev)
        self.dist = torch.from_numpy(wl.dist).to(dev)
        mass = torch.from_numpy(wl.mass).to(dev)
        self.tables = torch.empty(pb.pilc_ansai_table_bytes(wl.prec_bits, d, x), dtype=torch.uint8, device=dev)
        pb.pilc_ansai_build_tables(wl.prec_bits, d, x, mass, self.tables)
        ws_bytes, max_coded = pb.pilc_ansai_workspace_size(self.shape)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.empty(max_coded, dtype=torch.uint8, device=dev)
        self.out = torch.empty_like(self.sym)
        self.name = "table-driven coder (Sec. 3.2 Algs. 3-4): %s, %d symbols, X=%d" % (wl.name, wl.symbols, x)
        self.bits_key = "bits_per_symbol"
        self.raw = wl.symbols
        self.probe_src = self.sym          # plain copy of known size: 1 byte per symbol
        self.probe_bytes = 2.0 * wl.symbols
        self.step = "pilc_ansai_encode + pilc_ansai_decode of the whole batch"
        self.cpu_sample = 131072 * 1000 // wl.count

    def cpu(self, scale=1.0):
        return cpu_baseline_pieces(self.wl, max(64, int(self.cpu_sample * scale)))

    def algo_bytes(self, nbytes):
        # either coder kernel: symbols and distribution indices (1 byte each) plus the coded words
        return 2.0 * self.raw + nbytes

    def encode(self):
        return self.pb.pilc_ansai_encode(self.shape, self.sym, self.dist, self.tables, self.workspace,
                                         self.coded)[1]

    def decode(self, nbytes):
        self.pb.pilc_ansai_decode(self.shape, self.coded, nbytes, self.dist, self.tables, self.workspace,
                                  self.out)

    def reference(self):
        return self.sym

    timed = Run.timed


def cpu_baseline_twar(img, sample_images):
    from oracle import twar_oracle as to

    k = min(sample_images, img.shape[0])
    cores = max(1, min(16, os.cpu_count() or 1))
    per = -(-k // cores)
    jobs = [np.ascontiguousarray(img[a:min(a + per, k)]) for a in range(0, k, per)]
    p = to.make_params(*TWAR_WEIGHTS)
    to.lib()

    def both(x):
        r = to.forward(p, x)
        assert np.array_equal(to.inverse(p, r), x)

    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        t0 = time.perf_counter()
        list(pool.map(both, jobs))
        t1 = time.perf_counter()
    raw_mb = img[:k].size / 1e6
    t2 = time.perf_counter()
    both(jobs[0])
    t3 = time.perf_counter()
    return {"value": raw_mb / (t1 - t0), "unit": "MB/s", "cores": len(jobs), "kind": "oracle",
            "sample": "first %d images (%.1f MB), forward + inverse, %d slabs in a thread pool" % (k, raw_mb, len(jobs)),
            "one_core": {"value": jobs[0].size / 1e6 / (t3 - t2), "sample_MB": jobs[0].size / 1e6}}


class TwarRun:
    """pilc_twar_forward + pilc_twar_inverse over the images of a workload (Sec. 3.1 eqs. (2)-(4))."""

    def __init__(self, config, images):
        import torch
        from paper_2206_05279_amd import binding as pb
        from paper_2206_05279_amd import synth

        self.torch, self.pb = torch, pb
        t = time.perf_counter()
        wl = synth.make_workload(config, images)
        self.gen_s = time.perf_counter() - t
        self.img_np = wl.img
        self.img = torch.from_numpy(wl.img).to("cuda:0")
        self.res = torch.empty_like(self.img)
        self.out = torch.empty_like(self.img)
        self.params = pb.make_twar_params(*TWAR_WEIGHTS)
        self.name = "Three-Way AR transform (Sec. 3.1 eqs. 2-4): cfg%d %s images: %d x %dx%dx3 uint8" % (
            config, wl.name, wl.n, wl.h, wl.w)
        self.raw = wl.subpixels
        self.probe_src = self.img
        self.probe_bytes = 2.0 * wl.subpixels
        self.step = "pilc_twar_forward + pilc_twar_inverse of the whole batch"
        self.cpu_sample = max(1, 61440000 // (wl.h * wl.w * 3))     # about 60 MB of images

    def cpu(self, scale=1.0):
        return cpu_baseline_twar(self.img_np, max(1, int(self.cpu_sample * scale)))

    def algo_bytes(self, nbytes):
        return 2.0 * self.raw  # either kernel reads and writes every subpixel once

    def encode(self):
        self.pb.pilc_twar_forward(self.params, self.img, self.res)
        return self.raw

    def decode(self, nbytes):
        self.pb.pilc_twar_inverse(self.params, self.res, self.out)

    def reference(self):
        return self.img

    timed = Run.timed


def cpu_baseline_mix(wl, sample_images):
    from oracle import mix_oracle as mx
    from oracle import pilc_oracle as orc

    n, h, w, m, mode, la, lb = wl.geom
    k = max(1, min(sample_images, n))
    cores = max(1, min(16, os.cpu_count() or 1))
    per = -(-k // cores)
    slabs = [(a, min(a + per, k)) for a in range(0, k, per)]   # lanes never span images here

    def prep(a, b):
        sl = slice(a, b)
        return (orc.make_geom(b - a, h, w, m, mode, la, lb), wl.img[sl].copy(), wl.mu[sl].copy(),
                wl.log_scale[sl].copy(), wl.weight[sl].copy(), wl.chan_coef[sl].copy())

    jobs = [prep(a, b) for a, b in slabs]
    mx.lib()

    def enc(job):
        rc, coded = mx.encode(job[0], wl.num_comp, *job[1:])
        assert rc == mx.OK
        return coded

    def dec(args):
        job, coded = args
        rc, img = mx.decode(job[0], wl.num_comp, coded, *job[2:])
        assert rc == mx.OK and np.array_equal(img, job[1])

    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        t0 = time.perf_counter()
        coded = list(pool.map(enc, jobs))
        t1 = time.perf_counter()
        list(pool.map(dec, zip(jobs, coded)))
        t2 = time.perf_counter()
    raw_mb = k * h * w * 3 / 1e6
    t3 = time.perf_counter()
    c0 = enc(jobs[0])
    t4 = time.perf_counter()
    dec((jobs[0], c0))
    t5 = time.perf_counter()
    mb0 = jobs[0][1].size / 1e6
    return {
        "value": raw_mb / (t2 - t0), "unit": "MB/s", "cores": len(jobs), "kind": "oracle",
        "sample": "first %d images of the workload (%.2f MB raw), encode+decode, %d slabs in a thread pool"
                  % (k, raw_mb, len(jobs)),
        "compress_MB_s": raw_mb / (t1 - t0), "decompress_MB_s": raw_mb / (t2 - t1),
        "one_core": {"value": mb0 / (t5 - t3), "compress_MB_s": mb0 / (t4 - t3),
                     "decompress_MB_s": mb0 / (t5 - t4), "sample_MB": mb0},
    }


class MixRun:
    """pilc_mix_encode + pilc_mix_decode: the lanes of a base config under K logistic laws per subpixel."""

    def __init__(self, config, images, components):
        import torch
        from paper_2206_05279_amd import binding as pb
        from paper_2206_05279_amd import synth_mix

        self.torch, self.pb = torch, pb
        dev = torch.device("cuda:0")
        config = config if config in MIX_IMAGES else 2
        t = time.perf_counter()
        self.wl = wl = synth_mix.make_mix_workload(config, images or MIX_IMAGES[config], components)
        self.gen_s = time.perf_counter() - t
        self.k = wl.num_comp
        self.geom = pb.make_geom(*wl.geom)
        self.img = torch.from_numpy(wl.img).to(dev)
        self.mu = torch.from_numpy(wl.mu).to(dev)
        self.ls = torch.from_numpy(wl.log_scale).to(dev)
        self.weight = torch.from_numpy(wl.weight).to(dev)
        self.coef = torch.from_numpy(wl.chan_coef).to(dev)
        ws_bytes, max_coded = pb.pilc_workspace_size(self.geom)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.empty(max_coded, dtype=torch.uint8, device=dev)
        self.out = torch.empty_like(self.img)
        self.name = "mixture of logistic laws (Sec. 2): cfg%d %s: %d x %dx%dx3 uint8, K=%d, M=%d, %d lanes" % (
            config, wl.name, wl.n, wl.h, wl.w, self.k, wl.prec_bits, pb.pilc_lane_count(self.geom))
        self.raw = wl.subpixels
        self.probe_src = self.img
        self.probe_bytes = 2.0 * wl.subpixels
        self.step = "pilc_mix_encode + pilc_mix_decode of the whole batch"
        self.cpu_sample = 1024

    def cpu(self, scale=1.0):
        return cpu_baseline_mix(self.wl, max(1, int(self.cpu_sample * scale)))

    def algo_bytes(self, nbytes):
        # either lane kernel: per subpixel 1 B pixel, 2 K B means, 2 K B log-scales and a third of the
        # pixel's 2 K B of weights, plus the container
        return (1.0 + 4.0 * self.k + 2.0 * self.k / 3.0) * self.raw + nbytes

    def reference(self):
        return self.img

    def encode(self):
        return self.pb.pilc_mix_encode(self.geom, self.k, self.img, self.mu, self.ls, self.weight, self.coef,
                                       self.workspace, self.coded)[1]

    def decode(self, nbytes):
        self.pb.pilc_mix_decode(self.geom, self.k, self.coded, nbytes, self.mu, self.ls, self.weight,
                                self.coef, self.workspace, self.out)

    timed = Run.timed


def video_margin(r, frames):
    """Decode and encode time per 1920x1080 frame against the 33.3 ms a 30 frames/s stream allows
    (the paper's requirement of 187 MB/s for 1080p30, Sec. 1)."""
    raw_mb = r["raw"] / 1e6
    dec_ms = raw_mb / r["decompress_MB_s"] * 1e3 / frames
    enc_ms = raw_mb / r["compress_MB_s"] * 1e3 / frames
    return {"decode_ms_per_frame": dec_ms, "encode_ms_per_frame": enc_ms, "budget_ms_per_frame": 1000.0 / 30.0,
            "required_MB_s": 1920 * 1080 * 3 * 30 / 1e6}


def copy_bandwidth(torch, src, reps=10):
    """GB/s (bytes read plus bytes written) of a plain device-to-device copy of `src`: what a
    streaming kernel can reach on this GPU, to set beside the 8 TB/s peak."""
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * src.numel() * src.element_size() * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def headline_run(args):
    if args.workload == "mix":
        return MixRun(args.config, args.images, args.components)
    if args.workload == "ansai":
        return PieceRun(args.config if args.config in (0, 1, 2) else 1, args.images)
    if args.workload == "twar":
        return TwarRun(args.config, args.images)
    return Run(args.config, args.images, args.prec_bits, args.lanes_per_image)


def other_runs(args):
    """The other workloads of the default run, as (label, factory) in the order they are run; a
    factory may return several runs that share their input arrays."""
    import dataclasses

    def stress():
        from paper_2206_05279_amd import synth
        full = synth.make_workload(4, None, prec_bits=12, lanes_per_image=64)
        px = full.h * full.w
        yield Run(4, None, workload=full)
        yield Run(4, None, workload=dataclasses.replace(full, prec_bits=16, name="entropy-extreme-M16-L64"))
        half = full.n // 2
        pick = np.r_[0:256, half:half + 256]     # 256 random and 256 constant images
        sub = dataclasses.replace(full, n=512, img=np.ascontiguousarray(full.img[pick]),
                                  mu=np.ascontiguousarray(full.mu[pick]),
                                  log_scale=np.ascontiguousarray(full.log_scale[pick]),
                                  chan_coef=np.ascontiguousarray(full.chan_coef[pick]))
        del full
        yield Run(4, None, workload=dataclasses.replace(sub, lane_a=px, name="entropy-extreme-M12-L1 (512 images)"))
        yield Run(4, None, workload=dataclasses.replace(sub, lane_a=px // 1024,
                                                        name="entropy-extreme-M12-L1024 (512 images)"))

    plan = [(lambda c=c: [Run(c, None)]) for c in (0, 2, 3) if not (args.workload == "pilc" and args.config == c)]
    if not (args.workload == "pilc" and args.config == 1):
        plan.insert(1, lambda: [Run(1, None)])
    plan += [stress,
             lambda: [PieceRun(1, None)],      # the paper's own coder variant on its coder-measurement recipe
             lambda: [PieceRun(2, None)],      # the stream of vector indices
             lambda: [TwarRun(1, None)], lambda: [TwarRun(2, None)], lambda: [TwarRun(3, None)],
             lambda: [MixRun(2, None, 10)]]    # the dynamic-coder workload Sec. 2 names as the slow case
    return plan


def report(run, r, seg, torch, with_copy=False):
    """The figures of one workload: rates, the dominant kernel against the roofline, traffic."""
    kernel_ms, nbytes = r["kernel_ms"], r["nbytes"]
    dom = max(kernel_ms, key=kernel_ms.get)
    algo = run.algo_bytes(nbytes)
    achieved = algo / (kernel_ms[dom] * 1e-3) / 1e9
    traffic, detail = traffic_of(dom, seg, probe_copy_bytes(run))
    twar = isinstance(run, TwarRun)
    out = {
        "step": run.step,
        ("forward_MB_s" if twar else "compress_MB_s"): r["compress_MB_s"],
        ("inverse_MB_s" if twar else "decompress_MB_s"): r["decompress_MB_s"],
        "round_trip_exact": r["ok"],
        "kernel_ms": kernel_ms,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_detail": detail,
                     "algorithmic_bytes": algo, "avg_ms": kernel_ms[dom], "valu": valu_of(dom, seg),
                     "calibration_copy_bytes": probe_copy_bytes(run)},
    }
    if not twar:
        out[getattr(run, "bits_key", "bits_per_subpixel")] = 8.0 * nbytes / r["raw"]
        out["coded_bytes"] = nbytes
    if with_copy:
        out["roofline"]["plain_copy_GBs"] = copy_bandwidth(torch, run.probe_src)
    if isinstance(run, Run) and run.config == 3:
        out["video_1080p30"] = video_margin(r, run.wl.n)
    return out


def lane_sweep():
    """The stress workload over lanes per image: whole pilc_encode / pilc_decode calls, mean of
    three after a warm-up, round trip checked in every row."""
    import dataclasses
    import torch
    from paper_2206_05279_amd import binding as pb
    from paper_2206_05279_amd import synth

    wl = synth.make_workload(4, 512, prec_bits=12, lanes_per_image=64)
    dev = torch.device("cuda:0")
    img, mu, ls, coef = (torch.from_numpy(a).to(dev) for a in (wl.img, wl.mu, wl.log_scale, wl.chan_coef))
    out = torch.empty_like(img)
    px = wl.h * wl.w
    rows = []

    def one(m, per_image, policy):
        pb.pilc_set_kernel_policy(policy)
        geom = pb.make_geom(wl.n, wl.h, wl.w, m, 0, px // per_image, 0)
        ws, mc = pb.pilc_workspace_size(geom)
        work = torch.empty(ws, dtype=torch.uint8, device=dev)
        coded = torch.empty(mc, dtype=torch.uint8, device=dev)
        pb.pilc_set_timing(True)
        enc, dec, nb, te, td = [], [], 0, None, None
        for it in range(4):
            _, nb = pb.pilc_encode(geom, img, mu, ls, coef, work, coded)
            te = pb.pilc_last_timing()
            pb.pilc_decode(geom, coded, nb, mu, ls, coef, work, out)
            td = pb.pilc_last_timing()
            if it:
                enc.append(te[0][1])
                dec.append(td[0][1])
        raw = float(wl.subpixels)
        rows.append({"M": m, "lanes_per_image": per_image, "lanes": wl.n * per_image,
                     "policy": {0: "automatic", 1: "thread per lane", 2: "few-lane kernels"}[policy],
                     "encode_kernel": te[1][0], "decode_kernel": td[-1][0],
                     "encode_ms": float(np.mean(enc)), "decode_ms": float(np.mean(dec)),
                     "compress_GB_s": raw / np.mean(enc) / 1e6, "decompress_GB_s": raw / np.mean(dec) / 1e6,
                     "bits_per_subpixel": 8.0 * nb / raw, "round_trip_exact": bool(torch.equal(out, img))})

    try:
        for per_image in (1, 2, 4, 8, 16, 32, 64, 256, 1024):
            one(12, per_image, 0)
        for per_image in (1, 64, 1024):
            one(16, per_image, 0)
        for per_image in (8, 16, 32, 64):
            one(12, per_image, 1)
            one(12, per_image, 2)
    finally:
        pb.pilc_set_kernel_policy(0)
    print(json.dumps({"workload": "cfg4 entropy extremes, 256 random + 256 constant images of 256x256x3 "
                                  "(%.1f MB raw)" % (wl.subpixels / 1e6), "rows": rows}))
    if not all(r["round_trip_exact"] for r in rows):
        sys.exit(4)


def piece_sweep():
    """The table-driven coder over the number of pieces in flight (one thread each): whole
    pilc_ansai_encode / pilc_ansai_decode calls, mean of three after a warm-up, round trip
    checked in every row.  The recipe is that of the paper's Fig. 5 (Sec. 4.3)."""
    import torch
    from paper_2206_05279_amd import binding as pb
    from paper_2206_05279_amd import synth_pieces

    wl = synth_pieces.make_piece_workload(1, 1_000_000, threads=16)
    dev = torch.device("cuda:0")
    d, x = wl.mass.shape
    sym_all, dist_all = torch.from_numpy(wl.sym).to(dev), torch.from_numpy(wl.dist).to(dev)
    tables = torch.empty(pb.pilc_ansai_table_bytes(wl.prec_bits, d, x), dtype=torch.uint8, device=dev)
    pb.pilc_ansai_build_tables(wl.prec_bits, d, x, torch.from_numpy(wl.mass).to(dev), tables)
    pb.pilc_set_timing(True)
    rows = []
    for pieces in (64, 256, 1024, 4096, 16384, 65536, 262144, 1_000_000):
        shape = pb.make_ansai_shape(pieces, wl.count, wl.prec_bits, d, x)
        sym, dist = sym_all[:pieces].contiguous(), dist_all[:pieces].contiguous()
        ws, mc = pb.pilc_ansai_workspace_size(shape)
        work = torch.empty(ws, dtype=torch.uint8, device=dev)
        coded = torch.empty(mc, dtype=torch.uint8, device=dev)
        out = torch.empty_like(sym)
        enc, dec, nb = [], [], 0
        for it in range(4):
            nb = pb.pilc_ansai_encode(shape, sym, dist, tables, work, coded)[1]
            te = pb.pilc_last_timing()
            pb.pilc_ansai_decode(shape, coded, nb, dist, tables, work, out)
            td = pb.pilc_last_timing()
            if it:
                enc.append(te[0][1])
                dec.append(td[0][1])
        raw = float(pieces) * wl.count
        rows.append({"pieces": pieces, "wavefronts": (pieces + 63) // 64,
                     "encode_ms": float(np.mean(enc)), "decode_ms": float(np.mean(dec)),
                     "encode_MB_s": raw / np.mean(enc) / 1e3, "decode_MB_s": raw / np.mean(dec) / 1e3,
                     "bits_per_symbol": 8.0 * nb / raw, "round_trip_exact": bool(torch.equal(out, sym))})
        del work, coded, out
    print(json.dumps({"workload": "table-driven coder, pieces of %d symbols, D = %d, X = %d, M = %d"
                                  % (wl.count, d, x, wl.prec_bits), "rows": rows}))
    if not all(r["round_trip_exact"] for r in rows):
        sys.exit(4)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU runs are not "
              "part of it", file=sys.stderr)
        sys.exit(2)
    if args.lane_sweep:
        lane_sweep()
        return
    if args.piece_sweep:
        piece_sweep()
        return
    extras = not args.no_extra and args.images is None

    # children first: this process has not initialised HIP yet
    child_argv = ["--config", str(args.config), "--workload", args.workload, "--components", str(args.components)]
    for flag, val in (("--images", args.images), ("--prec-bits", args.prec_bits),
                      ("--lanes-per-image", args.lanes_per_image)):
        if val is not None:
            child_argv += [flag, str(val)]
    if not extras:
        child_argv.append("--no-extra")

    import torch
    from paper_2206_05279_amd import binding as pb

    def all_runs():
        yield headline_run(args)
        if extras:
            for factory in other_runs(args):
                for run in factory():
                    yield run
                torch.cuda.empty_cache()

    if args.pmc_child:
        if not torch.cuda.is_available():
            sys.exit(3)
        pb.lib()
        for run in all_runs():
            run.timed(1, 1)
            # a plain pass over a buffer of known size (every byte read once and written once) under
            # a kernel name nothing else here uses: it ends the workload's segment and calibrates
            src = run.probe_src.view(torch.uint8).reshape(-1)[:int(probe_copy_bytes(run))]
            probe = torch.empty_like(src)
            torch.bitwise_not(src, out=probe)
            torch.cuda.synchronize()
            del probe, src, run
        return

    traffic = None
    if not args.no_traffic:
        # the number of workloads is known without building them: 1 + what other_runs yields
        count = 1 + ((len(other_runs(args)) - 1 + 4) if extras else 0)
        traffic = measure_traffic(child_argv, count)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    pb.lib()

    result, others, ok = None, {}, True
    for i, run in enumerate(all_runs()):
        seg = traffic[i] if traffic else None
        if i == 0:
            r = run.timed(args.steps, args.warmup)
            rep = report(run, r, seg, torch, with_copy=True)
            result = {
                "metric": {PieceRun: METRIC_ANSAI, TwarRun: METRIC_TWAR, MixRun: METRIC_MIX}.get(type(run), METRIC),
                "value": r["raw"] / 1e6 / (r["elapsed"] / args.steps),
                "unit": "MB/s",
                "n_gpus": 1,
                "steps": args.steps,
                "warmup": args.warmup,
                "ms_per_step": 1e3 * r["elapsed"] / args.steps,
                "higher_is_better": True,
                "scaling": "weak",
                "vs_baseline": None,
                "dtype": "u32",
                "data": "synthetic",
                "config": {"workload": run.name, "step": run.step},
            }
            rep.pop("step")
            result.update(rep)
            result["paper_context"] = ("PILC reports about 200 MB/s end to end and 675/672 MB/s for its coder "
                                       "phases on one V100 (table-driven coder; Tab. 5 of the paper, another "
                                       "machine and workload: context, not a baseline)")
            result["input_generation_s"] = run.gen_s
            if not args.no_cpu_baseline:
                if args.cpu_sample_images:
                    run.cpu_sample = args.cpu_sample_images
                result["cpu_baseline"] = run.cpu()
        else:
            # (two warm-up steps: the GPU has idled while the oracle was timed on the host)
            other_steps = max(5, args.steps // 2)
            r = run.timed(other_steps, 2)
            rep = report(run, r, seg, torch)
            rep["value"] = r["raw"] / 1e6 / (r["elapsed"] / other_steps)
            rep["unit"] = "MB/s"
            if not args.no_cpu_baseline:
                rep["cpu_baseline"] = run.cpu(0.35)
            others[run.name] = rep
        ok = ok and r["ok"]
        del run
    if others:
        result["other_workloads"] = others
    print(json.dumps(result))
    if not ok:
        sys.exit(4)


if __name__ == "__main__":
    main()
