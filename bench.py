#!/usr/bin/env python3
"""Benchmark of the resharding hot path on one MI355X.

A step is one whole reconfiguration of the workload's job state: tpx_plan (host: split / re-partition /
merge into a copy list with its tiling), the upload of the plan tables, and tpx_execute (one kernel
launch that moves all state).  Source and destination rank buffers are resident in HBM before the timed
region.  Steps run back to back, so the host planning of one step overlaps the kernel of the previous
one; the latency of a single isolated reconfiguration is reported separately.

Prints one JSON line.  `value` is state bytes read + written per second of step time; `roofline`
describes the copy kernel alone, timed with HIP events on the launch stream (`traffic` comes from the
counter record under profiles/ and is null unless that record was taken on the present library sources and
plan); `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

GPT_STATE = (2, 4, 4, 4)
_TINY = dict(n_layers=2, hidden=256, n_heads=4, ffn=1024, vocab_true=1024, max_pos=1024, state_elem_bytes=(4, 4, 4))
_G13 = dict(n_layers=24, hidden=2048, n_heads=16, ffn=8192, vocab_true=50304, state_elem_bytes=GPT_STATE)
_G27 = dict(n_layers=32, hidden=2560, n_heads=32, ffn=10240, vocab_true=50304, state_elem_bytes=GPT_STATE)
_G67 = dict(n_layers=32, hidden=4096, n_heads=32, ffn=16384, vocab_true=50304, state_elem_bytes=GPT_STATE)
_ODD = dict(n_layers=24, hidden=3072, n_heads=24, ffn=12288, vocab_true=50257, vocab_divisor=128, state_elem_bytes=GPT_STATE)
_BERT = dict(n_layers=24, hidden=1024, n_heads=16, ffn=4096, vocab_true=30522, vocab_divisor=128, max_pos=512,
             state_elem_bytes=GPT_STATE)


def _c(T, P, D, **kw):
    return dict(T=T, P=P, D=D, **kw)


WORKLOADS = {
    # the five workloads of the benchmark spec: name -> (model kwargs, src, dst, synth mix name, seed)
    "tiny_2L_h256_(2,1,1)->(4,2,1)": (_TINY, _c(2, 1, 1), _c(4, 2, 1), "tiny", 1),
    "gpt1.3b_(4,2,1)->(2,4,1)": (_G13, _c(4, 2, 1), _c(2, 4, 1), "gpt", 2),
    "gpt2.7b_(4,4,2)->(2,4,1)": (_G27, _c(4, 4, 2), _c(2, 4, 1, stage_first_layer=(0, 7, 16, 25, 32)), "gpt", 3),
    "gpt6.7b_(8,1,1)->(1,8,1)": (_G67, _c(8, 1, 1), _c(1, 8, 1), "gpt", 4),
    "gpt_h3072_T3->T4_padded_vocab": (_ODD, _c(3, 1, 1), _c(4, 1, 1), "gpt", 5),
}
# the paper's own reconfigurations (sections 6.2, 6.3, 6.6, 6.8) at the same shapes
PAPER_PAIRS = {}
for _n, _m in (("gpt1.3b", _G13), ("gpt2.7b", _G27), ("gpt6.7b", _G67)):
    if _n != "gpt6.7b":        # 94 GB source + 188 GB destination does not fit one GPU
        PAPER_PAIRS[f"{_n}_(4,2,1)->(4,2,2)_dp"] = (_m, _c(4, 2, 1), _c(4, 2, 2), "gpt", 11)
    PAPER_PAIRS[f"{_n}_(4,2,1)->(4,4,1)_pp"] = (_m, _c(4, 2, 1), _c(4, 4, 1), "gpt", 12)
    PAPER_PAIRS[f"{_n}_(4,2,1)->(8,2,1)_tp"] = (_m, _c(4, 2, 1), _c(8, 2, 1), "gpt", 13)
    PAPER_PAIRS[f"{_n}_(4,2,1)->(4,2,1)_redeploy"] = (_m, _c(4, 2, 1), _c(4, 2, 1), "gpt", 14)
PAPER_PAIRS["gpt1.3b_(2,4,2)->(2,4,1)_elastic"] = (_G13, _c(2, 4, 2), _c(2, 4, 1), "gpt", 15)
PAPER_PAIRS["gpt1.3b_(2,4,1)->(2,2,1)_elastic"] = (_G13, _c(2, 4, 1), _c(2, 2, 1), "gpt", 16)
for _a, _b in (((1, 1, 4), (1, 1, 8)), ((1, 4, 1), (1, 8, 1)), ((4, 1, 1), (8, 1, 1))):
    PAPER_PAIRS[f"bert-large_{_a}->{_b}".replace(" ", "")] = (_BERT, _c(*_a), _c(*_b), "gpt", 17)
    PAPER_PAIRS[f"bert-large_{_b}->{_a}".replace(" ", "")] = (_BERT, _c(*_b), _c(*_a), "gpt", 18)
WORKLOADS.update(PAPER_PAIRS)
# layout-changing reshards: fused-QKV order and transposed ([in, out]) weight storage on the destination
LAYOUT_PAIRS = {
    "gpt1.3b_(4,2,1)->(2,4,1)_qkv_major_dst": (_G13, _c(4, 2, 1), _c(2, 4, 1, qkv_layout=1), "gpt", 21),
    "gpt1.3b_(4,2,1)->(2,4,1)_transposed_dst": (_G13, _c(4, 2, 1), _c(2, 4, 1, w_transposed=1), "gpt", 22),
    "gpt1.3b_(4,2,1)->(4,2,1)_transposed_dst": (_G13, _c(4, 2, 1), _c(4, 2, 1, w_transposed=1), "gpt", 23),
}
WORKLOADS.update(LAYOUT_PAIRS)
# sharded data parallelism: the fp32 optimizer state (kinds 1-3) is cut between the D replicas instead of copied
SHARDED_PAIRS = {
    "gpt2.7b_(2,2,4)->(4,2,2)_sharded_opt": (_G27, _c(2, 2, 4, shard_kinds=14), _c(4, 2, 2, shard_kinds=14), "gpt", 31),
    "gpt1.3b_(4,1,4)->(2,2,2)_sharded_opt": (_G13, _c(4, 1, 4, shard_kinds=14), _c(2, 2, 2, shard_kinds=14), "gpt", 32),
}
# interleaved (virtual) pipeline: each of 4 stages holds 2 chunks of 3 layers; folded back to 2 plain stages
SHARDED_PAIRS["gpt1.3b_(2,4,1)_interleaved->(4,2,1)"] = (_G13, _c(2, 4, 1, layer_stage=tuple((l // 3) % 4 for l in range(24))),
                                                         _c(4, 2, 1), "gpt", 33)
WORKLOADS.update(SHARDED_PAIRS)
# failure recovery (section 5.3): one replica of every (t, p) share of (4,2,2) is lost; only those eight ranks are
# rebuilt, each from its surviving replica
_LOST = [1 if (r % 4 + r // 8) % 2 == (r // 4) % 2 else 0 for r in range(16)]      # rank = t + 4*(d + 2*p)
RECOVERY = {
    "gpt2.7b_(4,2,2)_rebuild_8_lost_of_16": (_G27, _c(4, 2, 2, rank_alive=[1 - x for x in _LOST]),
                                             _c(4, 2, 2, rank_alive=_LOST), "gpt", 41),
}
WORKLOADS.update(RECOVERY)
DATASET_WORKLOAD = "dataset_1e8_D6->D4"
DATASET_CFG = dict(n_samples=10 ** 8, global_batch=768, D_src=6, D_dst=4, steps_done=65000, seed=6)
DEFAULT_WORKLOAD = "gpt6.7b_(8,1,1)->(1,8,1)"

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def source_hash() -> str:
    """Fingerprint of everything that decides what the kernel does and what a plan contains: the library's sources."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2312_05181_amd", "csrc", "*"))) + [os.path.join(ROOT, "include", "tpx.h")]
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(key: str, stats: dict):
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes recorded in profiles/hbm_traffic.json
    (counter means in KiB, each scaled by what the same counter read for a plain copy of known size in the same run),
    or None with the reason when the record was not taken on these sources and this plan."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)["workloads"].get(key)
    except (OSError, ValueError, KeyError):
        rec = None
    if rec is None:
        return None, "no counter record for this workload"
    if rec["source_hash"] != source_hash():
        return None, "the counter record was taken on other library sources"
    if rec["n_tiles"] != stats["n_tiles"] or rec["algorithmic_bytes"] != stats["bytes_read"] + stats["bytes_written"]:
        return None, "the counter record was taken on a different plan"
    traffic = int(round(1024 * (rec["fetch_size_kib"] * rec["fetch_scale"] + rec["write_size_kib"] * rec["write_scale"])))
    return traffic, rec["profile"]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS) + [DATASET_WORKLOAD])
    ap.add_argument("--cpu-layers", type=int, default=16, help="layers in the CPU oracle's sample (0 = skip)")
    ap.add_argument("--tile-bytes", type=int, default=0)
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--streams", type=int, default=0)
    ap.add_argument("--chunk", type=int, default=-1, help="executor knob: tiles an XCD takes in a row (0 = automatic)")
    ap.add_argument("--occupancy", type=int, default=-1, help="executor knob: workgroups per CU (0 = automatic)")
    ap.add_argument("--ab", default=None, metavar="CFG;CFG;...",
                    help="compare settings inside ONE process on fixed buffers (differences between processes are larger than most "
                         "effects): each CFG is a comma list of key=value with keys streams, chunk, occupancy, variant (executor "
                         "knobs), tile_bytes, max_multicast, share_reads, pack_bytes (plan options) and dst_shift_kib, rank_skew_kib (all buffers "
                         "of a side in one allocation at 2 MiB boundaries; the destination side moved by that many KiB, rank buffer r "
                         "by (r mod 8) times that many KiB); prints one JSON line")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--settle-s", type=float, default=4.0,
                    help="before the warm-up steps, keep the device under load (untimed launches of the same plan) for this many "
                         "seconds: its memory throughput steps up by about 0.8 %% after some 3.5 s of sustained load, and a "
                         "reconfiguration interrupts a job whose GPU is already under load (0 = none)")
    ap.add_argument("--share-reads", action="store_true",
                    help="plan with the share_reads option: replicas of a group are all written from one read")
    ap.add_argument("--fill", choices=["synth", "cheap"], default="synth",
                    help="source contents: seeded synthetic state, or one cheap fill per buffer (for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (all partitions of both configurations live in one "
              "GPU's HBM); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2312_05181_amd as tpx
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    if args.variant >= 0:
        tpx.tpx_set_option("variant", args.variant)
    if args.streams:
        tpx.tpx_set_option("streams", args.streams)
    if args.chunk >= 0:
        tpx.tpx_set_option("chunk", args.chunk)
    if args.occupancy >= 0:
        tpx.tpx_set_option("occupancy", args.occupancy)
    args.opts = dict(tile_bytes=args.tile_bytes, share_reads=int(args.share_reads))
    if args.ab:
        return ab_compare(args)

    if args.workload == DATASET_WORKLOAD:
        return bench_dataset(args)

    model, src, dst, mixname, seed = WORKLOADS[args.workload]
    mix = synth.MIX_TINY if mixname == "tiny" else synth.MIX_GPT
    plan = tpx.tpx_plan(model, src, dst, args.opts)
    stats = plan.stats()
    n_src, n_dst = plan.num_buffers(0), plan.num_buffers(1)

    def descs_of(side, r):
        return [synth.ShardDesc(e.tensor_id, e.kind, e.elem_bytes, e.offset, tuple(e.full_shape[:e.ndim]),
                                tuple(e.lo[:e.ndim]), tuple(e.hi[:e.ndim]), tuple(e.perm[:e.ndim]))
                for e in plan.manifest(side, r)]

    t_setup = time.time()
    src_bufs, dst_bufs = [], []
    for r in range(n_src):
        b = torch.empty(plan.buffer_bytes(0, r), dtype=torch.uint8, device="cuda")
        if args.fill == "synth":
            synth.fill_buffer(b, descs_of(0, r), seed, mix)
        else:
            b.fill_(r + 1)
        src_bufs.append(b)
    for r in range(n_dst):
        dst_bufs.append(torch.zeros(plan.buffer_bytes(1, r), dtype=torch.uint8, device="cuda"))
    two = TwoWorkspaces(plan.workspace_bytes())
    ws = two.ws[0]
    src_ptrs = [b.data_ptr() for b in src_bufs]
    dst_ptrs = [b.data_ptr() for b in dst_bufs]
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    state_bytes = stats["bytes_read"] + stats["bytes_written"]

    def step(ev0=None, ev1=None):
        p = tpx.tpx_plan(model, src, dst, args.opts)   # a1-a5: host planner
        k, w, upload_stream = two.next()
        p.prepare(w, upload_stream)                 # tile table -> HBM (waits for the copy)
        if ev0 is not None:
            ev0.record()
        p.execute(src_ptrs, dst_ptrs, w, stream)    # a6: one launch
        if ev1 is not None:
            ev1.record()
        two.used(k)
        return p

    settle(args.settle_s, lambda: plan.execute(src_ptrs, dst_ptrs, ws.data_ptr(), stream))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    plans = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        plans.append(step(*evs[i]))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = [a.elapsed_time(b) for a, b in evs]
    kernel_ms_avg = sum(kernel_ms) / len(kernel_ms)
    plan_ms = sum(p.stats()["plan_ns"] for p in plans) / len(plans) / 1e6
    del plans

    # latency of one isolated reconfiguration (nothing overlaps: plan, table upload, kernel, wait)
    lat = []
    for _ in range(5):
        torch.cuda.synchronize()
        a = time.perf_counter()
        step()
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - a) * 1e3)
    latency_ms = sorted(lat)[len(lat) // 2]

    achieved = state_bytes / (kernel_ms_avg * 1e-3) / 1e9
    traffic, traffic_from = measured_traffic(args.workload + ("|share_reads" if args.share_reads else ""), stats)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_from": traffic_from,
                "kernel": "tpx_execute_tiles", "kernel_ms_avg": round(kernel_ms_avg, 4),
                "kernel_ms_min": round(min(kernel_ms), 4), "kernel_ms_median": round(sorted(kernel_ms)[len(kernel_ms) // 2], 4),
                "algorithmic_bytes_per_launch": state_bytes}

    probe = memcpy_probe = probe_bytes = read_probe = write_probe = None
    if not args.no_probe:
        n = min(8 << 30, min(b.numel() for b in src_bufs if b.numel()) // 16 * 16, dst_bufs[0].numel() // 16 * 16)
        a, b = src_bufs[0], dst_bufs[0]
        probe_bytes = n
        for _ in range(2):
            tpx.tpx_probe_copy(b.data_ptr(), a.data_ptr(), n, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            tpx.tpx_probe_copy(b.data_ptr(), a.data_ptr(), n, stream)
        e1.record()
        torch.cuda.synchronize()
        probe = round(2 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        # the runtime's own device-to-device copy of the same bytes (torch issues a hipMemcpyAsync for it)
        for _ in range(2):
            b[:n].copy_(a[:n])
        e0.record()
        for _ in range(5):
            b[:n].copy_(a[:n])
        e1.record()
        torch.cuda.synchronize()
        memcpy_probe = round(2 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        # pure read and pure write streams (the library's yardsticks): a copy lies between the two
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
        for which in ("read", "fill"):
            def one():
                if which == "read":
                    tpx.tpx_probe_read(a.data_ptr(), n, sink.data_ptr(), stream)
                else:
                    tpx.tpx_probe_fill(b.data_ptr(), n, 0x5A5A5A5A, stream)
            for _ in range(2):
                one()
            e0.record()
            for _ in range(5):
                one()
            e1.record()
            torch.cuda.synchronize()
            rate = round(n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
            if which == "read":
                read_probe = rate
            else:
                write_probe = rate

    cpu = None
    if args.cpu_layers > 0:
        cpu = cpu_baseline(args, model, src, dst, plan, src_bufs, dst_bufs, src_ptrs, dst_ptrs, ws, stream)

    out = {
        "metric": "reshard_GBps_state_bytes_read_plus_written",
        "value": round(state_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "state_bytes_read": stats["bytes_read"],
                   "state_bytes_written": stats["bytes_written"], "n_boxes": stats["n_boxes"],
                   "n_tiles": stats["n_tiles"], "src_ranks": n_src, "dst_ranks": n_dst,
                   "share_reads": int(args.share_reads)},
        "pct_of_hbm_peak": round(100 * achieved / HBM_PEAK_GBPS, 2),
        "ms_per_reconfig": {"plan_host": round(plan_ms, 4), "kernel": round(kernel_ms_avg, 4),
                            "isolated_plan_upload_kernel": round(latency_ms, 4),
                            "back_to_back_step": round(ms_per_step, 4)},
        "copy_probe_GBps": probe,
        "copy_probe_bytes": probe_bytes,
        "memcpy_d2d_GBps": memcpy_probe,
        "read_probe_GBps": read_probe,
        "write_probe_GBps": write_probe,
        # the rate of a memory that serves the reads at the read-only rate and the writes at the write-only rate, in turn
        "read_write_mix_GBps": round(2 / (1 / read_probe + 1 / write_probe), 1) if read_probe and write_probe else None,
        "pct_of_read_write_mix": round(100 * achieved / (2 / (1 / read_probe + 1 / write_probe)), 2) if read_probe and write_probe else None,
        "pct_of_copy_probe": round(100 * achieved / probe, 2) if probe else None,
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def settle(seconds, launch):
    """Keep the device busy with `launch` (asynchronous, queued a few deep) for about `seconds` of wall-clock time."""
    import torch
    t_end = time.perf_counter() + seconds
    while seconds > 0 and time.perf_counter() < t_end:
        for _ in range(4):
            launch()
        torch.cuda.synchronize()


class TwoWorkspaces:
    """The plan tables of consecutive steps go to two workspaces in turn, uploaded on a stream of their own, so that the
    upload for step i + 1 runs while step i's kernel (which reads the other workspace) is still busy, and kernel i + 1 is
    queued right behind kernel i.  Before a workspace is overwritten, the upload stream waits for the last kernel that
    read it."""

    def __init__(self, nbytes):
        import torch
        self.ws = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
        self.upload = torch.cuda.Stream()
        self.done = [None, None]
        self.turn = 0

    def next(self):
        import torch
        k = self.turn
        self.turn ^= 1
        if self.done[k] is not None:
            self.upload.wait_event(self.done[k])
        return k, self.ws[k].data_ptr(), self.upload.cuda_stream

    def used(self, k):
        import torch
        self.done[k] = torch.cuda.Event()
        self.done[k].record()


PLAN_KEYS = ("tile_bytes", "max_multicast", "share_reads", "pack_bytes")
KNOB_DEFAULTS = {"streams": 4, "chunk": 0, "occupancy": 0, "variant": 0}


def ab_compare(args) -> int:
    """A/B/A comparison of executor knobs and plan options on one workload, inside one process: every setting runs on
    the same source and destination buffers (so on the same physical pages), in three interleaved rounds of six launches,
    timed with HIP events.  Reports bytes moved per second per round for every setting.  Settings are tpx_plan_opts
    fields, tpx_set_option keys and dst_shift_kib (see below: where the destination buffers sit relative to the sources)."""
    import torch

    import paper_2312_05181_amd as tpx

    cfgs = []
    for text in args.ab.split(";"):
        cfg = dict((kv.split("=")[0].strip(), int(kv.split("=")[1])) for kv in text.split(",") if kv.strip())
        unknown = set(cfg) - set(PLAN_KEYS) - set(KNOB_DEFAULTS) - {"dst_shift_kib", "rank_skew_kib"}
        if unknown:
            print(f"bench.py --ab: unknown key {sorted(unknown)[0]}", file=sys.stderr)
            return 2
        cfgs.append((text.strip() or "default", cfg))

    def make_plan(cfg):
        opts = dict(args.opts)
        opts.update({k: v for k, v in cfg.items() if k in PLAN_KEYS})
        if args.workload == DATASET_WORKLOAD:
            c = DATASET_CFG
            cur = [c["steps_done"] * (c["global_batch"] // c["D_src"])] * c["D_src"]
            return tpx.tpx_plan_dataset(c["n_samples"], c["global_batch"], c["D_src"], c["D_dst"], cur, opts=opts)
        model, src, dst, _, _ = WORKLOADS[args.workload]
        return tpx.tpx_plan(model, src, dst, opts)

    plans = [make_plan(cfg) for _, cfg in cfgs]
    p0 = plans[0]
    ws = torch.empty(max(p.workspace_bytes() for p in plans), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    shifts = [cfg.get("dst_shift_kib", 0) << 10 for _, cfg in cfgs]
    skews = [cfg.get("rank_skew_kib", 0) << 10 for _, cfg in cfgs]
    placed = any(shifts) or any(skews)
    if not placed:
        src_bufs = [torch.full((max(1, p0.buffer_bytes(0, r)),), r + 1, dtype=torch.uint8, device="cuda") for r in range(p0.num_buffers(0))]
        dst_bufs = [torch.zeros(max(1, p0.buffer_bytes(1, r)), dtype=torch.uint8, device="cuda") for r in range(p0.num_buffers(1))]
        sp, dp = [b.data_ptr() for b in src_bufs], [b.data_ptr() for b in dst_bufs]
    else:
        # placement study: all rank buffers of a side inside one allocation, each at a 2 MiB boundary, the destination
        # side as a whole moved by the setting's shift, and rank buffer r of either side moved by (r mod 8) x the
        # setting's skew (multiples of 16 bytes, as tpx_execute requires)
        mib2 = 1 << 21
        sp = dp = None

        def arena(side, extra):
            offs, off = [], 0
            for r in range(p0.num_buffers(side)):
                offs.append(off)
                off = (off + p0.buffer_bytes(side, r) + 7 * max(skews) + mib2 - 1) // mib2 * mib2     # room for the largest skew
            mem = torch.full((off + extra + mib2,), 1 + side, dtype=torch.uint8, device="cuda")
            base = (mem.data_ptr() + mib2 - 1) // mib2 * mib2
            return mem, [base + o for o in offs]
        src_mem, sp0 = arena(0, 0)
        dst_mem, dp0 = arena(1, max(shifts))

    def timed(plan, cfg, launches=6):
        nonlocal sp, dp
        for key, default in KNOB_DEFAULTS.items():
            tpx.tpx_set_option(key, cfg.get(key, default))
        if placed:
            # rank buffer r of either side starts r * rank_skew_kib past its 2 MiB boundary (r mod 8, so the skew stays small)
            shift, skew = cfg.get("dst_shift_kib", 0) << 10, cfg.get("rank_skew_kib", 0) << 10
            if shift % 16 or skew % 16:
                raise SystemExit("dst_shift_kib and rank_skew_kib must give multiples of 16 bytes")
            sp = [q + (r % 8) * skew for r, q in enumerate(sp0)]
            dp = [q + shift + (r % 8) * skew for r, q in enumerate(dp0)]
        tpx.tpx_workspace_forget(ws.data_ptr())
        for _ in range(2):
            plan.execute(sp, dp, ws.data_ptr(), stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            plan.execute(sp, dp, ws.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        st = plan.stats()
        return (st["bytes_read"] + st["bytes_written"]) / (e0.elapsed_time(e1) / launches * 1e-3) / 1e9

    t_end = time.perf_counter() + args.settle_s          # device under load for a while before anything is compared
    while time.perf_counter() < t_end:
        timed(plans[0], cfgs[0][1])
    rounds = [[] for _ in cfgs]
    for _ in range(3):
        for i, ((_, cfg), plan) in enumerate(zip(cfgs, plans)):
            rounds[i].append(round(timed(plan, cfg), 1))
    for key, default in KNOB_DEFAULTS.items():
        tpx.tpx_set_option(key, default)
    print(json.dumps({"workload": args.workload, "unit": "GB/s", "peak": HBM_PEAK_GBPS,
                      "settings": [{"setting": name, "n_tiles": plan.stats()["n_tiles"], "rounds": r, "best": max(r),
                                    "pct_of_hbm_peak": round(100 * max(r) / HBM_PEAK_GBPS, 2)}
                                   for (name, _), plan, r in zip(cfgs, plans, rounds)]}), flush=True)
    return 0


def bench_dataset(args) -> int:
    """Dataset-state workload: 10^8 sample ids (uint64), global batch 768, 6 -> 4 replicas after 65,000 steps.
    A step is tpx_plan_dataset + table upload + tpx_execute; the oracle repartitions the same arrays on the CPU."""
    import numpy as np
    import torch

    import paper_2312_05181_amd as tpx
    import synth

    c = DATASET_CFG
    n, B, D, D2 = c["n_samples"], c["global_batch"], c["D_src"], c["D_dst"]
    b = B // D
    full, tail = n // B, n % B
    cursors = [min(full * b + max(0, min(b, tail - j * b)), c["steps_done"] * b) for j in range(D)]
    plan = tpx.tpx_plan_dataset(n, B, D, D2, cursors, opts=args.opts)
    stats = plan.stats()
    G = synth.epoch_order(n, c["seed"])
    # replica j holds, step by step, entries [k*B + j*b, k*B + (j+1)*b) of the global order
    parts = []
    for j in range(D):
        body = G[:full * B].reshape(full, B)[:, j * b:(j + 1) * b].reshape(-1)
        parts.append(np.concatenate([body, G[full * B + j * b: full * B + min(tail, (j + 1) * b)]]))
    src_bufs = [torch.from_numpy(p.view(np.uint8)).cuda() for p in parts]
    dst_bufs = [torch.zeros(plan.buffer_bytes(1, j), dtype=torch.uint8, device="cuda") for j in range(D2)]
    two = TwoWorkspaces(plan.workspace_bytes())
    ws = two.ws[0]
    sp, dp = [x.data_ptr() for x in src_bufs], [x.data_ptr() for x in dst_bufs]
    stream = torch.cuda.current_stream().cuda_stream
    state_bytes = stats["bytes_read"] + stats["bytes_written"]

    def step(e0=None, e1=None):
        p = tpx.tpx_plan_dataset(n, B, D, D2, cursors, opts=args.opts)
        k, w, upload_stream = two.next()
        p.prepare(w, upload_stream)
        if e0 is not None:
            e0.record()
        p.execute(sp, dp, w, stream)
        if e1 is not None:
            e1.record()
        two.used(k)
        return p

    settle(args.settle_s, lambda: plan.execute(sp, dp, ws.data_ptr(), stream))
    for _ in range(args.warmup):
        step()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    keep = [step(*e) for e in evs]
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = [a.elapsed_time(b_) for a, b_ in evs]
    kavg = sum(kernel_ms) / len(kernel_ms)
    achieved = state_bytes / (kavg * 1e-3) / 1e9
    traffic, traffic_from = measured_traffic(args.workload, stats)
    del keep

    cpu = None
    if args.cpu_layers > 0:
        from oracle import dataset as ods
        t0 = time.perf_counter()
        want, want_cur = ods.repartition(parts, cursors, B, D2)
        secs = time.perf_counter() - t0
        ok = plan.dst_cursors == want_cur and all(
            np.array_equal(dst_bufs[j].cpu().numpy().view(np.uint64), want[j]) for j in range(D2))
        cpu = {"value": round(state_bytes / secs / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "the whole workload (10^8 ids), numpy, single thread", "seconds": round(secs, 2),
               "gpu_matches_oracle_on_sample": bool(ok)}
    out = {"metric": "reshard_GBps_state_bytes_read_plus_written", "value": round(state_bytes / (ms_per_step * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
           "config": {"workload": args.workload, "state_bytes_read": stats["bytes_read"],
                      "state_bytes_written": stats["bytes_written"], "n_boxes": stats["n_boxes"], "n_tiles": stats["n_tiles"],
                      "src_ranks": D, "dst_ranks": D2},
           "pct_of_hbm_peak": round(100 * achieved / HBM_PEAK_GBPS, 2),
           "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_from": traffic_from,
                        "kernel": "tpx_execute_tiles",
                        "kernel_ms_avg": round(kavg, 4), "kernel_ms_min": round(min(kernel_ms), 4),
                        "kernel_ms_median": round(sorted(kernel_ms)[len(kernel_ms) // 2], 4),
                        "algorithmic_bytes_per_launch": state_bytes},
           "cpu_baseline": cpu}
    print(json.dumps(out), flush=True)
    return 0


def _cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(args, model, src, dst, plan, src_bufs, dst_bufs, src_ptrs, dst_ptrs, ws, stream):
    """Time the CPU oracle (numpy: paste the old shards into the full tensor, slice it anew) on the state
    tensors of the first `--cpu-layers` layers, threaded over tensors; check the GPU result against it."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor

    from oracle import reshard as oreshard
    from oracle import spec

    om = spec.Model(model["n_layers"], model["hidden"], model["n_heads"], model["ffn"], model["vocab_true"],
                    model.get("max_pos", 1024), model.get("vocab_divisor", 0), tuple(model["state_elem_bytes"]))
    def opar(c):
        return spec.Parallel(c["T"], c["P"], c["D"], c.get("stage_first_layer"), c.get("qkv_layout", 0),
                             c.get("w_transposed", 0), c.get("shard_kinds", 0), c.get("layer_stage"))
    osrc, odst = opar(src), opar(dst)
    src_lay, dst_lay = oreshard.Layout(om, osrc), oreshard.Layout(om, odst)
    layers = min(args.cpu_layers, om.n_layers)
    work = [(4 + l * 12 + k, kind) for l in range(layers) for k in range(12) for kind in range(len(om.state_elem_bytes))]
    # fetch the sample's source shards to host memory first (not timed)
    cache = {}
    for tid, kind in work:
        for rank, e in src_lay.by_tensor[(tid, kind)]:
            n = int(np.prod([h - l for l, h in zip(e.lo, e.hi)])) * e.elem_bytes
            cache[(rank, e.offset)] = src_bufs[rank][e.offset:e.offset + n].cpu().numpy()

    def read(rank, off, n):
        return cache[(rank, off)]

    threads = max(1, min(16, os.cpu_count() or 1))
    results = {}

    def one(tk):
        results[tk] = oreshard.reshard_tensor(om, osrc, odst, src_lay, dst_lay, tk[0], tk[1], read)

    passes = 3  # the same sample several times: about 15 s of CPU time in all
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        for _ in range(passes):
            list(ex.map(one, work))
    secs = (time.perf_counter() - t0) / passes
    moved = 0
    plan.execute(src_ptrs, dst_ptrs, ws.data_ptr(), stream)
    torch.cuda.synchronize()
    ok = True
    built = dst.get("rank_alive")
    for tk, outs in results.items():
        for rank, e, block in outs:
            if built is not None and not built[rank]:
                continue                      # a destination rank that is not rebuilt
            moved += 2 * block.nbytes
            have = dst_bufs[rank][e.offset:e.offset + block.nbytes].cpu().numpy()
            ok = ok and bool(np.array_equal(have, block.reshape(-1).view(np.uint8)))
    return {"value": round(moved / secs / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"all state tensors of the first {layers} of {om.n_layers} layers "
                      f"({moved / 2e9:.2f} GB read + the same written, counted on the oracle's output: where the new "
                      f"configuration does not slice a tensor its re-slice is a view and only the paste copies), numpy, "
                      f"{threads} threads over tensors, mean of {passes} passes",
            "seconds": round(secs, 2), "host_cpus_online": os.cpu_count(), "host_cpu_model": _cpu_model(),
            "gpu_matches_oracle_on_sample": ok}


if __name__ == "__main__":
    sys.exit(main())
