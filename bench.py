#!/usr/bin/env python3
"""Benchmark of the EFIM serving hot path on one MI355X.

A step is one pass of the whole path over one synthetic ragged batch:
efim_rope_append (RoPE at offset positions + paged KV append) followed by
efim_extend_attention, i.e. one attention layer's worth of a serving step (no
projections or MLP: those are not part of this path).  The headline workload is
the mixed serving step (64 requests, half cache hits, half misses); the other
workloads and the fixed-inc sweeps are reported in the same JSON line under
"workloads"; the service replay, the decode step and the 8-bit KV cache have sections of their own.

Prints ONE JSON line.  All inputs are seeded and synthetic and resident in HBM
before the timed region starts.
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

# HBM traffic of the dominant kernel on the headline workload, bytes per launch, taken from the
# rocprofv3 --pmc runs summarised under profiles/ (FETCH_SIZE + WRITE_SIZE, each scaled by what
# the same counter reads for a 1 GiB copy).  Valid only for the kernel source it was measured
# on: the digest of extend_attention.hip is recorded with it and checked at run time.
MEASURED_TRAFFIC = {
    # workload: (bytes per launch, sha256 of csrc/extend_attention.hip when measured)
    "c5": (2586449093, "670040b0231dcd4819c4ba31518c52aebdefded2f1c99ae12c236741e673c4eb"),
}

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", help="headline workload (c2..c5)")
    ap.add_argument("--inc", type=int, default=0,
                    help="give every request of the headline workload this many new tokens (the fixed-inc sweeps: "
                         "1, 8, 16 on c2/c3; 256, 1024 on c4); 0 keeps the workload's own draw")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads and sweeps")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured-ceiling kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extra-iters", type=int, default=100)
    ap.add_argument("--decode-only", action="store_true",
                    help="run only the decode-step section (used to profile that kernel on its own; "
                         "--workload c2 or c3 restricts it to that batch shape)")
    ap.add_argument("--fp8-only", action="store_true",
                    help="run only the 8-bit KV cache section (to profile those kernels on their own; "
                         "--workload c2 or c3 restricts it to that batch shape)")
    ap.add_argument("--ceilings-only", action="store_true",
                    help="run only the measured-ceiling kernels (dense MFMA loop, streaming read, copy)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain 1 GiB device copy (reference dispatch for the HBM byte counters)")
    return ap.parse_args()


class DeviceBatch:
    """A workload's lengths and block table plus `copies` independent sets of device tensors
    (rotated between iterations so that the 256 MB last-level cache cannot hold the K/V)."""

    def __init__(self, torch, E, W, name, lengths=None, copies=1, seed=0):
        self.name = name
        self.host = W.make_batch(name, with_history=False, with_tensors=False, lengths=lengths)
        b = self.host
        self.table = torch.from_numpy(b.block_table).cuda()
        self.desc = E.BatchDesc(b.cached_len, b.new_len, self.table, b.num_q_heads, b.num_kv_heads,
                                b.head_dim, b.page_size, b.num_pages)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1000 + seed)
        t = b.total_new

        def gauss(shape):
            x = torch.empty(shape, dtype=torch.float32, device="cuda")
            x.normal_(0.0, b.sigma, generator=gen)
            return x.to(torch.bfloat16)

        self.sets = []
        for _ in range(copies):
            s = {
                # a rotation of iid Gaussian pairs is again Gaussian, so the cached part of the
                # cache is drawn directly instead of being built by appending a history
                "k_cache": gauss(b.cache_shape()), "v_cache": gauss(b.cache_shape()),
                "q_raw": gauss((t, b.num_q_heads, b.head_dim)),
                "k_new": gauss((t, b.num_kv_heads, b.head_dim)),
                "v_new": gauss((t, b.num_kv_heads, b.head_dim)),
            }
            s["q"] = s["q_raw"].clone()
            s["out"] = torch.empty_like(s["q"])
            self.sets.append(s)
        self.ws_bytes = E.efim_extend_workspace_bytes(self.desc)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device="cuda")
        self.flops = W.attention_flops(b)
        self.attn_bytes = W.attention_bytes(b)
        self.rope_bytes = W.rope_append_bytes(b)


def run_step(E, db, s, stream):
    b = db.host
    E.efim_rope_append(db.desc, s["q"], s["k_new"], s["v_new"], s["k_cache"], s["v_cache"], b.rope_base, 0, stream)
    E.efim_extend_attention(db.desc, s["q"], s["k_cache"], s["v_cache"], s["out"], 0.0, db.ws, db.ws_bytes, stream)


def time_parts(torch, E, db, iters, warmup):
    """Device times in microseconds (HIP events on the launch stream), everything queued back to
    back as a serving engine issues it (the device stays as warm as in the headline loop).
    Phase 1, whole steps (rope_append + extend_attention): the main attention kernel alone, one
    pair of events per step recorded by the library around it.  Phase 2: the whole
    efim_rope_append call and the whole efim_extend_attention call (main kernel, merge pass,
    launch gaps), total over the queue divided by the number of calls."""
    stream = torch.cuda.current_stream()
    e0, e1 = E.HipEvent(), E.HipEvent()
    b = db.host
    pairs = [(E.HipEvent(), E.HipEvent()) for _ in range(iters)]
    try:
        for it in range(warmup + iters):
            s = db.sets[it % len(db.sets)]
            if it >= warmup:
                E.efim_set_kernel_events(pairs[it - warmup][0].ptr, pairs[it - warmup][1].ptr)
            E.efim_rope_append(db.desc, s["q"], s["k_new"], s["v_new"], s["k_cache"], s["v_cache"], b.rope_base, 0, stream)
            E.efim_extend_attention(db.desc, s["q"], s["k_cache"], s["v_cache"], s["out"], 0.0, db.ws, db.ws_bytes, stream)
        torch.cuda.synchronize()
    finally:
        E.efim_set_kernel_events(None, None)
    kern = [a.elapsed_ms(c) * 1e3 for a, c in pairs]

    def queued(call, reps=3):
        times = []
        for _ in range(reps):
            torch.cuda.synchronize()
            e0.record(stream)
            for it in range(iters):
                call(db.sets[it % len(db.sets)])
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_ms(e1) * 1e3 / iters)
        return float(np.median(times))

    # (roping an already roped q again only changes values, not the work)
    rope = queued(lambda s: E.efim_rope_append(db.desc, s["q"], s["k_new"], s["v_new"], s["k_cache"], s["v_cache"],
                                               b.rope_base, 0, stream))
    attn = queued(lambda s: E.efim_extend_attention(db.desc, s["q"], s["k_cache"], s["v_cache"], s["out"], 0.0,
                                                    db.ws, db.ws_bytes, stream))
    med = lambda x: float(np.median(x))
    return {"rope_us": rope, "attn_call_us": attn, "attn_kernel_us": med(kern),
            "attn_kernel_us_mean": float(np.mean(kern)), "attn_kernel_us_min": float(np.min(kern))}


def summarize(db, parts):
    us = parts["attn_kernel_us"]
    call = parts["attn_call_us"]
    return {
        "T_new": db.host.total_new,
        "rope_append_us": round(parts["rope_us"], 2),
        "rope_append_GBps": round(db.rope_bytes / parts["rope_us"] / 1e3, 1),
        "rope_append_frac_hbm": round(db.rope_bytes / parts["rope_us"] / 1e3 / PEAK_HBM_GBPS, 4),
        # "call" = the whole efim_extend_attention call on the stream (main kernel, merge pass,
        # launch gaps); "kernel" = its main kernel alone
        "attn_call_us": round(call, 2),
        "attn_kernel_us": round(us, 2),
        "attn_TFLOPs": round(db.flops / call / 1e6, 2),
        "attn_frac_mfma": round(db.flops / call / 1e6 / PEAK_BF16_TFLOPS, 4),
        "attn_GBps": round(db.attn_bytes / call / 1e3, 1),
        "attn_frac_hbm": round(db.attn_bytes / call / 1e3 / PEAK_HBM_GBPS, 4),
        "attn_kernel_frac_mfma": round(db.flops / us / 1e6 / PEAK_BF16_TFLOPS, 4),
        "attn_kernel_frac_hbm": round(db.attn_bytes / us / 1e3 / PEAK_HBM_GBPS, 4),
        "step_us": round(parts["rope_us"] + call, 2),
    }


def replay_lengths(E, W, scheme, docs):
    """(cached_len, new_len) of every round of the service replay under one scheme: 'baseline'
    recomputes every prompt, 'fim' sends PSM prompts to a prefix-matching cache with 16-token
    pages, 'efim' puts the session pool's rewrite in front of the same cache (EFIM Sec. 4.2)."""
    pool = None if scheme == "baseline" else E.SessionPool(*W.REPLAY_MARKERS, reuse_granularity=16,
                                                           always_psm=(scheme == "fim"))
    rounds = []
    for docs_round in docs:
        c, n = [], []
        for user, (prefix, suffix) in enumerate(docs_round):
            if pool is None:
                c.append(0)
                n.append(len(prefix) + len(suffix) + 3)
            else:
                info = pool.efim_session_transform(user, prefix, suffix)
                c.append(info["cached_len"])
                n.append(info["new_len"])
        rounds.append((np.asarray(c, dtype=np.int32), np.asarray(n, dtype=np.int32)))
    if pool is not None:
        pool.close()
    return rounds


def replay(torch, E, W, iters):
    """Kernel-level replay of the 16-user, 5-round service of EFIM Sec. 4.2: per head layout and
    scheme, the device time of one attention layer's step (rope_append + extend_attention) in
    every round, the share of prompt tokens served from the cache, and prompt tokens per
    second of that one layer."""
    out = {}
    docs = W.replay_documents()
    for spec in ("replay", "replay_mha"):
        per_scheme = {}
        for scheme in ("baseline", "fim", "efim"):
            round_us, cached, total = [], 0, 0
            for c, n in replay_lengths(E, W, scheme, docs):
                d = DeviceBatch(torch, E, W, spec, lengths=(c, n), copies=2)
                parts = time_parts(torch, E, d, iters=iters, warmup=10)
                round_us.append(round(parts["rope_us"] + parts["attn_call_us"], 2))
                cached += int(c.sum())
                total += int(c.sum() + n.sum())
                del d
                torch.cuda.empty_cache()
            per_scheme[scheme] = {"round_us": round_us, "total_us": round(sum(round_us), 2),
                                  "reuse_rate": round(cached / total, 4),
                                  "prompt_tokens_per_s": round(total / (sum(round_us) * 1e-6), 1)}
        base = per_scheme["baseline"]["total_us"]
        for scheme in per_scheme:
            per_scheme[scheme]["time_vs_baseline"] = round(per_scheme[scheme]["total_us"] / base, 4)
        out[spec] = per_scheme
    return out


def decode_steps(torch, E, W, iters, shapes=("c2", "c3", "c2:8", "c2:16", "c3:4")):
    """Decode (one new token per request) and other short steps ("c2:16" = 16 new tokens per
    request) at the batch shapes of c2 and c3: device time of the step through the two calls
    (efim_rope_append + efim_extend_attention) and through the single-launch efim_decode_step;
    steps queued back to back, HIP events around the queue."""
    out = {}
    stream = torch.cuda.current_stream()
    for shape in shapes:
        base, _, inc = shape.partition(":")
        inc = int(inc or 1)
        spec = W.make_batch(base, with_history=False, with_tensors=False)
        d = DeviceBatch(torch, E, W, base, lengths=(spec.cached_len, np.full_like(spec.new_len, inc)), copies=3)
        nbytes = E.efim_decode_workspace_bytes(d.desc)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        e0, e1 = E.HipEvent(), E.HipEvent()
        b = d.host

        def queued(call, reps=5):
            times = []
            for _ in range(reps):
                torch.cuda.synchronize()
                e0.record(stream)
                for it in range(iters):
                    call(d.sets[it % len(d.sets)])
                e1.record(stream)
                e1.synchronize()
                times.append(e0.elapsed_ms(e1) * 1e3 / iters)
            return times[1:]  # the first repetition warms up

        two = queued(lambda s: run_step(E, d, s, stream))
        one = queued(lambda s: E.efim_decode_step(d.desc, s["q_raw"], s["k_new"], s["v_new"], s["k_cache"],
                                                  s["v_cache"], s["out"], b.rope_base, 0, 0.0, ws, nbytes, stream))
        t2, t1 = float(np.median(two)), float(np.median(one))
        # the same step as a plan object: work list in the caller's workspace, kernels only; eager,
        # and captured into a HIP graph of `iters` steps (rotating over the tensor sets)
        plan = E.Plan(d.desc, decode=True)
        pbytes = E.efim_plan_workspace_bytes(plan)
        pws = torch.empty(pbytes, dtype=torch.uint8, device="cuda")
        E.efim_plan_upload(plan, pws, pbytes, stream)
        planned_call = lambda s, st=stream: E.efim_decode_step_planned(plan, d.table, s["q_raw"], s["k_new"], s["v_new"],
                                                                       s["k_cache"], s["v_cache"], s["out"], b.rope_base,
                                                                       0, 0.0, pws, st)
        tp = float(np.median(queued(planned_call)))
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            cur = torch.cuda.current_stream()
            for it in range(iters):
                planned_call(d.sets[it % len(d.sets)], cur)
        gt = []
        for _ in range(5):
            torch.cuda.synchronize()
            e0.record(stream)
            graph.replay()
            e1.record(stream)
            e1.synchronize()
            gt.append(e0.elapsed_ms(e1) * 1e3 / iters)
        tg = float(np.median(gt[1:]))
        del graph
        plan.close()
        nbytes_step = d.attn_bytes + d.rope_bytes
        out[base + ("_decode" if inc == 1 else "_inc%d_one_launch" % inc)] = {
            "batch": b.batch, "new_tokens_per_request": inc, "two_call_us": round(t2, 2), "single_launch_us": round(t1, 2),
            "speedup": round(t2 / t1, 3),
            "planned_us": round(tp, 2), "planned_graph_replay_us": round(tg, 2),
            "planned_graph_replay_frac_hbm": round(nbytes_step / tg / 1e3 / PEAK_HBM_GBPS, 4),
            "single_launch_GBps": round(nbytes_step / t1 / 1e3, 1),
            "single_launch_frac_hbm": round(nbytes_step / t1 / 1e3 / PEAK_HBM_GBPS, 4),
            "two_call_frac_hbm": round(nbytes_step / t2 / 1e3 / PEAK_HBM_GBPS, 4),
        }
        del d, ws
        torch.cuda.empty_cache()
    return out


def fp8_cache(torch, E, W, iters, shapes=("c2", "c3")):
    """The 8-bit (E4M3, per-tensor scale) KV cache on decode-like steps at the batch shapes of c2
    and c3: the whole efim_extend_attention_fp8 call at one new token per request and the
    single-launch efim_decode_step_fp8, next to their bf16 counterparts.  Bytes are the
    algorithmic ones with one byte per cache element."""
    out = {}
    stream = torch.cuda.current_stream()
    for base in shapes:
        spec = W.make_batch(base, with_history=False, with_tensors=False)
        d = DeviceBatch(torch, E, W, base, lengths=(spec.cached_len, np.ones_like(spec.new_len)), copies=3)
        b = d.host
        scale = 4.0 * b.sigma / 448.0   # four standard deviations reach the largest code
        for s in d.sets:
            for name in ("k_cache", "v_cache"):
                s[name + "8"] = (s[name].float() / scale).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8)
        nbytes = E.efim_decode_workspace_bytes(d.desc)
        ws = torch.empty(max(nbytes, d.ws_bytes, 256), dtype=torch.uint8, device="cuda")
        e0, e1 = E.HipEvent(), E.HipEvent()

        def queued(call, reps=5):
            times = []
            for _ in range(reps):
                torch.cuda.synchronize()
                e0.record(stream)
                for it in range(iters):
                    call(d.sets[it % len(d.sets)])
                e1.record(stream)
                e1.synchronize()
                times.append(e0.elapsed_ms(e1) * 1e3 / iters)
            return float(np.median(times[1:]))

        a16 = queued(lambda s: E.efim_extend_attention(d.desc, s["q"], s["k_cache"], s["v_cache"], s["out"], 0.0,
                                                       ws, d.ws_bytes, stream))
        a8 = queued(lambda s: E.efim_extend_attention_fp8(d.desc, s["q"], s["k_cache8"], s["v_cache8"], s["out"], 0.0,
                                                          scale, scale, ws, d.ws_bytes, stream))
        s16 = queued(lambda s: E.efim_decode_step(d.desc, s["q_raw"], s["k_new"], s["v_new"], s["k_cache"],
                                                  s["v_cache"], s["out"], b.rope_base, 0, 0.0, ws, nbytes, stream))
        s8 = queued(lambda s: E.efim_decode_step_fp8(d.desc, s["q_raw"], s["k_new"], s["v_new"], s["k_cache8"],
                                                     s["v_cache8"], s["out"], b.rope_base, 0, 0.0, scale, scale,
                                                     ws, nbytes, stream))
        bytes8 = W.attention_bytes(b, 1)
        step8 = bytes8 + W.rope_append_bytes(b, 1)
        out[base + "_inc1"] = {
            "batch": b.batch,
            "attn_call_us_bf16": round(a16, 2), "attn_call_us_fp8": round(a8, 2), "attn_speedup": round(a16 / a8, 3),
            "attn_fp8_GBps": round(bytes8 / a8 / 1e3, 1), "attn_fp8_frac_hbm": round(bytes8 / a8 / 1e3 / PEAK_HBM_GBPS, 4),
            "decode_step_us_bf16": round(s16, 2), "decode_step_us_fp8": round(s8, 2),
            "decode_step_speedup": round(s16 / s8, 3),
            "decode_step_fp8_frac_hbm": round(step8 / s8 / 1e3 / PEAK_HBM_GBPS, 4),
        }
        del d, ws
        torch.cuda.empty_cache()
    return out


def measure_ceilings(torch, E, reps=7):
    """What kernels that do nothing but the bound operation reach on this device (the kernels
    of libefim_ceilings.so, which is not part of the library): dense bf16 MFMA from registers on
    N(0,1) operands with every SIMD busy, a streaming read and a streaming copy of 2 GiB.
    Device times from HIP events around each launch; the median of `reps` launches."""
    import ctypes
    from paper_2505_21889_amd import build as _build
    if not os.path.exists(_build.CEILINGS_PATH):
        _build.build_ceilings()
    lib = ctypes.CDLL(_build.CEILINGS_PATH)
    vp = ctypes.c_void_p
    lib.efim_ceiling_mfma_operand_bytes.argtypes = [ctypes.c_int]
    lib.efim_ceiling_mfma_operand_bytes.restype = ctypes.c_size_t
    lib.efim_ceiling_mfma_flops.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.efim_ceiling_mfma_flops.restype = ctypes.c_double
    lib.efim_ceiling_mfma_bf16.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp]
    lib.efim_ceiling_tile_loop_operand_bytes.argtypes = [ctypes.c_int]
    lib.efim_ceiling_tile_loop_operand_bytes.restype = ctypes.c_size_t
    lib.efim_ceiling_tile_loop_flops.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.efim_ceiling_tile_loop_flops.restype = ctypes.c_double
    lib.efim_ceiling_tile_loop.argtypes = [ctypes.c_int, vp, vp, vp, ctypes.c_int, ctypes.c_int, vp]
    lib.efim_ceiling_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int, vp]
    lib.efim_ceiling_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    e0, e1 = E.HipEvent(), E.HipEvent()

    def timed(launch):
        times = []
        for _ in range(reps + 2):
            e0.record(stream)
            rc = launch()
            e1.record(stream)
            e1.synchronize()
            assert rc == 0, "ceiling kernel failed: %d" % rc
            times.append(e0.elapsed_ms(e1) * 1e-3)
        return float(np.median(times[2:]))   # the first two launches warm up

    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    nbytes = lib.efim_ceiling_mfma_operand_bytes(cus)
    ops = torch.empty(nbytes // 2, dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen).to(torch.bfloat16)
    sink = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    iters = 2000
    t_mfma = timed(lambda: lib.efim_ceiling_mfma_bf16(ops.data_ptr(), sink.data_ptr(), cus, iters, sp))
    flops = lib.efim_ceiling_mfma_flops(cus, iters)
    # the attention kernel's tile loop, one ingredient at a time (fixed data, no paging or masks)
    tl_ops = torch.empty(lib.efim_ceiling_tile_loop_operand_bytes(cus) // 2, dtype=torch.float32,
                         device="cuda").normal_(0.0, 1.0, generator=gen).to(torch.bfloat16)
    tl_gather = torch.empty(cus * 131072 // 2, dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen).to(torch.bfloat16)
    tiles = 2000
    tl_flops = lib.efim_ceiling_tile_loop_flops(cus, tiles)
    tile_loop = {}
    for mode, label in enumerate(("mfma_only", "with_lds_operands", "with_softmax", "with_gather")):
        t = timed(lambda: lib.efim_ceiling_tile_loop(mode, tl_ops.data_ptr(), tl_gather.data_ptr(), sink.data_ptr(),
                                                     cus, tiles, sp))
        tile_loop[label + "_TFLOPs"] = round(tl_flops / t / 1e12, 1)
    del tl_ops, tl_gather
    size = 2 << 30
    src = torch.empty(size, dtype=torch.uint8, device="cuda")
    src.random_(0, 256, generator=gen)
    dst = torch.empty_like(src)
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    t_read = timed(lambda: lib.efim_ceiling_read(src.data_ptr(), size, word.data_ptr(), cus * 8, sp))
    t_copy = timed(lambda: lib.efim_ceiling_copy(dst.data_ptr(), src.data_ptr(), size, cus * 8, sp))
    del src, dst, ops, sink
    torch.cuda.empty_cache()
    return {
        "mfma_TFLOPs": round(flops / t_mfma / 1e12, 1), "mfma_frac_of_peak": round(flops / t_mfma / 1e12 / PEAK_BF16_TFLOPS, 4),
        "read_GBps": round(size / t_read / 1e9, 1), "read_frac_of_peak": round(size / t_read / 1e9 / PEAK_HBM_GBPS, 4),
        "copy_GBps": round(2 * size / t_copy / 1e9, 1), "copy_frac_of_peak": round(2 * size / t_copy / 1e9 / PEAK_HBM_GBPS, 4),
        # what the tile loop's structure (eight waves of 32 rows, 64-key tiles, a barrier per tile)
        # reaches as its ingredients are added: MFMAs alone, + K / V^T operands from LDS, + the
        # softmax arithmetic, + the direct-to-LDS loads of the next tiles
        "tile_loop": tile_loop,
        "what": "libefim_ceilings.so: v_mfma_f32_32x32x16_bf16 from registers (2 waves per SIMD, %d workgroups, N(0,1) "
                "operands); streaming read of 2 GiB; streaming copy of 2 GiB (read + written bytes); tile_loop: %d workgroups "
                "of 8 waves x 32 rows over 2000 64-key tiles each, 8.39e6 flop per tile" % (cus, cus),
    }


def recorded_traffic(name):
    import hashlib
    rec = MEASURED_TRAFFIC.get(name)
    if not rec:
        return None
    src = os.path.join(ROOT, "paper_2505_21889_amd", "csrc", "extend_attention.hip")
    with open(src, "rb") as fh:
        digest = hashlib.sha256(fh.read()).hexdigest()
    return rec[0] if digest == rec[1] else None


def cpu_baseline(W, name):
    """The CPU oracle timed on a bounded sample of the headline workload."""
    from oracle import efim_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    full = W.make_batch(name, with_history=False, with_tensors=False)
    c, n = full.cached_len, full.new_len
    if name == "c5":
        hits = [r for r in range(len(c)) if c[r] > 0]
        misses = [r for r in range(len(c)) if c[r] == 0][:4]
        sel = sorted(hits + misses)
        what = "the %d cache hits and the first %d misses of the mixed step, all heads" % (len(hits), len(misses))
    else:
        sel = list(range(min(2, len(c))))
        what = "requests %s, all heads" % sel
    b = W.make_batch(name, with_history=False, lengths=(c[sel], n[sel]), seed=4242)
    rng = np.random.default_rng(4243)
    kc = W.gaussian_bf16(rng, b.cache_shape(), b.sigma)
    vc = W.gaussian_bf16(rng, b.cache_shape(), b.sigma)
    t0 = time.perf_counter()
    q_roped, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new,
                               b.v_new, kc, vc, b.rope_base)
    O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    dt = time.perf_counter() - t0
    flops = W.attention_flops(b)
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": what + "; %.1f s, %.3e flop" % (dt, flops), "seconds": round(dt, 2)}


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this path runs on ONE GPU only (no sharding, no collectives); "
                         "--gpus %d is not supported\n" % args.gpus)
        sys.exit(2)
    import torch
    from paper_2505_21889_amd import binding as E, workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.calibrate_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.ceilings_only:
        print(json.dumps({"ceilings": measure_ceilings(torch, E)}))
        return

    if args.decode_only:
        kw = {"shapes": (args.workload,)} if args.workload in ("c2", "c3") else {}
        print(json.dumps({"decode_step": decode_steps(torch, E, W, iters=args.extra_iters, **kw)}))
        return

    if args.fp8_only:
        shapes = (args.workload,) if args.workload in ("c2", "c3") else ("c2", "c3")
        print(json.dumps({"fp8_kv_cache": fp8_cache(torch, E, W, iters=args.extra_iters, shapes=shapes)}))
        return

    name = args.workload
    copies = 3   # independent tensor sets, rotated between steps: the last-level cache cannot hold the K/V
    lengths = None
    if args.inc > 0:
        spec = W.make_batch(name, with_history=False, with_tensors=False)
        lengths = (spec.cached_len, np.full_like(spec.new_len, args.inc))
    db = DeviceBatch(torch, E, W, name, lengths=lengths, copies=copies)

    # ---- headline: K timed steps, wall clock around a synchronised region ------------
    for it in range(args.warmup):
        run_step(E, db, db.sets[it % copies], stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(args.steps):
        run_step(E, db, db.sets[it % copies], stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    parts = time_parts(torch, E, db, iters=max(5, min(args.steps, 30)), warmup=10)
    head = summarize(db, parts)
    kernel_us = parts["attn_kernel_us_mean"]
    mfma_bound = db.flops / PEAK_BF16_TFLOPS / 1e12 >= db.attn_bytes / PEAK_HBM_GBPS / 1e9
    if mfma_bound:
        ach = db.flops / kernel_us / 1e6
        roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": None}
    else:
        ach = db.attn_bytes / kernel_us / 1e3
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBPS, 4), "traffic": None}
    roofline["traffic"] = recorded_traffic(name) if args.inc == 0 else None
    roofline["kernel"] = "extend_attention_kernel<%d>" % db.host.head_dim
    roofline["kernel_avg_us"] = round(kernel_us, 2)
    # what this device reaches on the bound operation alone, measured in this run
    ceilings = None if args.no_ceilings else measure_ceilings(torch, E)
    if ceilings:
        roofline["measured_ceiling"] = ceilings["mfma_TFLOPs"] if mfma_bound else ceilings["read_GBps"]
        roofline["frac_of_measured_ceiling"] = round(ach / roofline["measured_ceiling"], 4)

    result = {
        "metric": "extend-attention TFLOP/s over one serving step (rope_append + extend_attention)",
        "value": round(db.flops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "us_per_step": round(ms_per_step * 1e3, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s%s" % (name, W.SPECS[name].describe,
                                             "; every request with %d new tokens" % args.inc if args.inc > 0 else ""),
                   "batch": db.host.batch,
                   "total_new_tokens": db.host.total_new, "page_size": db.host.page_size,
                   "heads": "%d/%d" % (db.host.num_q_heads, db.host.num_kv_heads), "head_dim": db.host.head_dim},
        "pct_bf16_mfma_peak": round(100 * db.flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
        "step_hbm_GBps": round((db.attn_bytes + db.rope_bytes) / (ms_per_step * 1e-3) / 1e9, 1),
        "headline_parts": head,
        "roofline": roofline,
        "ceilings": ceilings,
    }
    del db
    torch.cuda.empty_cache()

    # ---- the other workloads and the fixed-inc sweeps (device times per call) ---------
    if not args.no_extra:
        extra = {}
        todo = [(n, None) for n in ("c2", "c3", "c4", "c5") if n != name]
        for base in ("c2", "c3"):
            spec = W.make_batch(base, with_history=False, with_tensors=False)
            for inc in (1, 8, 16):
                todo.append(("%s_inc%d" % (base, inc), (base, (spec.cached_len, np.full_like(spec.new_len, inc)))))
        spec = W.make_batch("c4", with_history=False, with_tensors=False)
        for inc in (256, 1024):
            todo.append(("c4_inc%d" % inc, ("c4", (spec.cached_len, np.full_like(spec.new_len, inc)))))
        for label, over in todo:
            base, lengths = (label, None) if over is None else over
            d = DeviceBatch(torch, E, W, base, lengths=lengths, copies=3)
            extra[label] = summarize(d, time_parts(torch, E, d, iters=args.extra_iters, warmup=10))
            del d
            torch.cuda.empty_cache()
        result["workloads"] = extra
        result["service_replay"] = replay(torch, E, W, iters=max(5, args.extra_iters // 3))
        result["decode_step"] = decode_steps(torch, E, W, iters=args.extra_iters)
        result["fp8_kv_cache"] = fp8_cache(torch, E, W, iters=args.extra_iters)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, name)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
