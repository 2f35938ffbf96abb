#!/usr/bin/env python3
"""Decode-step benchmark of the four token mixers at batch 64 on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one new token for each of 64 sequences through one layer of every mixer at the paper's
15B-class shapes: a GDN step and a KDA step (32 heads, 128x128 fp32 state per head), full GQA
attention over 32768-token paged bf16 caches, and sliding-window attention (w = 4096) over the same
caches with context lengths uniform in [8192, 32768].  Inputs are synthetic, seeded and resident in
HBM before the timed region.  Prints ONE JSON line; `value` is sequences advanced per second through
that four-mixer layer set, `kernels` gives every kernel's own tokens/s and fraction of the 8 TB/s
HBM peak, `roofline` is the dominant kernel (the full-attention K/V stream).
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

HBM_PEAK_GBS = 8000.0
B, H, DK, DV = 64, 32, 128, 128
HQ, HKV, D, PAGE = 32, 8, 128, 16
CTX, WINDOW = 32768, 4096
N_STATE_SETS = 8      # 8 x 128 MiB per recurrent mixer: the working set exceeds the 256 MB last-level cache
N_RING = 8            # distinct pre-staged operand sets
# HBM bytes per launch of the full-attention split kernel (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the
# copy-kernel calibration) are read at run time from this summary, together with the hash of the sources it was taken on.
TRAFFIC_PROFILE = os.path.join("profiles", "batch64_step_all_kernels_hbm_bytes.txt")


def profiled_traffic():
    """(bytes per launch or None, where the figure comes from).  The summary carries two `name = value` lines:
    `fa_split_traffic_bytes` and `library_sources_sha16` (the sources the counters were collected on)."""
    from paper_2604_19877_amd.build import source_sha16
    src = {"file": TRAFFIC_PROFILE, "library_sources_sha16_now": source_sha16()}
    try:
        vals = {}
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
            for line in f:
                name, sep, val = line.partition("=")
                if sep and name.strip() in ("fa_split_traffic_bytes", "library_sources_sha16"):
                    vals[name.strip()] = val.strip()
        traffic = int(vals["fa_split_traffic_bytes"].replace(",", ""))
        src["library_sources_sha16_when_profiled"] = vals.get("library_sources_sha16")
        src["same_sources"] = src["library_sources_sha16_when_profiled"] == src["library_sources_sha16_now"]
        return traffic, src
    except (OSError, KeyError, ValueError) as e:
        src["error"] = "%s: %s" % (type(e).__name__, e)
        return None, src


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (for profiler runs)")
    ap.add_argument("--no-extras", action="store_true", help="skip batch 256, back-to-back and ragged-length cases")
    ap.add_argument("--no-verify", action="store_true", help="skip the 4-token verify measurements")
    ap.add_argument("--no-placement", action="store_true", help="skip the 48-layer placement stack at batch 128")
    ap.add_argument("--cost-table", action="store_true",
                    help="only fit the per-mixer cost model 1/throughput = sum_m c_m n_m over 14 allocations of a 48-layer "
                         "stack (batch 32, 16384-token contexts) and print it")
    ap.add_argument("--preset-speedups", action="store_true",
                    help="time the paper's recommended presets (layer counts per mixer) at 16384- and 32768-token contexts and print "
                         "their decode speedup over the all-FA preset, mixers only")
    ap.add_argument("--prefill", type=int, default=0, metavar="T",
                    help="only run the chunk-parallel recurrent kernels over T tokens per sequence (batch 64) and print their times")
    ap.add_argument("--literal-configs", action="store_true",
                    help="also run 256 GDN and 256 KDA steps on one 128 MiB state set (BASELINE configs 2 and 3 as written) when "
                         "--no-extras is given (profiler runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run the plain 1 GiB copy kernel 3 times after the timed region (counter calibration)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2604_19877_amd import binding as sa
    from paper_2604_19877_amd import inputs as gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    if args.cost_table:
        print(json.dumps(cost_table(np, torch, gen, stream)))
        return
    if args.preset_speedups:
        print(json.dumps(preset_speedups(torch, gen, stream)))
        return
    if args.prefill > 0:
        g = torch.Generator(device="cuda")
        g.manual_seed(1234)
        print(json.dumps({"workload": "chunk-parallel recurrent prefill, 64 sequences x 32 heads x %d tokens" % args.prefill,
                          **chunk_cases(torch, sa, args.prefill, DK ** -0.5, stream, g)}))
        return

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()

    # ---------------------------------------------------------------- recurrent operands and states
    g = torch.Generator(device="cuda")
    g.manual_seed(1002)
    rec = {}
    for name, kda in (("gdn", False), ("kda", True)):
        ring = [{n: dev(a) for n, a in gen.recurrent_inputs(1002 + 17 * i + kda, B, 1, H, H, DK, DV, kda).items()}
                for i in range(N_RING)]
        states = torch.empty((N_STATE_SETS, B * H, DK, DV), dtype=torch.float32, device="cuda")
        states.normal_(0.0, 0.02, generator=g)
        out = torch.empty((B, 1, H, DV), dtype=torch.float32, device="cuda")
        rec[name] = (ring, states, out)
    rec_scale = DK ** -0.5

    # ---------------------------------------------------------------- paged KV cache
    max_pages = CTX // PAGE
    table_h, n_pages = gen.page_table(1004, np.full(B, CTX, dtype=np.int32), max_pages)
    table = dev(table_h)
    kpool = torch.empty((n_pages, HKV, PAGE * D), dtype=torch.bfloat16, device="cuda")
    vpool = torch.empty((n_pages, HKV, PAGE * D), dtype=torch.bfloat16, device="cuda")
    kpool.normal_(generator=g)
    vpool.normal_(generator=g)
    lens_fa_h = np.full(B, CTX, dtype=np.int32)
    lens_swa_h = gen.context_lengths(1005, B, 8192, CTX)
    lens_fa, lens_swa = dev(lens_fa_h), dev(lens_swa_h)
    q_ring_h = [gen.attention_inputs(1006 + i, B, 1, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"] for i in range(N_RING)]
    q_ring = [dev(q) for q in q_ring_h]
    attn_scale = D ** -0.5
    ws_bytes = max(sa.attn_decode_workspace_bytes(B, 1, HQ, HKV, D, CTX, 0),
                   sa.attn_decode_workspace_bytes(B, 1, HQ, HKV, D, CTX, WINDOW))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    out_fa = torch.empty((B, 1, HQ, D), dtype=torch.float32, device="cuda")
    out_swa = torch.empty((B, 1, HQ, D), dtype=torch.float32, device="cuda")

    def step(i):
        for name, fn in (("gdn", sa.gdn_decode_step), ("kda", sa.kda_decode_step)):
            ring, states, out = rec[name]
            x, s = ring[i % N_RING], states[i % N_STATE_SETS]
            fn(x["q"], x["k"], x["v"], x["alpha"], x["beta"], s, s, out, None, None, 0, B, 1, H, H, DK, DV, rec_scale, 1,
               stream)
        q = q_ring[i % N_RING]
        sa.attn_decode(q, kpool, vpool, n_pages, table, max_pages, lens_fa, None, 0, out_fa, B, 1, HQ, HKV, D, PAGE, CTX, 0,
                       attn_scale, ws, ws_bytes, stream)
        sa.attn_decode(q, kpool, vpool, n_pages, table, max_pages, lens_swa, None, 0, out_swa, B, 1, HQ, HKV, D, PAGE, CTX,
                       WINDOW, attn_scale, ws, ws_bytes, stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    sa.sa_prof_enable(True)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sa.sa_prof_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    copy_entry = None
    if args.copy_calibration or not args.no_extras:   # the plain copy's GB/s is reported beside the kernels' as a reference
        n_copy = 1 << 30
        src = torch.empty(n_copy, dtype=torch.uint8, device="cuda")
        dst = torch.empty(n_copy, dtype=torch.uint8, device="cuda")
        src.random_(0, 255, generator=g)
        sa.sa_prof_enable(True)
        for _ in range(3):
            sa.sa_copy_bytes(src, dst, n_copy, stream)
        torch.cuda.synchronize()
        sa.sa_prof_enable(False)
        _, _, copy_ms = sa.sa_prof_read(sa.SA_K_COPY, 8)
        avg = sum(copy_ms) / len(copy_ms)
        copy_entry = {"avg_us": round(avg * 1e3, 2), "bytes_read_plus_written": 2 * n_copy,
                      "GBps": round(2 * n_copy / (avg * 1e-3) / 1e9, 1)}

    # ---------------------------------------------------------------- per-kernel durations (HIP events)
    cap = 2 * args.steps + 8
    _, _, gdn_ms = sa.sa_prof_read(sa.SA_K_GDN, cap)
    _, _, kda_ms = sa.sa_prof_read(sa.SA_K_KDA, cap)
    _, _, split_ms = sa.sa_prof_read(sa.SA_K_ATTN_SPLIT, cap)
    _, _, merge_ms = sa.sa_prof_read(sa.SA_K_ATTN_MERGE, cap)
    fa_ms, swa_ms = split_ms[0::2], split_ms[1::2]          # launch order within a step: FA, then SWA
    fa_merge_ms = merge_ms          # the windowed launch has one range per (request, KV head): no merge kernel

    state_bytes = 2 * B * H * DK * DV * 4
    rec_operands = B * (2 * H * DK * 2 + H * DV * 2 + H * DV * 4 + H * 4)     # q,k,v bf16, out fp32, beta
    alg = {
        "gdn_decode_step": state_bytes + rec_operands + B * H * 4,
        "kda_decode_step": state_bytes + rec_operands + B * H * DK * 4,
        "attn_split_fa": int(lens_fa_h.astype(np.int64).sum()) * 2 * HKV * D * 2,
        "attn_split_swa": int(np.minimum(lens_swa_h, WINDOW).astype(np.int64).sum()) * 2 * HKV * D * 2,
    }

    def entry(ms_list, nbytes):
        avg = sum(ms_list) / max(len(ms_list), 1)
        gbs = nbytes / (avg * 1e-3) / 1e9 if avg > 0 else 0.0
        return {"avg_us": round(avg * 1e3, 2), "min_us": round(min(ms_list) * 1e3, 2) if ms_list else None,
                "launches": len(ms_list), "alg_bytes": nbytes, "GBps": round(gbs, 1),
                "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "tokens_per_s": round(B / (avg * 1e-3), 1) if avg > 0 else None}

    kernels = {
        "gdn_decode_step": entry(gdn_ms, alg["gdn_decode_step"]),
        "kda_decode_step": entry(kda_ms, alg["kda_decode_step"]),
        "attn_split_fa": entry(fa_ms, alg["attn_split_fa"]),
        "attn_split_swa": entry(swa_ms, alg["attn_split_swa"]),
        "attn_merge_fa": {"avg_us": round(sum(fa_merge_ms) / max(len(fa_merge_ms), 1) * 1e3, 2), "launches": len(fa_merge_ms)},
    }
    if copy_entry:
        kernels["copy_1GiB"] = copy_entry
    dom = kernels["attn_split_fa"]
    traffic, traffic_source = profiled_traffic()
    roofline = {"kernel": "attn_split_kernel (full attention, 64 x 32768 tokens)", "bound": "hbm",
                "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom["frac_hbm_peak"],
                "traffic": traffic, "traffic_source": traffic_source, "algorithmic_bytes": dom["alg_bytes"]}

    # ---------------------------------------------------------------- 4-token verify step of every mixer
    verify = None
    if not args.no_verify:
        verify = verify_step(np, torch, sa, gen, dev, rec, kpool, vpool, n_pages, table, max_pages, lens_fa, lens_swa,
                             rec_scale, attn_scale, stream, alg)

    # ---------------------------------------------------------------- other configurations of the same kernels
    extras = None
    if not args.no_extras:
        extras = extra_cases(np, torch, sa, gen, dev, kpool, vpool, n_pages, table, max_pages, lens_swa, lens_swa_h,
                             rec_scale, attn_scale, stream, g)

    if extras:
        # what bare streams of the same access patterns reach on this machine in this run (no arithmetic): the practical ceiling
        roofline["ceiling"] = {
            "read_stream_GBps": extras["state_tiles_read_only_b64"]["GBps"],
            "read_write_stream_GBps": extras["state_tiles_read_write_only_b64"]["GBps"],
            "tile_copy_1GiB_GBps": kernels.get("copy_1GiB", {}).get("GBps"),
            "note": "sa_stream_tiles over 128 MiB of 64 KiB tiles (read only / read, scale, write back) and sa_copy_bytes "
                    "over 1 GiB (64 KiB tiles, non-temporal), kernel-attached events; frac_of_read_stream = achieved / read_stream"}
        roofline["ceiling"]["frac_of_read_stream"] = round(dom["GBps"] / roofline["ceiling"]["read_stream_GBps"], 4)

    if extras is None and args.literal_configs:
        extras = literal_state_set_cases(torch, sa, gen, dev, rec_scale, stream, g)

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = cpu_numpy = None
    if not args.no_cpu_baseline:
        cpu, cpu_numpy = cpu_baseline(np, torch, gen, rec, q_ring_h[0], kpool, vpool, table_h, lens_fa_h, lens_swa_h, rec_scale,
                                      attn_scale)

    # ---------------------------------------------------------------- 48-layer placement stack (batch 128)
    placement = None
    if not args.no_placement:
        del kpool, vpool, rec
        torch.cuda.empty_cache()
        placement = placement_stack(torch, sa, stream)
        torch.cuda.empty_cache()
        scattered = placement_stack(torch, sa, stream, page_scatter="global")
        placement["pages_shuffled_over_the_whole_pool"] = {k: scattered[k] for k in ("ms_per_step", "tokens_per_s", "frac_hbm_peak")}
        placement["launch_bound_case"] = small_stack_graph(torch)
        torch.cuda.empty_cache()
        # Section 4 "Cost model" on this GPU, mixers only: 1/throughput = sum_m c_m n_m fitted on 7 allocations (the four
        # pure stacks and three mixed ones); --cost-table fits 14
        placement["cost_model"] = cost_table(np, torch, gen, stream, steps=4, allocations=SHORT_ALLOCATIONS)

    line = {
        "metric": "mixer decode tokens/s at batch 64 + % of MI355X peak HBM GB/s",
        "value": round(B / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "operand_dtype": "bf16 (q, k, v, KV cache); fp32 states, gates and outputs",
        "data": "synthetic",
        "config": {"workload": "batch-64 decode step through one GDN, one KDA, one FA (32768-token contexts) and one SWA "
                               "(w=4096, contexts U[8192,32768]) layer; 32 heads, 128x128 fp32 states, 32q/8kv heads, "
                               "head dim 128, 16-token pages, shuffled page table",
                   "batch": B, "state_sets_rotated": N_STATE_SETS},
        "hbm_frac_by_kernel": {k: v["frac_hbm_peak"] for k, v in kernels.items() if "frac_hbm_peak" in v},
        "kernels": kernels,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "cpu_baseline_numpy": cpu_numpy,
        "placement48": placement,
        "verify": verify,
        "extras": extras,
    }
    print(json.dumps(line))


def verify_step(np, torch, sa, gen, dev, rec, kpool, vpool, n_pages, table, max_pages, lens_fa, lens_swa, rec_scale,
                attn_scale, stream, alg, reps=9):
    """Multi-token verify for self-speculative decoding: 4 and 8 drafted tokens per sequence scored in one pass
    of each mixer at the batch-64 shapes (same state / KV bytes as a single-token step).  Median of the launches
    after the first: the first launches of a kernel variant after a change of workload run several per cent slow."""
    res = {}

    def median(ms):
        tail = sorted(ms[1:])
        return tail[len(tail) // 2]

    for T in (4, 8):
        for name, kda, fn, kids in (("gdn", False, sa.gdn_decode_step, (sa.SA_K_GDN, sa.SA_K_GDN_CHUNK)),
                                    ("kda", True, sa.kda_decode_step, (sa.SA_K_KDA, sa.SA_K_KDA_CHUNK))):
            x = {n: dev(a) for n, a in gen.recurrent_inputs(1900 + kda + T, B, T, H, H, DK, DV, kda).items()}
            states = rec[name][1]
            out = torch.empty((B, T, H, DV), dtype=torch.float32, device="cuda")
            sa.sa_prof_enable(True)
            for i in range(reps):   # out of place: draft state kept, all T steps committed to the next set
                fn(x["q"], x["k"], x["v"], x["alpha"], x["beta"], states[i % N_STATE_SETS], states[(i + 1) % N_STATE_SETS], out,
                   None, None, 0, B, T, H, H, DK, DV, rec_scale, T, stream)
            torch.cuda.synchronize()
            sa.sa_prof_enable(False)
            ms = [t for kid in kids for t in sa.sa_prof_read(kid, reps)[2]]   # 5 tokens and more run on the chunk kernels
            avg = median(ms)
            one = alg[name + "_decode_step"]
            # a pass over T tokens moves the state once and the per-token operands and outputs T times
            nbytes = 2 * B * H * DK * DV * 4 + T * (one - 2 * B * H * DK * DV * 4)
            res["%s_T%d" % (name, T)] = {"median_us": round(avg * 1e3, 2), "tokens_per_s": round(B * T / (avg * 1e-3), 1),
                                         "alg_bytes": nbytes, "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                         "frac_hbm_peak_on_one_token_bytes": round(one / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        q = dev(gen.attention_inputs(1910 + T, B, T, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"])
        ws_bytes = max(sa.attn_decode_workspace_bytes(B, T, HQ, HKV, D, CTX, 0),
                       sa.attn_decode_workspace_bytes(B, T, HQ, HKV, D, CTX, WINDOW))
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        out = torch.empty((B, T, HQ, D), dtype=torch.float32, device="cuda")
        for name, lens, window in (("fa", lens_fa, 0), ("swa", lens_swa, WINDOW)):
            sa.sa_prof_enable(True)
            for _ in range(reps):
                sa.attn_decode(q, kpool, vpool, n_pages, table, max_pages, lens, None, 0, out, B, T, HQ, HKV, D, PAGE, CTX, window,
                               attn_scale, ws, ws_bytes, stream)
            torch.cuda.synchronize()
            sa.sa_prof_enable(False)
            _, _, ms = sa.sa_prof_read(sa.SA_K_ATTN_SPLIT, reps)
            sa.sa_prof_read(sa.SA_K_ATTN_MERGE, reps)
            avg = median(ms)
            nbytes = alg["attn_split_" + name]
            res["%s_T%d" % (name, T)] = {"median_us": round(avg * 1e3, 2), "tokens_per_s": round(B * T / (avg * 1e-3), 1),
                                         "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    return res


def extra_cases(np, torch, sa, gen, dev, kpool, vpool, n_pages, table, max_pages, lens_swa, lens_swa_h, rec_scale, attn_scale,
                stream, g, reps=24):
    """Batch 256 for the recurrent mixers (bandwidth saturation), the recurrent steps launched back to back
    (no read-only kernel in between to hide their write-back), the whole-block step, the chunk-parallel kernels
    at 16 to 512 tokens per sequence, and full attention at ragged lengths."""
    res = {}
    for nb, sets in ((256, 4), (64, 8)):
        for name, kda, fn, kid in (("gdn", False, sa.gdn_decode_step, sa.SA_K_GDN), ("kda", True, sa.kda_decode_step, sa.SA_K_KDA)):
            x = {n: dev(a) for n, a in gen.recurrent_inputs(1800 + kda + nb, nb, 1, H, H, DK, DV, kda).items()}
            states = torch.empty((sets, nb * H, DK, DV), dtype=torch.float32, device="cuda")
            states.normal_(0.0, 0.02, generator=g)
            out = torch.empty((nb, 1, H, DV), dtype=torch.float32, device="cuda")
            # one untimed pass over every state set first: the first step over a freshly filled set runs 5-20 % slow
            # (batch 64: 47-53 us against 43-44 us for every later one), which is the fill's doing, not the kernel's
            for i in range(sets + reps):
                if i == sets:
                    torch.cuda.synchronize()
                    sa.sa_prof_enable(True)
                s = states[i % sets]
                fn(x["q"], x["k"], x["v"], x["alpha"], x["beta"], s, s, out, None, None, 0, nb, 1, H, H, DK, DV, rec_scale, 1,
                   stream)
            torch.cuda.synchronize()
            sa.sa_prof_enable(False)
            _, _, ms = sa.sa_prof_read(kid, reps)
            avg = sum(ms[2:]) / (len(ms) - 2)
            nbytes = 2 * nb * H * DK * DV * 4 + nb * (2 * H * DK * 2 + H * DV * 2 + H * DV * 4 + H * 4) + \
                nb * H * (DK if kda else 1) * 4
            res["%s_b%d_back_to_back" % (name, nb)] = {
                "avg_us": round(avg * 1e3, 2), "tokens_per_s": round(nb / (avg * 1e-3), 1),
                "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            if kda and nb == 64:
                # what the step's access pattern reaches with no arithmetic: the same tiles read only, written only,
                # and read + written back, launched back to back like the steps above
                tile_bytes = nb * H * DK * DV * 4
                for kind, label, passes in ((0, "read", 1), (1, "write", 1), (2, "read_write", 2)):
                    sa.sa_prof_enable(True)
                    for i in range(reps):
                        sa.sa_stream_tiles(kind, states[i % sets], nb * H, stream)
                    torch.cuda.synchronize()
                    sa.sa_prof_enable(False)
                    _, _, ms = sa.sa_prof_read(sa.SA_K_STREAM, reps)
                    avg = sum(ms[2:]) / (len(ms) - 2)
                    res["state_tiles_%s_only_b64" % label] = {
                        "avg_us": round(avg * 1e3, 2), "bytes": passes * tile_bytes,
                        "GBps": round(passes * tile_bytes / (avg * 1e-3) / 1e9, 1),
                        "frac_hbm_peak": round(passes * tile_bytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            del states
    res.update(literal_state_set_cases(torch, sa, gen, dev, rec_scale, stream, g))
    # whole-block step: convolution + SiLU, L2 norm, gates, state update and gated RMS norm in one launch
    for name, kda, fn, kid in (("gdn", False, sa.gdn_block_decode, sa.SA_K_GDN_BLOCK), ("kda", True, sa.kda_block_decode, sa.SA_K_KDA_BLOCK)):
        taps, sets = 4, 8
        hp = gen.block_inputs(1830 + kda, B, H, H, DK, DV, taps, kda)
        x = {n: dev(a) for n, a in hp.items()}
        io = sa.make_block_io(xq=x["xq"], xk=x["xk"], xv=x["xv"], wq=x["wq"], wk=x["wk"], wv=x["wv"], conv_q_in=x["conv_q"],
                              conv_k_in=x["conv_k"], conv_v_in=x["conv_v"], conv_q_out=x["conv_q"], conv_k_out=x["conv_k"],
                              conv_v_out=x["conv_v"], conv_taps=taps, beta_raw=x["beta_raw"], alpha_raw=x["alpha_raw"],
                              A_log=x["A_log"], dt_bias=x["dt_bias"], z=x["z"], norm_weight=x["norm_weight"], norm_eps=1e-5,
                              gate_act=0)
        states = torch.empty((sets, B * H, DK, DV), dtype=torch.float32, device="cuda")
        states.normal_(0.0, 0.02, generator=g)
        out = torch.empty((B, H, DV), dtype=torch.float32, device="cuda")
        sa.sa_prof_enable(True)
        for i in range(reps):
            s = states[i % sets]
            fn(io, s, s, out, None, None, 0, B, H, H, DK, DV, rec_scale, stream)
        torch.cuda.synchronize()
        sa.sa_prof_enable(False)
        _, _, ms = sa.sa_prof_read(kid, reps)
        avg = sum(ms[2:]) / (len(ms) - 2)
        nbytes = 2 * B * H * DK * DV * 4 + sum(a.nbytes for n, a in hp.items() if n[0] in "xz") + \
            2 * sum(hp[n].nbytes for n in ("conv_q", "conv_k", "conv_v")) + B * H * DV * 4
        res["%s_block_b64_back_to_back" % name] = {
            "avg_us": round(avg * 1e3, 2), "tokens_per_s": round(B / (avg * 1e-3), 1), "alg_bytes": nbytes,
            "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del states
    # many tokens per state pass (prefill-like): the chunk-parallel kernels at 16, 64 and 512 tokens per sequence
    for T in (16, 64, 512):
        res.update(chunk_cases(torch, sa, T, rec_scale, stream, g))
    q = dev(gen.attention_inputs(1820, B, 1, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"])
    ws_bytes = sa.attn_decode_workspace_bytes(B, 1, HQ, HKV, D, CTX, 0)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    out = torch.empty((B, 1, HQ, D), dtype=torch.float32, device="cuda")
    sa.sa_prof_enable(True)
    for _ in range(reps):
        sa.attn_decode(q, kpool, vpool, n_pages, table, max_pages, lens_swa, None, 0, out, B, 1, HQ, HKV, D, PAGE, CTX, 0,
                       attn_scale, ws, ws_bytes, stream)
    torch.cuda.synchronize()
    sa.sa_prof_enable(False)
    _, _, ms = sa.sa_prof_read(sa.SA_K_ATTN_SPLIT, reps)
    sa.sa_prof_read(sa.SA_K_ATTN_MERGE, reps)
    avg = sum(ms[2:]) / (len(ms) - 2)
    nbytes = int(lens_swa_h.astype(np.int64).sum()) * 2 * HKV * D * 2
    res["fa_ragged_U8192_32768"] = {"avg_us": round(avg * 1e3, 2), "tokens_per_s": round(B / (avg * 1e-3), 1),
                                    "alg_bytes": nbytes, "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    # the same full-attention step through a regular page table (every sequence's pages in a row): what a freshly filled
    # cache looks like, and the pattern that concentrates on few memory channels unless workgroups are staggered
    lens_full = torch.full((B,), CTX, dtype=torch.int32, device="cuda")
    rows_table = torch.arange(B * max_pages, dtype=torch.int32, device="cuda").reshape(B, max_pages)
    sa.sa_prof_enable(True)
    for _ in range(reps):
        sa.attn_decode(q, kpool, vpool, n_pages, rows_table, max_pages, lens_full, None, 0, out, B, 1, HQ, HKV, D, PAGE, CTX, 0,
                       attn_scale, ws, ws_bytes, stream)
    torch.cuda.synchronize()
    sa.sa_prof_enable(False)
    _, _, ms = sa.sa_prof_read(sa.SA_K_ATTN_SPLIT, reps)
    sa.sa_prof_read(sa.SA_K_ATTN_MERGE, reps)
    avg = sum(ms[2:]) / (len(ms) - 2)
    nbytes = B * CTX * 2 * HKV * D * 2
    res["fa_32768_pages_in_a_row"] = {"avg_us": round(avg * 1e3, 2), "tokens_per_s": round(B / (avg * 1e-3), 1),
                                      "alg_bytes": nbytes, "frac_hbm_peak": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    return res


def literal_state_set_cases(torch, sa, gen, dev, rec_scale, stream, g, n_steps=256):
    """BASELINE configs 2 and 3 to the letter: 256 consecutive steps on ONE state set (128 MiB, which fits the 256 MB
    last-level cache) with fresh operands per step, beside the rotation over 8 sets that the headline figures use."""
    res = {}
    for name, kda, fn, kid in (("gdn", False, sa.gdn_decode_step, sa.SA_K_GDN), ("kda", True, sa.kda_decode_step, sa.SA_K_KDA)):
        ring = [{n: dev(a) for n, a in gen.recurrent_inputs(1850 + 7 * i + kda, B, 1, H, H, DK, DV, kda).items()} for i in range(N_RING)]
        state = torch.empty((B * H, DK, DV), dtype=torch.float32, device="cuda")
        state.normal_(0.0, 0.02, generator=g)
        out = torch.empty((B, 1, H, DV), dtype=torch.float32, device="cuda")
        sa.sa_prof_enable(True)
        for i in range(n_steps):
            x = ring[i % N_RING]
            fn(x["q"], x["k"], x["v"], x["alpha"], x["beta"], state, state, out, None, None, 0, B, 1, H, H, DK, DV, rec_scale, 1, stream)
        torch.cuda.synchronize()
        sa.sa_prof_enable(False)
        _, _, ms = sa.sa_prof_read(kid, n_steps)
        avg = sum(ms[8:]) / (len(ms) - 8)
        nbytes = 2 * B * H * DK * DV * 4 + B * (2 * H * DK * 2 + H * DV * 2 + H * DV * 4 + H * 4) + B * H * (DK if kda else 1) * 4
        res["%s_b64_one_state_set_256_steps" % name] = {
            "avg_us": round(avg * 1e3, 2), "min_us": round(min(ms) * 1e3, 2), "tokens_per_s": round(B / (avg * 1e-3), 1),
            "frac_hbm_peak_if_all_bytes_came_from_hbm": round(nbytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "the same 128 MiB of states re-stepped while it may still sit in the 256 MB last-level cache"}
        del state, ring
    return res


def chunk_cases(torch, sa, T, rec_scale, stream, g, reps=6):
    """gdn_chunk_steps / kda_chunk_steps over T tokens for each of 64 sequences x 32 heads; inputs drawn on the
    device with the recipe's distributions, states rotating over 4 sets."""
    res = {}
    nrm = lambda x: (x / x.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    xq = nrm(torch.empty((B, T, H, DK), device="cuda").normal_(generator=g).bfloat16().float())
    xk = nrm(torch.empty((B, T, H, DK), device="cuda").normal_(generator=g).bfloat16().float())
    xv = torch.empty((B, T, H, DV), device="cuda").normal_(generator=g).bfloat16()
    beta = torch.sigmoid(torch.empty((B, T, H), device="cuda").normal_(generator=g))
    states = torch.empty((4, B * H, DK, DV), dtype=torch.float32, device="cuda")
    states.normal_(0.0, 0.02, generator=g)
    out = torch.empty((B, T, H, DV), dtype=torch.float32, device="cuda")
    for name, kda, fn, kid in (("gdn", False, sa.gdn_chunk_steps, sa.SA_K_GDN_CHUNK),
                               ("kda", True, sa.kda_chunk_steps, sa.SA_K_KDA_CHUNK)):
        alpha = torch.exp(-torch.nn.functional.softplus(
            torch.empty((B, T, H, DK) if kda else (B, T, H), device="cuda").normal_(generator=g) + 2.0))
        sa.sa_prof_enable(True)
        for i in range(reps):
            s = states[i % 4]
            fn(xq, xk, xv, alpha, beta, s, s, out, None, None, 0, B, T, H, H, DK, DV, rec_scale, stream=stream)
        torch.cuda.synchronize()
        sa.sa_prof_enable(False)
        _, _, ms = sa.sa_prof_read(kid, reps)
        avg = sum(ms[2:]) / (len(ms) - 2)
        res["%s_chunk_T%d" % (name, T)] = {"avg_us": round(avg * 1e3, 2), "us_per_token": round(avg * 1e3 / T, 3),
                                           "tokens_per_s": round(B * T / (avg * 1e-3), 1)}
        del alpha
    return res


SHORT_ALLOCATIONS = [(48, 0, 0, 0), (0, 48, 0, 0), (0, 0, 48, 0), (0, 0, 0, 48), (24, 24, 0, 0), (12, 12, 12, 12), (0, 16, 16, 16)]


def cost_table(np, torch, gen, stream, batch=32, ctx=16384, steps=6, allocations=None):
    """The paper's linear cost model (Section 4, "Cost model": 1/throughput = sum over mixers of c_m * n_m,
    fitted on measured placements) for the mixers-only stack on this GPU: all requests of a batch share one
    placement, as in the paper's single-preset measurements."""
    from paper_2604_19877_amd.workloads import PlacementWorkload
    if allocations is None:
        allocations = [(48, 0, 0, 0), (0, 48, 0, 0), (0, 0, 48, 0), (0, 0, 0, 48), (24, 24, 0, 0), (24, 0, 24, 0), (24, 0, 0, 24),
                       (12, 12, 12, 12), (0, 16, 16, 16), (6, 30, 6, 6), (3, 25, 4, 16), (0, 10, 5, 33), (12, 26, 6, 4), (0, 30, 5, 13)]
    rows, times = [], []
    for i, (f, s_, k, g_) in enumerate(allocations):
        placement = gen.placement_string(6000 + i, 48, {"F": f, "S": s_, "K": k, "G": g_})
        w = PlacementWorkload(B=batch, L=48, ctx=ctx, window=WINDOW, T=1, seed=6100 + i, placements=[placement])
        try:
            for _ in range(2):
                w.step(stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                w.step(stream)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
        finally:
            w.close()
        del w
        torch.cuda.empty_cache()
        rows.append((f, s_, k, g_))
        times.append(ms * 1e-3 / batch)                      # seconds per token = 1 / throughput
    A, y = np.array(rows, dtype=np.float64), np.array(times)
    c, *_ = np.linalg.lstsq(A, y, rcond=None)
    pred = A @ c
    r2 = 1.0 - float(np.sum((y - pred) ** 2) / np.sum((y - y.mean()) ** 2))
    return {"workload": "48-layer mixers-only stack, batch %d, contexts %d, one placement per run, w=%d" % (batch, ctx, WINDOW),
            "allocations_F_S_K_G": rows, "ms_per_step": [round(t * batch * 1e3, 3) for t in times],
            "cost_us_per_layer_per_token": dict(zip("FSKG", [round(float(x) * 1e6, 4) for x in c])),
            "relative_cost": dict(zip(["FA", "SWA", "KDA", "GDN"], [round(float(x / c[0]), 4) for x in c])),
            "r2": round(r2, 5), "mean_abs_rel_err": round(float(np.mean(np.abs(pred - y) / y)), 4),
            "paper_relative_cost_context_only": {"FA": 1.0, "SWA": 0.48, "KDA": 0.21, "GDN": 0.14,
                                                 "note": "1xH100, whole 15B model incl. FFNs, vLLM, 16k, regression over 84 placements"}}


def preset_speedups(torch, gen, stream, batch=32, contexts=(16384, 32768), steps=6):
    """Decode speedup of the paper's recommended presets over its all-FA preset at 16384- and 32768-token contexts
    (Section 7, "Placement Presets": layer counts per mixer; the appendix table of full results: speedups at 16k and
    32k), for the mixers alone on this GPU: all requests share the preset, as in the paper's single-preset
    measurements; which layers get which mixer is a seeded shuffle (time depends on the counts only)."""
    from paper_2604_19877_amd.workloads import PlacementWorkload
    presets = [("all-FA", (48, 0, 0, 0), {16384: 1.0, 32768: 1.0}), ("Reg|Lklhd-26", (12, 26, 6, 4), {16384: 1.5, 32768: 2.85}),
               ("Reg|Lklhd-18", (3, 25, 4, 16), {16384: 2.2, 32768: 4.76}), ("Reg|Lklhd-13", (0, 16, 13, 19), {16384: 2.7, 32768: 6.9}),
               ("Reg|Lklhd-10", (0, 10, 5, 33), {16384: 4.2, 32768: 10.69}), ("Idealized|All-18", (13, 32, 1, 2), {16384: 1.1, 32768: 1.99}),
               ("Idealized|Lklhd-6 / All-6", (0, 30, 5, 13), {16384: 2.4, 32768: 6.2})]
    tables = []
    for ctx in contexts:
        rows = []
        for i, (name, (f, s_, k, g_), paper) in enumerate(presets):
            placement = gen.placement_string(6300 + i, 48, {"F": f, "S": s_, "K": k, "G": g_})
            w = PlacementWorkload(B=batch, L=48, ctx=ctx, window=WINDOW, T=1, seed=6400 + i, placements=[placement])
            try:
                for _ in range(2):
                    w.step(stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    w.step(stream)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / steps
                nbytes = w.algorithmic_bytes()
            finally:
                w.close()
            del w
            torch.cuda.empty_cache()
            rows.append({"preset": name, "layers_F_S_K_G": [f, s_, k, g_], "ms_per_step": round(ms, 3),
                         "tokens_per_s": round(batch / (ms * 1e-3), 1), "alg_bytes": nbytes,
                         "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "paper_speedup_context_only": paper.get(ctx)})
        base_ms, base_bytes = rows[0]["ms_per_step"], rows[0]["alg_bytes"]
        for r in rows:
            r["speedup_over_all_FA"] = round(base_ms / r["ms_per_step"], 2)
            r["speedup_from_bytes_alone"] = round(base_bytes / r["alg_bytes"], 2)
        tables.append({"workload": "48-layer mixers-only stack, batch %d, contexts %d, w=%d, one preset per run" % (batch, ctx, WINDOW),
                       "context": ctx, "presets": rows})
    return {"tables": tables,
            "paper_note": "the paper's speedups are decode throughput of the whole 15B model (FFNs, sampler, scheduler) under vLLM "
                          "on 1xH100; here only the token mixers run"}


def placement_stack(torch, sa, stream, steps=8, warmup=2, page_scatter="layer"):
    """One decode step of the 48-layer mixers-only stack at batch 128, 16384-token contexts, three
    placements of 12 FA / 12 SWA / 12 KDA / 12 GDN layers assigned per request."""
    from paper_2604_19877_amd.workloads import PlacementWorkload
    w = PlacementWorkload(B=128, L=48, ctx=16384, window=WINDOW, T=1, seed=5000, page_scatter=page_scatter)
    try:
        for _ in range(warmup):
            w.step(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.step(stream)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        nbytes = w.algorithmic_bytes()
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"workload": "48-layer mixers-only stack, batch 128, contexts 16384, 3 placements (12 FA/12 SWA/12 KDA/12 GDN "
                            "each) assigned per request, one global paged KV pool (%s), bounded SWA caches"
                            % ("every layer's pages shuffled inside a region of its own" if page_scatter == "layer"
                               else "all layers' pages shuffled over the whole pool"),
                "ms_per_step": round(ms, 3), "tokens_per_s": round(w.B / (ms * 1e-3), 1), "steps": steps,
                "alg_bytes": nbytes, "GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                "kv_pool_GiB": round(2 * w.n_pages * HKV * PAGE * D * 2 / 2 ** 30, 1)}
    finally:
        w.close()


def small_stack_graph(torch, steps=20, warmup=3):
    """The launch-bound end of the same path: the 48-layer stack at batch 8 with 2048-token contexts moves so few
    bytes that issuing its ~190 kernels costs more than running them; the step is captured into a HIP graph once
    (the hot calls only enqueue kernels) and replayed."""
    from paper_2604_19877_amd.workloads import PlacementWorkload
    w = PlacementWorkload(B=8, L=48, ctx=2048, window=1024, T=1, seed=5100)
    try:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for _ in range(warmup):
                w.step(side)
            side.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                w.step(side)
            side.synchronize()
            eager_ms = (time.perf_counter() - t0) * 1e3 / steps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            w.step(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        nbytes = w.algorithmic_bytes()
        res = {"workload": "48-layer mixers-only stack, batch 8, contexts 2048, window 1024, 3 placements",
               "eager_ms_per_step": round(eager_ms, 3), "graph_ms_per_step": round(graph_ms, 3), "alg_bytes": nbytes,
               "graph_frac_hbm_peak": round(nbytes / (graph_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    finally:
        w.close()
    # the same stack as a verify pass over 4 drafted tokens per request
    w = PlacementWorkload(B=8, L=48, ctx=2048, window=1024, T=4, seed=5100)
    try:
        s = torch.cuda.current_stream()
        for _ in range(warmup):
            w.step(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.step(s)
        torch.cuda.synchronize()
        res["verify_T4_eager_ms_per_pass"] = round((time.perf_counter() - t0) * 1e3 / steps, 3)
    finally:
        w.close()
    return res


def cpu_baseline(np, torch, gen, rec, q_h, kpool, vpool, table_h, lens_fa_h, lens_swa_h, rec_scale, attn_scale):
    """The oracle, as it stands, timed on the host's cores on a sample of the same step and scaled to the full step:
    `cpu_baseline` is its fp64 C / OpenMP form (oracle/mixers_omp.c, all cores; admitted by tests/test_oracle_omp.py
    only while it agrees with the numpy oracle to 1e-12), `cpu_baseline_numpy` the numpy oracle itself."""
    from oracle import kv_layout as kl
    from oracle import mixers as om
    from oracle import omp

    tbl = torch.from_numpy(table_h).cuda()

    def host_pools(seqs, lens):
        """The pages of the sampled sequences as compact host pools (physical in-page order) with their page table."""
        ks, vs, rows, at = [], [], np.full((len(seqs), table_h.shape[1]), -1, dtype=np.int32), 0
        for i, b in enumerate(seqs):
            n = (int(lens[b]) + PAGE - 1) // PAGE
            pages = tbl[b, :n].long()
            ks.append(kpool[pages].view(torch.int16).cpu().numpy().view(np.uint16))
            vs.append(vpool[pages].view(torch.int16).cpu().numpy().view(np.uint16))
            rows[i, :n] = np.arange(at, at + n, dtype=np.int32)
            at += n
        return np.concatenate(ks), np.concatenate(vs), rows

    # ---- C / OpenMP twin: both recurrent steps on all 64 sequences, FA and SWA on 32 of the 64 sequences (all KV heads)
    n_seq_attn = 32
    t_omp = {}
    for name, kda, fn in (("gdn", False, omp.gdn_steps), ("kda", True, omp.kda_steps)):
        p = gen.recurrent_inputs(1002 + kda, B, 1, H, H, DK, DV, kda)
        S0 = rec[name][1][0].view(B, H, DK, DV).cpu().numpy()
        t = time.perf_counter()
        fn(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, rec_scale)
        t_omp[name] = time.perf_counter() - t
    seqs = list(range(0, B, B // n_seq_attn))
    for name, lens, window in (("fa", lens_fa_h, 0), ("swa", lens_swa_h, WINDOW)):
        kph, vph, rows = host_pools(seqs, lens)
        t = time.perf_counter()
        omp.attn_decode(q_h[seqs], kph, vph, rows, lens[seqs], window, attn_scale, physical=True)
        t_omp[name] = (time.perf_counter() - t) * (B / len(seqs))
        del kph, vph
    t_step = sum(t_omp.values())
    fast = {"value": round(B / t_step, 3), "unit": "tokens/s", "cores": omp.threads(), "kind": "oracle",
            "host_cores_available": len(os.sched_getaffinity(0)),
            "sample": "fp64 C/OpenMP form of the oracle (plain loops, parallel over (sequence, head)): one GDN and one KDA step "
                      "on all 64 sequences, FA and SWA on %d of the 64 sequences (all 8 KV heads) scaled to 64" % len(seqs),
            "seconds_per_full_step_extrapolated": round(t_step, 3),
            "seconds_by_mixer": {k: round(v, 3) for k, v in t_omp.items()}}

    # ---- the numpy oracle itself
    n_seq, n_groups = 64, 96   # about 8 s of numpy work on the host
    t_rec = {}
    for name, kda, fn in (("gdn", False, om.gdn_steps), ("kda", True, om.kda_steps)):
        p = gen.recurrent_inputs(1002 + kda, B, 1, H, H, DK, DV, kda)
        S0 = rec[name][1][0].view(B, H, DK, DV)[:n_seq].cpu().numpy()
        t = time.perf_counter()
        fn(p["q"][:n_seq], p["k"][:n_seq], p["v"][:n_seq], p["alpha"][:n_seq], p["beta"][:n_seq], S0, rec_scale)
        t_rec[name] = (time.perf_counter() - t) * (B / n_seq)
    t_attn = {}
    rng = np.random.default_rng(77)
    for name, lens, window in (("fa", lens_fa_h, 0), ("swa", lens_swa_h, WINDOW)):
        total = 0.0
        for _ in range(n_groups):
            b, grp = int(rng.integers(B)), int(rng.integers(HKV))
            L = int(lens[b])
            pages = tbl[b, :(L + PAGE - 1) // PAGE].long()
            kph = kpool[pages, grp].view(torch.int16).cpu().numpy().view(np.uint16)[:, None]
            vph = vpool[pages, grp].view(torch.int16).cpu().numpy().view(np.uint16)[:, None]
            klog, vlog = kl.to_logical(kph, vph, D)
            ident = np.arange(len(pages), dtype=np.int32)[None]
            heads = slice(grp * (HQ // HKV), (grp + 1) * (HQ // HKV))
            qs = q_h[b:b + 1, :, heads]
            t = time.perf_counter()
            om.attn_decode(qs, klog, vlog, ident, [L], window, attn_scale)   # 4 query heads on one KV head
            total += time.perf_counter() - t
        t_attn[name] = total * (B * HKV / n_groups)
    t_step = t_rec["gdn"] + t_rec["kda"] + t_attn["fa"] + t_attn["swa"]
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = 1
    slow = {"value": round(B / t_step, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "numpy fp64 oracle timed on %d of 64 sequences (all 32 heads) for one GDN and one KDA step and on "
                      "%d of 512 (sequence, KV head) groups (4 query heads each) for FA and for SWA, each scaled to the "
                      "full step; its einsum parts run on one thread, only matrix-vector products use the BLAS threads counted "
                      "in `cores`" % (n_seq, n_groups),
            "seconds_per_full_step_extrapolated": round(t_step, 2)}
    return fast, slow


if __name__ == "__main__":
    main()
