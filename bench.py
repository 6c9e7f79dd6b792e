#!/usr/bin/env python3
"""Benchmark of the prefix-cached extend-prefill hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch already resident in HBM:
match_prefixes -> extend_attention -> append_kv.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload agent_tree]

value      extend (newly prefilled) tokens per second over the whole step, on --workload (default: agent_tree,
           the largest of the configurations: 128 requests, 74 k new tokens, 2.9 TFLOP of attention)
roofline   the extend-attention kernel against the roof that binds it for this workload:
           algorithmic bytes or flops per launch / average kernel time from HIP events
configs    the same measurement, shorter, on each of the four bf16 configurations (tool use, long-document QA,
           agent tree, video QA): step time, per-kernel times, both roofline fractions; and on long-document QA
           with the KV pool in its fp8 form (--kv-pool fp8 makes that the headline's pool)
cpu_baseline  the CPU oracle, as it stands, on a bounded sample of the headline workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3
BF16_CONFIGS = ["tool_use", "long_doc_qa", "agent_tree", "video_qa"]
FP8_POOL_CONFIGS = ["long_doc_qa"]   # measured once more with the KV pool held in 8 bits per element

# HBM bytes per launch of the extend-attention kernel, measured with rocprofv3 --pmc in runs of their own (a counter
# run cannot share a process with the timed one): FETCH_SIZE x the factor that the same counter shows for append_kv, a
# plain copy of known size, + WRITE_SIZE x its factor (KiB).  The runs are summarised in
# profiles/extend_attention_<workload>.md, which is the source named beside each figure.  None = not measured.
MEASURED_TRAFFIC_BYTES = {"tool_use": 199_497_651, "agent_tree": 2_460_216_010, "long_doc_qa": 451_358_556,
                          "video_qa": 346_810_464, "programming": 231_169_958, "decode": 300_863_715,
                          "long_doc_qa_fp8_pool": 294_184_352}


def algorithmic_work(wl, prefix_len):
    """Algorithmic bytes and flops of one extend-attention launch.

    bytes: each request reads its own prefix K and V rows once per KV head (no credit for sharing
    between requests), its slot ids, and q/k_ext/v_ext once; out is written once.
    flops: QK^T and PV on visible (query, key) pairs only.
    """
    import numpy as np
    el = 4 if wl.dtype == "f32" else 2
    P = prefix_len.astype(np.int64)
    E = wl.ext_len.astype(np.int64)
    T = int(E.sum())
    kv_bytes = int(P.sum()) * wl.Hkv * wl.D * el * 2
    if wl.dtype == "bf16_kv8":   # a pool row is D one-byte codes and one exponent byte
        kv_bytes = int(P.sum()) * wl.Hkv * (wl.D + 1) * 2
    slot_bytes = 4 * int(P.sum())
    io_bytes = T * (2 * wl.Hq * wl.D * el + 2 * wl.Hkv * wl.D * el)
    flops = 4 * wl.D * wl.Hq * int((E * P + E * (E + 1) // 2).sum())
    return kv_bytes + slot_bytes + io_bytes, flops


def workspace_traffic(wl, hdr):
    """Bytes the launch moves through its workspace beyond the algorithmic ones: every part of a row tile whose key
    range was split writes fp32 partial outputs and (maximum, sum) for its 128 rows and every KV head, and the merge
    kernel reads them back (counted with all 128 rows of a tile in use).  hdr = (row tiles, items, tiles merged)."""
    n_tiles, n_items, n_merge = hdr[:3]
    split_items = n_items - (n_tiles - n_merge)
    return 2 * split_items * wl.Hkv * 128 * (wl.D + 2) * 4


def cpu_baseline(wl, budget_s=15.0):
    """The oracle on the first n requests of the workload (all of their rows), n chosen so that the
    attention part takes about budget_s."""
    import oracle
    trie = oracle.Trie()
    for i in range(wl.n_cached):
        trie.insert(*wl.cached_seq(i))
    pool_k, pool_v = oracle.new_pool(wl.num_slots, wl.Hkv, wl.D, wl.dtype)
    oracle.append_kv(pool_k, pool_v, wl.pool_slots, wl.pool_k, wl.pool_v, wl.dtype)
    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or (os.cpu_count() or 1)
    t0 = time.perf_counter()
    pl, si = trie.match(wl.tokens, wl.offsets)
    t_match = time.perf_counter() - t0

    def run(n):
        eo = wl.ext_offsets[:n + 1]
        T = int(eo[-1])
        t = time.perf_counter()
        oracle.extend_attention(wl.q_ext[:T], wl.k_ext[:T], wl.v_ext[:T], pool_k, pool_v, si, wl.offsets[:n + 1],
                                pl[:n], wl.ext_len[:n], eo, wl.scale, wl.dtype)
        return time.perf_counter() - t, T

    t1, T1 = run(1)
    n = int(max(1, min(wl.B, budget_s / max(t1, 1e-6))))
    if n > 1:
        t_att, Tn = run(n)
    else:
        t_att, Tn = t1, T1
    t = time.perf_counter()
    oracle.append_kv(pool_k, pool_v, wl.new_slots[:Tn], wl.k_ext[:Tn], wl.v_ext[:Tn], wl.dtype)
    t_app = time.perf_counter() - t
    total = t_match * n / wl.B + t_att + t_app
    return {"value": Tn / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {n} of {wl.B} requests ({Tn} of {wl.T} extend tokens, all heads): trie match {t_match * n / wl.B:.3f}s "
                      f"(whole batch {t_match:.3f}s, {wl.B / t_match:.0f} req/s), fp64 attention {t_att:.2f}s, append {t_app:.4f}s"}


def extras(pa, g, wl, prefix_len, slot_idx, out, ws, main_k, nbytes):
    """Measurements beside the step: the extend-attention kernel with cold caches (1 GiB streamed through the
    chip between launches: the L2s and the memory-side cache hold none of the K/V when it starts), and the matcher
    on a batch large enough to show its bandwidth (4,096 requests resampled from the workload's), what it costs to
    bring the tree's device mirror up to date after a small change, and what the machine itself reaches on a plain
    copy and on a loop of nothing but MFMAs (the published peaks are 8 TB/s and 2.5 PFLOP/s)."""
    import numpy as np
    import torch
    dev = g.tokens.device
    ex = {}
    # ---- cold caches ----
    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    pa.profile_enable(True)
    n_cold = 10
    for i in range(n_cold):
        flush.fill_(i)
        pa.extend_attention(g.q, g.k, g.v, g.pool, slot_idx, g.offsets, prefix_len, g.ext_len, g.ext_offsets, wl.scale,
                            max_kv_len=g.max_kv_len, out=out, workspace=ws, **g.kw)
    torch.cuda.synchronize()
    pa.profile_enable(False)
    ms, n = pa.profile_read(main_k)
    if n:
        t = ms / n * 1e-3
        ex["extend_cold_cache"] = {"avg_kernel_us": t * 1e6, "launches": n, "GBps_algorithmic": nbytes / t / 1e9,
                                   "hbm_frac": nbytes / t / 1e9 / HBM_PEAK_GBS, "flushed_bytes_between_launches": 1 << 30}
    del flush
    # ---- what the machine reaches: a plain copy of 1 GiB, and a loop of nothing but bf16 MFMAs ----
    src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    cal = torch.zeros(1 << 16, dtype=torch.uint8, device=dev)
    iters = 4096
    for _ in range(2):
        pa.calib_copy(dst, src)
        flops = pa.calib_mfma(cal, iters)
    pa.profile_enable(True)
    for _ in range(5):
        pa.calib_copy(dst, src)
    for _ in range(5):
        pa.calib_mfma(cal, iters)
    torch.cuda.synchronize()
    pa.profile_enable(False)
    ms_c, n_c = pa.profile_read("calib_copy")
    ms_m, n_m = pa.profile_read("calib_mfma")
    cyc, ticks = cal[:16].view(torch.int64).tolist()
    ex["achievable"] = {"copy_GBps": 2.0 * src.numel() / (ms_c / n_c * 1e-3) / 1e9, "copy_bytes_moved": 2 * src.numel(),
                        "mfma_bf16_TFLOPs": flops / (ms_m / n_m * 1e-3) / 1e12, "mfma_flops_per_launch": flops,
                        "mfma_shader_mhz": 100.0 * cyc / ticks if ticks else 0.0}
    del src, dst
    # ---- matcher at a batch that fills the chip ----
    rng = np.random.default_rng(0)
    Bbig = 4096
    pick = rng.integers(0, wl.B, Bbig)
    lens = (wl.offsets[1:] - wl.offsets[:-1])[pick].astype(np.int64)
    off = np.zeros(Bbig + 1, np.int64)
    off[1:] = np.cumsum(lens)
    if off[-1] < 2 ** 31 - 64:
        toks = np.concatenate([wl.tokens[wl.offsets[r]:wl.offsets[r + 1]] for r in pick]).astype(np.int32)
        t_d, o_d = torch.from_numpy(toks).to(dev), torch.from_numpy(off.astype(np.int32)).to(dev)
        pl = torch.empty(Bbig, dtype=torch.int32, device=dev)
        si = torch.empty_like(t_d)
        for _ in range(2):
            pa.match_prefixes(g.tree, t_d, o_d, pl, si)
        pa.profile_enable(True)
        for _ in range(5):
            pa.match_prefixes(g.tree, t_d, o_d, pl, si)
        torch.cuda.synchronize()
        pa.profile_enable(False)
        ms, n = pa.profile_read("match_prefixes")
        assert (pl.cpu().numpy() == wl.designed_prefix_len[pick]).all()
        t = ms / n * 1e-3
        matched = int(wl.designed_prefix_len[pick].astype(np.int64).sum())
        ex["match_scaled"] = {"requests": Bbig, "avg_kernel_us": t * 1e6, "reqs_per_s": Bbig / t, "matched_tokens_per_s": matched / t,
                              "GBps": 16.0 * matched / t / 1e9, "bytes_per_matched_token": 16}
    # ---- tree mirror: an upload after one small change, and one that copies the whole flat form ----
    vocab_hi = int(wl.tokens.max()) + 1 if wl.tokens.size else 1

    def timed_uploads(n_up):
        call, landed = [], []
        for i in range(n_up):
            junk = np.array([vocab_hi + i, 1, 2, 3], np.int32)            # a sequence no prompt starts with
            g.tree.insert(junk, np.arange(4, dtype=np.int32) + wl.num_slots)  # (slots no request can reach)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.tree.upload()
            t1 = time.perf_counter()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            call.append((t1 - t0) * 1e6)
            landed.append((t2 - t0) * 1e6)
        return float(np.mean(call[1:])), float(np.mean(landed[1:]))

    nodes, toks_in_tree = g.tree.stats()
    part = timed_uploads(9)
    g.tree.set_incremental_upload(False)
    whole = timed_uploads(5)
    g.tree.set_incremental_upload(True)
    ex["tree_upload"] = {"tree_nodes": nodes, "tree_tokens": toks_in_tree, "after_one_insert_call_us": part[0],
                         "after_one_insert_landed_us": part[1], "whole_tree_call_us": whole[0], "whole_tree_landed_us": whole[1]}
    return ex


def measure(name, steps, warmup, args, with_extras, kv_pool="bf16"):
    """All GPU measurements of one workload.  -> (result dict, the workload)."""
    import dataclasses

    import torch

    from paper_2407_00023_amd import binding as pa
    from paper_2407_00023_amd import workloads as W
    from paper_2407_00023_amd.resident import ResidentWorkload

    dev = torch.device("cuda:0")
    wl = W.CONFIGS[name]()
    if kv_pool == "fp8" and wl.dtype == "bf16":
        wl = dataclasses.replace(wl, dtype="bf16_kv8")
    g = ResidentWorkload(wl, dev)
    tdt = g.tdtype
    # every buffer of the step is allocated once, outside the timed region
    prefix_len = torch.empty(wl.B, dtype=torch.int32, device=dev)
    slot_idx = torch.empty_like(g.tokens)
    out = torch.empty_like(g.q)
    ws = torch.empty(pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, tdt), dtype=torch.uint8, device=dev)

    def step():
        if args.only in ("", "match"):
            pa.match_prefixes(g.tree, g.tokens, g.offsets, prefix_len, slot_idx)
        if args.only in ("", "extend"):
            pa.extend_attention(g.q, g.k, g.v, g.pool, slot_idx, g.offsets, prefix_len, g.ext_len, g.ext_offsets, wl.scale,
                                max_kv_len=g.max_kv_len, out=out, workspace=ws, **g.kw)
        if args.only in ("", "append"):
            pa.append_kv(g.pool, g.new_slots, g.k, g.v, **g.kw)

    pa.match_prefixes(g.tree, g.tokens, g.offsets, prefix_len, slot_idx)  # outputs valid whatever --only says
    step()
    torch.cuda.synchronize()
    # The step enqueues 4-5 short kernels and nothing else (no allocation, no host synchronisation), so it can be
    # captured once into a HIP graph and replayed (--graph).  The replay is checked against the eager result
    # before it is trusted.
    launch, mode = step, "eager"
    if args.graph:
        try:
            ref_pl, ref_out = prefix_len.clone(), out.clone()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            for _ in range(3):  # replays, with eager work and synchronisation between them, each checked
                prefix_len.zero_()
                out.zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                ok = bool((prefix_len == ref_pl).all()) if args.only in ("", "match") else True
                ok = ok and (bool(torch.equal(out, ref_out)) if args.only in ("", "extend") else True)
                if not ok:
                    raise RuntimeError("graph replay differs from the eager step")
            launch, mode = graph.replay, "hip graph replay"
        except Exception as e:  # capture not possible here: fall back to host launches, and say so
            print(f"bench.py: graph capture unavailable ({e}); timing eager launches", file=sys.stderr)
            torch.cuda.synchronize()
    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        launch()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    # same steps again with the library's per-kernel event timing switched on
    pa.profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    pa.profile_enable(False)
    kern = {}
    for kname in ("match_prefixes", "extend_plan", "extend_attention", "extend_merge", "extend_attention_f32", "append_kv"):
        ms, n = pa.profile_read(kname)
        if n:
            kern[kname] = {"avg_us": ms / n * 1e3, "launches_per_step": n / steps}
    shader_mhz = 0.0
    hdr = None
    if wl.dtype != "f32":
        pa.extend_status(ws)  # (raises if the work list of the launches above did not fit)
        hdr = ws[:16].view(torch.int32).tolist()
        # a few more steps with the clock probe in the kernel, kept out of the times above
        pa.profile_clock(ws, reset=True)
        pa.profile_enable(True, clock_probe=True)
        for _ in range(min(steps, 20)):
            step()
        torch.cuda.synchronize()
        pa.profile_enable(False)
        shader_mhz = pa.profile_clock(ws)

    pl = prefix_len.cpu().numpy()
    assert (pl == wl.designed_prefix_len).all(), "matcher disagrees with the designed prefix lengths"
    nbytes, flops = algorithmic_work(wl, pl)
    main_k = "extend_attention_f32" if wl.dtype == "f32" else "extend_attention"
    roofline = None
    if main_k in kern:
        t_k = kern[main_k]["avg_us"] * 1e-6
        gbs, tfs = nbytes / t_k / 1e9, flops / t_k / 1e12
        peak_f = FP32_VECTOR_PEAK_TFLOPS if wl.dtype == "f32" else MFMA_BF16_PEAK_TFLOPS
        t_mem, t_cmp = nbytes / (HBM_PEAK_GBS * 1e9), flops / (peak_f * 1e12)
        if t_mem >= t_cmp:
            roofline = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
        else:
            roofline = {"bound": "alu" if wl.dtype == "f32" else "mfma", "achieved": tfs, "peak": peak_f, "unit": "TFLOP/s",
                        "frac": tfs / peak_f}
        traffic = MEASURED_TRAFFIC_BYTES.get(name + ("_fp8_pool" if wl.dtype == "bf16_kv8" else ""))
        roofline.update({"traffic": traffic,
                         "traffic_source": (f"profiles/extend_attention_{name}{'_fp8_pool' if wl.dtype == 'bf16_kv8' else ''}.md "
                                            "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, runs of their own)") if traffic else None,
                         "kernel": main_k, "avg_kernel_us": kern[main_k]["avg_us"], "algorithmic_bytes": nbytes,
                         "algorithmic_flops": flops, "hbm_frac": gbs / HBM_PEAK_GBS, "compute_frac": tfs / peak_f})
        if hdr is not None:
            # traffic through the workspace (partial results of split row tiles, written by the attention kernel and
            # read back by the merge kernel): not part of algorithmic_bytes, shown beside it
            roofline["workspace_bytes"] = workspace_traffic(wl, hdr)
            roofline["work_list"] = {"row_tiles": hdr[0], "items": hdr[1], "tiles_merged_from_parts": hdr[2]}
        if shader_mhz > 0 and wl.dtype != "f32":
            # the clock the kernel ran at (shader cycles against the 100 MHz constant counter, across the key loop of a
            # few workgroups), and the matrix peak at that clock: 2.5 PFLOP/s is quoted at 2,400 MHz
            roofline["shader_mhz"] = shader_mhz
            roofline["compute_frac_at_measured_clock"] = tfs / (peak_f * shader_mhz / 2400.0)

    res = {
        "value": wl.T / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
        "dtype": "f32" if wl.dtype == "f32" else "bf16",
        "config": {"workload": name, "kv_pool": "fp8 codes + one exponent byte per row" if wl.dtype == "bf16_kv8" else wl.dtype, "requests": wl.B, "extend_tokens": wl.T, "prompt_tokens": int(wl.offsets[-1]),
                   "Hq": wl.Hq, "Hkv": wl.Hkv, "D": wl.D, "page_size": wl.page_size, "num_slots": wl.num_slots,
                   "cached_sequences": wl.n_cached, "only": args.only or "whole path", "launch": mode},
        "prompt_tokens_per_s": int(wl.offsets[-1]) / (ms_per_step * 1e-3),
        "kernels": kern,
        "roofline": roofline,
    }
    if "match_prefixes" in kern:
        res["match_reqs_per_s"] = wl.B / (kern["match_prefixes"]["avg_us"] * 1e-6)
    if "append_kv" in kern:
        el = 4 if wl.dtype == "f32" else 2
        app_bytes = 2 * (2 * wl.T * wl.Hkv * wl.D * el) + 4 * wl.T   # K and V rows read and written, slot ids read
        if wl.dtype == "bf16_kv8":
            app_bytes = 2 * wl.T * wl.Hkv * (wl.D * 2 + wl.D + 1) + 4 * wl.T   # bf16 rows read, codes and exponents written
        res["append_GBps"] = app_bytes / (kern["append_kv"]["avg_us"] * 1e-6) / 1e9
    if with_extras:
        res["extras"] = extras(pa, g, wl, prefix_len, slot_idx, out, ws, main_k, nbytes)
        ach = res["extras"].get("achievable")
        if ach and roofline and wl.dtype != "f32":
            # beside the fractions of the published peaks: of what a bare MFMA loop and a bare copy reach on this machine
            roofline["compute_frac_of_mfma_loop"] = roofline["compute_frac"] * MFMA_BF16_PEAK_TFLOPS / ach["mfma_bf16_TFLOPs"]
            roofline["hbm_frac_of_copy"] = roofline["hbm_frac"] * HBM_PEAK_GBS / ach["copy_GBps"]
    del g, out, ws
    torch.cuda.empty_cache()
    return res, wl


def summary(res):
    """One line of the `configs` array: what the headline carries for its own workload, shortened."""
    r = res["roofline"] or {}
    return {"workload": res["config"]["workload"], "kv_pool": res["config"]["kv_pool"], "requests": res["config"]["requests"],
            "extend_tokens": res["config"]["extend_tokens"], "steps": res["steps"], "ms_per_step": res["ms_per_step"],
            "extend_tokens_per_s": res["value"], "match_reqs_per_s": res.get("match_reqs_per_s"),
            "kernel_us": {k: round(v["avg_us"], 2) for k, v in res["kernels"].items()},
            "bound": r.get("bound"), "frac": r.get("frac"), "compute_frac": r.get("compute_frac"), "hbm_frac": r.get("hbm_frac"),
            "algorithmic_bytes": r.get("algorithmic_bytes"), "algorithmic_flops": r.get("algorithmic_flops"),
            "workspace_bytes": r.get("workspace_bytes"), "traffic": r.get("traffic"), "traffic_source": r.get("traffic_source"),
            "shader_mhz": r.get("shader_mhz")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="agent_tree", choices=["tiny_fp32", "tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"])
    ap.add_argument("--kv-pool", default="bf16", choices=["bf16", "fp8"], help="fp8: the KV pool of a bf16 workload in 8 bits per element")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the cold-cache and the scaled-matcher measurements")
    ap.add_argument("--no-configs", action="store_true", help="measure --workload only, not the other bf16 configurations beside it")
    ap.add_argument("--only", default="", help="time only one call of the path: match | extend | append (for profiling)")
    ap.add_argument("--graph", action="store_true", help="replay one captured HIP graph per step instead of launching its calls "
                    "from the host (measured: no faster, the gaps between the dependent kernels are not host-bound)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the path has no cross-GPU step); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU; there is no CPU fallback"
    head, wl = measure(args.workload, args.steps, args.warmup, args, with_extras=not args.no_extras and not args.only,
                       kv_pool=args.kv_pool)
    res = {"metric": "extend_prefill_tokens_per_s", "value": head["value"], "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic"}
    for k in ("config", "prompt_tokens_per_s", "kernels", "roofline", "match_reqs_per_s", "append_GBps", "extras"):
        if k in head:
            res[k] = head[k]
    if not args.no_configs and not args.only:
        rows = []
        for name in BF16_CONFIGS:
            if name == args.workload and args.kv_pool == "bf16":
                rows.append(summary(head))
            else:
                other, _ = measure(name, min(args.steps, 100), min(args.warmup, 10), args, with_extras=False)
                rows.append(summary(other))
        for name in FP8_POOL_CONFIGS:
            if name == args.workload and args.kv_pool == "fp8":
                rows.append(summary(head))
            else:
                other, _ = measure(name, min(args.steps, 100), min(args.warmup, 10), args, with_extras=False, kv_pool="fp8")
                rows.append(summary(other))
        res["configs"] = rows
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
