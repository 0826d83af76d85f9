#!/usr/bin/env python3
"""Benchmark of the MemoSight decode hot path on one MI355X.

One step = one pass of the whole hot path over the batch, shaped like a decode step of a
Qwen2.5-7B-sized model (28 attention layers, 28 query / 4 KV heads x 128, bf16):
  position ids of the block, built on the device from the next position ids
  28 x fused Predict+Verify attention, one per layer pool -> the HBM-bound part
  greedy longest-prefix acceptance on the device
  commit of the accepted verify rows into every layer's cache, the accept lengths read on the device
  every 14th step: the 56-token segment closed so far is compacted to 8 memory tokens
    (ratio 7, as in the paper's long-context analysis), in every layer (the host catches up here).
The workload is the metric point: batch 32, 8192 cached tokens per sequence, 5 verify + 4 foresight
queries, page tables shuffled over a shared pool.  All inputs are seeded and synthetic.

Prints ONE JSON line.  `value` is whole-step algorithmic KV throughput in GB/s with everything
resident in HBM; `roofline` prices the streaming attention kernel alone against 8 TB/s; the
`cpu_baseline` leg times the CPU oracle on a bounded sample of the same workload and the run fails
(exit status 3) if the GPU's result for that sample is outside the bf16 tolerance.  `roofline.traffic`
(HBM bytes per launch by the memory-side counters) comes from two short child runs of this script
under `rocprofv3 --pmc`, started before this process touches the GPU; if they cannot run, the
committed summary of the same two runs is reported instead and `traffic_source` says so.  The default run
also times two more points of the target's range -- batch 32 with 4096 cached tokens and the ragged
1k-16k batch -- for a few steps each and reports them under `also`.

`--workload compaction` is configuration 4: batch 16, 28 layers, every sequence closes a 256-token
segment into 8 memory tokens (microseconds and kernel launches per call), then 4 verify + 3
foresight queries attend over the caches that result.  `--workload decode_step` is the whole model
step (configuration 5).
"""
from __future__ import annotations

import argparse
import csv
import gc
import glob
import json
import os
import shutil
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
SEG_TOKENS, RATIO = 56, 7


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps before the timed ones; after an idle spell the part's power management needs "
                         "about ten steps (25 ms) of this workload to settle, during which launches run up to 10 %% slower")
    ap.add_argument("--layers", type=int, default=28)
    ap.add_argument("--batch", type=int, default=None, help="sequences (default: 32 for the attention workload, 64 for decode_step)")
    ap.add_argument("--kv", type=int, default=8192)
    ap.add_argument("--ragged", action="store_true", help="lengths uniform in [1k, 16k] instead of --kv")
    ap.add_argument("--q-heads", type=int, default=28, help="query heads (28 / 4: Qwen2.5-7B, 32 / 8: Llama-3.1-8B)")
    ap.add_argument("--kv-heads", type=int, default=4)
    ap.add_argument("--event-stride", type=int, default=None,
                    help="every n-th attention launch opens a span timed by one pair of HIP events (a pair costs the "
                         "stream a few microseconds); default: --layers for the attention workload, 29 for decode_step")
    ap.add_argument("--event-span", type=int, default=None,
                    help="attention launches one event pair covers (default: --layers for the attention workload, whose "
                         "layers launch back to back; 1 for decode_step, where other kernels run between them)")
    ap.add_argument("--no-also", action="store_true", help="skip the two extra points (batch 32 x 4096 tokens, ragged batch)")
    ap.add_argument("--queries", type=int, default=41, help="wide_step: causal queries per sequence (the memory tokens and <o>, or a prompt chunk)")
    ap.add_argument("--rows", type=int, default=448, help="projections: rows of the step (batch x queries)")
    ap.add_argument("--library-reference", action="store_true",
                    help="projections: also time torch.mm (hipBLASLt) on the same products, as a reference only")
    ap.add_argument("--workload", choices=["attention", "decode_step", "compaction", "wide_step", "projections"], default="attention",
                    help="attention: the metric's workload (default); compaction: configuration 4 (batch 16, 28 layers, "
                         "256 -> 8 tokens per sequence, then attention over the result); wide_step: a pass of --queries causal "
                         "queries; decode_step: the whole model step (Qwen2.5-7B shapes, batch 64, 8k cached tokens, 4 verify + "
                         "3 foresight)")
    ap.add_argument("--deterministic", action="store_true",
                    help="fixed tile-to-wave assignment in the attention kernel (bit-reproducible results, about 1.5 %% slower)")
    ap.add_argument("--host-commit", action="store_true",
                    help="attention workload: read the accept lengths back and commit from the host (synchronises the stream every step)")
    ap.add_argument("--no-live-traffic", action="store_true",
                    help="do not start the two rocprofv3 --pmc child runs that measure the attention kernel's HBM bytes per launch "
                         "(default workload only); the committed summary's figure is reported instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--read-probe", action="store_true",
                    help="time the library's plain read kernel over the layer pools even without the CPU baseline (with it, always)")
    ap.add_argument("--fused-lm-head", action="store_true",
                    help="decode_step: LM head and greedy token in one kernel of the library (fp32 sums, no logits)")
    ap.add_argument("--cpu-seqs", type=int, default=32, help="sequences the CPU oracle is timed on")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 1 GiB device copies, for scaling rocprofv3 byte counters")
    return ap.parse_args()


def live_traffic():
    """HBM bytes per launch of the attention kernel by the memory-side counters: two short runs of this
    script (the same workload, 3 steps, plus plain 1 GiB device copies that scale the counters) as
    children under `rocprofv3 --pmc`, one counter each -- rocprofv3 does not split passes, and a
    process whose counters are being read cannot also time itself.  Must be called before this
    process initialises the GPU.  Returns (bytes, note) or (None, reason)."""
    exe = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(exe):
        return None, "rocprofv3 not found"
    out = tempfile.mkdtemp(prefix="ms_pmc_", dir="/tmp")
    per_launch, scale, alg = {}, {}, None
    try:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            cmd = [exe, "--pmc", counter, "--output-format", "csv", "-d", os.path.join(out, counter), "-o", "pmc", "--",
                   sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1", "--no-cpu-baseline", "--no-also",
                   "--calibrate-copy", "--no-live-traffic"]
            try:
                res = subprocess.run(cmd, cwd="/tmp", env=dict(os.environ, TMPDIR="/tmp"), capture_output=True, text=True, timeout=150)
            except subprocess.TimeoutExpired:
                return None, f"the {counter} run under rocprofv3 did not finish in 150 s"
            if res.returncode != 0:
                return None, f"the {counter} run under rocprofv3 ended with status {res.returncode}"
            for line in res.stdout.splitlines():
                if line.startswith('{"metric"'):
                    alg = json.loads(line)["roofline"]["algorithmic_bytes_per_launch"]     # of the child's (shorter) run
            files = glob.glob(os.path.join(out, counter, "**", "*counter_collection.csv"), recursive=True)
            if not files:
                return None, f"the {counter} run left no counter file"
            kern, copy = [], []
            for r in csv.DictReader(open(files[0])):
                if r.get("Counter_Name") != counter:
                    continue
                if "pv_attn_mfma_stream" in r["Kernel_Name"]:
                    kern.append(float(r["Counter_Value"]))
                elif "copyBuffer" in r["Kernel_Name"]:
                    copy.append(float(r["Counter_Value"]))
            if not kern or not copy or max(copy) <= 0:
                return None, f"the {counter} file has no rows for the kernel or the copy"
            scale[counter] = 1048576.0 / max(copy)        # a 1 GiB copy reads and writes 1 GiB = 1048576 KiB
            per_launch[counter] = sum(kern) / len(kern)
        total = (per_launch["FETCH_SIZE"] * scale["FETCH_SIZE"] + per_launch["WRITE_SIZE"] * scale["WRITE_SIZE"]) * 1024.0
        note = ("two child runs of this script under rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; KiB per dispatch scaled by what a 1 GiB "
                f"copy reads: factors {scale['FETCH_SIZE']:.3f} and {scale['WRITE_SIZE']:.3f}): fetched "
                f"{per_launch['FETCH_SIZE'] * scale['FETCH_SIZE'] * 1024 / 1e6:.1f} MB, written "
                f"{per_launch['WRITE_SIZE'] * scale['WRITE_SIZE'] * 1024 / 1e6:.1f} MB per launch")
        if alg:
            note += f", against {alg / 1e6:.1f} MB algorithmic in those runs = {total / alg:.3f} x"
        return int(round(total)), note
    finally:
        shutil.rmtree(out, ignore_errors=True)


def read_probe(torch, M, ses, NL, achieved_gbps):
    """Plain read kernel of the library over the layer pools, ordinary and non-temporal loads; GB/s of the better one."""
    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    best = {}
    pool_bytes = ses.pool[0].numel() * ses.pool[0].element_size()
    warm = max(NL, int(40e-3 * 6e12 / pool_bytes))       # about 40 ms of reading first: the clocks settle (see --warmup)
    timed = max(NL, int(20e-3 * 6e12 / pool_bytes))
    for name, nt in (("ordinary", False), ("non_temporal", True)):
        for i in range(warm):
            M.ms_hbm_read_probe(ses.pool[i % NL], nt, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nbytes = 0
        for i in range(timed):
            nbytes += M.ms_hbm_read_probe(ses.pool[i % NL], nt, sink)
        e1.record()
        torch.cuda.synchronize()
        best[name] = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    top = max(best.values())
    return {"plain_read_gbps": {k: round(v, 1) for k, v in best.items()},
            "frac_of_plain_read": round(achieved_gbps / top, 4)}


def calibrate_copy(torch, dev, gen):
    """Plain 1 GiB device copies: what rocprofv3's byte counters read for a known size scales them."""
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=gen)   # 1 GiB
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.workload == "decode_step":
        return decode_step_bench(args)
    if args.workload == "compaction":
        return compaction_bench(args)
    if args.workload == "wide_step":
        return wide_step_bench(args)
    if args.workload == "projections":
        return projections_bench(args)
    args.batch = args.batch or 32
    default_point = not args.ragged and args.batch == 32 and args.kv == 8192 and args.layers == 28 and (args.q_heads, args.kv_heads) == (28, 4)
    live = None
    if default_point and not args.no_live_traffic:
        live = live_traffic()       # children first: this process has not touched the GPU yet
    import torch

    import workloads as W

    torch.cuda.set_device(0)
    sh = W.config3(n_layers=args.layers, batch=args.batch) if args.ragged else \
        W.metric_point(args.batch, args.kv, n_layers=args.layers)
    result = attention_workload(args, sh, args.steps, args.warmup, not args.no_cpu_baseline, args.ragged)
    if live is not None:
        nbytes, note = live
        if nbytes is not None:
            result["roofline"]["traffic"], result["roofline"]["traffic_source"] = nbytes, note
        else:
            result["roofline"]["traffic_source"] = (result["roofline"]["traffic_source"] or "none") + f"; no live measurement: {note}"
    if default_point and not args.no_also:
        # two more points of the target's range (batch 32, 4k to 16k tokens), a few steps each
        also = []
        for name, shape, ragged in (("batch32_kv4096", W.metric_point(32, 4096, n_layers=args.layers), False),
                                    ("config3_ragged_1k_16k", W.config3(n_layers=args.layers, batch=32), True)):
            r = attention_workload(args, shape, max(4, args.steps // 2), max(2, args.warmup // 2), False, ragged)
            also.append({"workload": r["config"]["workload"], "value": r["value"], "unit": "GB/s", "ms_per_step": r["ms_per_step"],
                         "steps": r["steps"], "pct_of_hbm_peak": r["pct_of_hbm_peak"], "roofline_frac": r["roofline"]["frac"],
                         "avg_kernel_ms": r["roofline"]["avg_kernel_ms"],
                         "algorithmic_bytes_per_launch": r["roofline"]["algorithmic_bytes_per_launch"]})
        result["also"] = also
    print(json.dumps(result))
    bad = result.get("cpu_baseline") and not result["cpu_baseline"]["within_tolerance"]
    if bad:
        print("bench.py: the GPU result is outside the bf16 tolerance of the oracle on the sampled sequences", file=sys.stderr)
        sys.exit(3)


def attention_workload(args, sh, steps, warmup, want_cpu, ragged):
    """Builds the caches of one workload shape, runs warm-up and timed steps, returns the result dict."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S

    dev = torch.device("cuda:0")
    if (args.q_heads, args.kv_heads) != (sh.n_q_heads, sh.n_kv_heads):
        if args.q_heads % args.kv_heads or args.kv_heads < 1:
            raise SystemExit("--q-heads must be a multiple of --kv-heads")
        sh.n_q_heads, sh.n_kv_heads = args.q_heads, args.kv_heads
    B, nq, nv, nf = sh.batch, sh.n_q, sh.n_verify, sh.n_foresight
    Hq, Hkv, D, NL = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.n_layers
    kv_label = sh.lengths[0]
    growth_pages = 8 * B                      # room for the tokens appended while the bench runs
    n_pages = sh.n_pages + growth_pages
    rng = W.make_rng(1000, B, NL)
    page_tables = W.shuffled_page_tables(rng, n_pages, sh.lengths)

    # ---- pool filled on the device from a seeded generator, N(0, 0.5), already "rotated" keys ----
    ses = S.Session(NL, Hq, Hkv, D, n_pages, M.MS_BF16, sh.rope_base, max_seqs=B,
                    max_pages_per_seq=max(len(p) for p in page_tables) + 64)
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED)
    for layer in range(NL):
        ses.pool[layer].normal_(0.0, sh.sigma, generator=gen)
    ids = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(sh.lengths, page_tables)]
    ids = M.int_array(ids)      # marshalled once: the same ids go into every call
    M.ms_attention_set_deterministic(ses.cache, args.deterministic)

    def dev_normal(*shape):
        return torch.empty(*shape, dtype=torch.bfloat16, device=dev).normal_(0.0, sh.sigma, generator=gen)

    q = dev_normal(B, nq, Hq, D)
    k_new = dev_normal(NL, B, nq, Hkv, D)
    v_new = dev_normal(NL, B, nq, Hkv, D)
    n_mem = SEG_TOKENS // RATIO
    mem_k = dev_normal(NL, B * n_mem, Hkv, D)
    mem_v = dev_normal(NL, B * n_mem, Hkv, D)
    out = torch.empty_like(q)
    draft_np, target_np = W.draft_and_target(rng, B, nv, 1000, forced_prefix=[nv - 1] * B)
    draft, target = S.ints_dev(draft_np).view(B, nv), S.ints_dev(target_np).view(B, nv)
    acc_d = torch.empty(B, dtype=torch.int32, device=dev)
    nxt_d = torch.empty(B, dtype=torch.int32, device=dev)
    acc_h = torch.empty(B, dtype=torch.int32, pin_memory=True)
    pos_h = torch.empty(B, nq, dtype=torch.int32, pin_memory=True)
    pos_d = torch.empty(B, nq, dtype=torch.int32, device=dev)
    mpos_h = torch.empty(B * n_mem, dtype=torch.int32, pin_memory=True)
    mpos_d = torch.empty(B * n_mem, dtype=torch.int32, device=dev)
    pos_np, mpos_np = pos_h.numpy(), mpos_h.numpy()     # views of the pinned buffers
    ses.ensure_workspace(B, nq)

    # raw position of each sequence's next token (about 3x the compressed length) and the open segment.
    # With the commit on the device the host learns the accepted counts only when it asks (for a
    # compaction, which needs exact segment ranges): `known` is what it knew at the last such point.
    next_pid = np.asarray([sh.first_query_pid(b) for b in range(B)], dtype=np.int32)
    seg_len = np.zeros(B, dtype=np.int64)
    cur_len = np.asarray(ses.lengths(ids), dtype=np.int64)
    acc_np = acc_h.numpy()
    total_steps = warmup + steps
    acc_log = torch.zeros(total_steps, B, dtype=torch.int32, device=dev)     # the device's accept lengths, step by step
    first_pid_d = S.ints_dev(next_pid)
    state = {"step": 0, "known": 0, "compacted_after": []}
    layer_args = [(k_new[layer], v_new[layer]) for layer in range(NL)]
    stream = torch.cuda.current_stream()
    sh_ = stream.cuda_stream    # raw handle for the library calls
    host_commit = args.host_commit

    def algorithmic_bytes(lengths):
        es = 2
        per_call = int(np.sum(2 * lengths * Hkv * D * es + 4 * (-(-lengths // 16))))
        per_call += B * nq * (2 * Hq + 2 * Hkv) * D * es
        return per_call

    def catch_up():
        """The host learns the accept lengths of the steps since it last asked (synchronises)."""
        i0, i1 = state["known"], state["step"]
        if i1 > i0:
            got = acc_log[i0:i1].cpu().numpy().astype(np.int64).sum(axis=0)
            next_pid[:] += got.astype(np.int32)
            seg_len[:] += got
            cur_len[:] += got
            state["known"] = i1

    def compact_if_due():
        # a8: close and compact the segment once it holds 56 tokens
        if seg_len.min() < SEG_TOKENS:
            return
        begin = cur_len - seg_len
        cnt = [M.ms_ama_count(int(n), RATIO) for n in seg_len]
        assert all(c == n_mem for c in cnt)
        off = 0
        for b in range(B):
            first = int(next_pid[b] - seg_len[b])
            mp = M.ms_upl_positions(first, int(seg_len[b]), RATIO)
            mpos_np[off:off + len(mp)] = mp
            off += len(mp)
        mpos_d.copy_(mpos_h, non_blocking=True)
        M.ms_compact_segment(ses.cache, ids, begin, seg_len, cnt, mem_k, mem_v, mpos_d)
        next_pid[:] = [M.ms_output_token_pid(int(p) - 1) + 1 for p in next_pid]   # <o> takes one position
        cur_len[:] += np.asarray(cnt) - seg_len
        seg_len_before = seg_len.copy()
        seg_len[:] = 0
        state["compacted_after"].append((state["step"], np.asarray(cnt, dtype=np.int64) - seg_len_before))
        if not host_commit:
            first_pid_d.copy_(torch.from_numpy(next_pid), non_blocking=False)

    def step():
        acc_d = acc_log[state["step"]]
        if host_commit:
            # a1: position layout on the host (verify block, then foresight tokens right after it)
            M.ms_step_positions(next_pid, nv, nf, pos_np)
            pos_d.copy_(pos_h, non_blocking=True)
        else:
            M.ms_step_positions_device(first_pid_d, nv, nf, pos_d, sh_)
        # a2-a5: attention in every layer
        for layer in range(NL):
            kl, vl = layer_args[layer]
            ses.attention(layer, ids, nv, nf, q, kl, vl, pos_d, None, 0.0, out, sh_)
        # a6: acceptance on the device
        M.ms_accept(B, nv, draft, target, None, acc_d, nxt_d, sh_)
        state["step"] += 1
        if host_commit:
            # accept lengths back to the host, a7: commit of the accepted verify rows in every layer
            acc_h.copy_(acc_d, non_blocking=True)
            stream.synchronize()
            M.ms_commit_accepted(ses.cache, ids, acc_np, nq, k_new, v_new, pos_d, sh_)
            next_pid[:] += acc_np
            seg_len[:] += acc_np
            cur_len[:] += acc_np
            state["known"] = state["step"]
            compact_if_due()
            return
        # a7 on the device: the kernel reads the accept lengths, takes pages in the host's order and
        # advances the lengths and the next position ids; the stream is not synchronised
        M.ms_commit_accepted_device(ses.cache, ids, acc_d, nq, nv, k_new, v_new, pos_d, first_pid_d, sh_)
        # the host asks only when the open segment could have reached 56 tokens by now
        if (seg_len + nv * (state["step"] - state["known"])).min() >= SEG_TOKENS:
            catch_up()
            compact_if_due()

    gc.collect()
    gc.disable()    # a full collection in the middle of a step stalls the launch thread for tens of milliseconds
    for _ in range(warmup):
        step()
    # one event pair per step around its NL back-to-back attention launches: nothing else runs on the
    # stream between them, so span time / NL is the kernel's duration plus the gap to the next launch.
    # Nothing slow may sit between the warm-up and the timed steps (a pause of some tens of milliseconds
    # lets the part drop its clocks, and the first ten steps after it run up to 10 % slower), so the
    # collector ran before the warm-up and only as many events are created as there are spans.
    ev_stride = args.event_stride or NL
    ev_span = min(args.event_span or NL, ev_stride)
    torch.cuda.synchronize()
    M.ms_profile_attention(ses.cache, -(-steps * NL // ev_stride), ev_stride, ev_span)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    kern_ms = M.ms_profile_read(ses.cache, steps * NL)
    M.ms_profile_attention(ses.cache, 0, 1, 1)
    M.ms_check_integrity(ses.cache)

    ms_per_step = (t1 - t0) * 1e3 / steps
    catch_up()
    lengths = np.asarray(ses.lengths(ids), dtype=np.int64)
    assert np.array_equal(lengths, cur_len), "host copy of the lengths drifted from the cache's"
    # the bytes every timed launch had to move, from the lengths step by step (replayed from the device's accept log)
    log = acc_log.cpu().numpy().astype(np.int64)
    lens = np.asarray(sh.lengths, dtype=np.int64)
    kv_bytes, accepted = 0.0, 0
    for i in range(total_steps):
        if i >= warmup:
            kv_bytes += NL * algorithmic_bytes(lens)
            accepted += int(log[i].sum())
        lens = lens + log[i]
        for after, delta in state["compacted_after"]:
            if after == i + 1:
                lens = lens + delta
    assert np.array_equal(lens, cur_len), "replayed lengths differ from the cache's"
    gbps = kv_bytes / (t1 - t0) / 1e9
    per_launch_bytes = int(round(kv_bytes / (steps * NL)))   # mean over the timed launches
    kern_avg_ms = float(np.mean(kern_ms)) if kern_ms else float("nan")
    achieved = per_launch_bytes / (kern_avg_ms * 1e-3) / 1e9 if kern_ms else float("nan")

    # HBM bytes per launch by the memory-side counters cannot be read from inside the process: they come
    # from two rocprofv3 --pmc runs of this command (FETCH_SIZE, WRITE_SIZE), whose summary is committed
    # under profiles/ for the default workload only; any other workload reports null
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "pv_attn_mfma_stream_batch32_kv8192_traffic.json")
    if os.path.exists(tpath) and not ragged and B == 32 and kv_label == 8192 and (Hq, Hkv) == (28, 4):
        try:
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
            traffic_source = "profiles/pv_attn_mfma_stream_batch32_kv8192_traffic.json (rocprofv3 --pmc runs of this command)"
        except Exception:
            traffic = None

    result = {
        "metric": f"predict_verify_attn_hbm_gbps_b{B}_" + ("ragged_1k_16k" if ragged else
                                                           f"kv{kv_label // 1024}k" if kv_label % 1024 == 0 else f"kv{kv_label}"),
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": ("config3_ragged_1k_16k" if ragged else f"batch{B}_kv{kv_label}") +
                        f"_layers{NL}_q{Hq}_kv{Hkv}_d{D}_verify{nv}_foresight{nf}",
            "batch": B, "mean_kv_len": round(float(np.mean(lengths)), 1), "layers": NL,
            "step": f"{NL}-layer attention + accept + commit, compaction 56->8 every 14 steps",
            "commit": "host-side: accept lengths read back, the stream synchronised every step" if host_commit else
                      "device-side: the kernel reads the accept lengths; the host synchronises only for a compaction",
            "attention_tile_assignment": "fixed (bit-reproducible)" if args.deterministic else
                                         "first come, first served (reproducible to rounding)",
        },
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "query_tokens_per_s": round(B * nq * steps / (t1 - t0), 1),
        "decode_tokens_per_s": round(accepted / (t1 - t0), 1),
        "accepted_per_step_per_seq": round(accepted / steps / B, 3),
        "roofline": {
            "kernel": "pv_attn_mfma_stream",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "traffic_source": traffic_source,
            "avg_kernel_ms": round(kern_avg_ms, 5),
            "median_kernel_ms": round(float(np.median(kern_ms)), 5) if kern_ms else None,
            "min_kernel_ms": round(float(np.min(kern_ms)), 5) if kern_ms else None,
            "launches": len(kern_ms) * ev_span,
            "launches_per_event_pair": ev_span,
            "algorithmic_bytes_per_launch": per_launch_bytes,
        },
    }

    if want_cpu or args.read_probe:
        # what a plain streaming read of the same layer pools reaches on this machine (the layers in turn, so
        # every pass comes from HBM): the other denominator beside the published peak
        result["roofline"].update(read_probe(torch, M, ses, NL, per_launch_bytes / (kern_avg_ms * 1e-3) / 1e9))
    if args.calibrate_copy:
        calibrate_copy(torch, dev, gen)
    if want_cpu:
        result["cpu_baseline"] = cpu_baseline(args, ses, sh, ids, lengths, q, k_new, v_new, pos_d, out, M, S, W)
    ses.close()
    del ses, q, k_new, v_new, mem_k, mem_v, layer_args
    torch.cuda.empty_cache()
    return result


def wide_step_bench(args):
    """A pass of many causal queries and no foresight tokens over the cache: the memory-token pass that
    closes a reasoning step (l + 1 queries, Algorithm 1) or a chunk of a prompt.  --queries queries
    per sequence (up to 64), --batch sequences of --kv cached tokens, one attention call per layer."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    B, NL, Hq, Hkv, D, nq = args.batch or 8, args.layers, args.q_heads, args.kv_heads, 128, args.queries
    sh = W.AttnShape("wide", "bf16", B, Hq, Hkv, D, nq, 0, [args.kv] * B, 0.5, 1000000.0, n_layers=NL)
    rng = W.make_rng(1006, B, NL)
    page_tables = W.shuffled_page_tables(rng, sh.n_pages, sh.lengths)
    ses = S.Session(NL, Hq, Hkv, D, sh.n_pages, M.MS_BF16, sh.rope_base, max_seqs=B, max_pages_per_seq=max(len(p) for p in page_tables) + 4)
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED + 6)
    for layer in range(NL):
        ses.pool[layer].normal_(0.0, sh.sigma, generator=gen)
    ids = M.int_array([M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(sh.lengths, page_tables)])

    def dev_normal(*shape):
        return torch.empty(*shape, dtype=torch.bfloat16, device=dev).normal_(0.0, sh.sigma, generator=gen)

    q, k_new, v_new = dev_normal(B, nq, Hq, D), dev_normal(NL, B, nq, Hkv, D), dev_normal(NL, B, nq, Hkv, D)
    out = torch.empty_like(q)
    pos_d = S.ints_dev(M.ms_step_positions(np.asarray([3 * n + 1 for n in sh.lengths], np.int32), nq, 0)).view(B, nq)
    ses.ensure_workspace(B, nq)
    sh_ = torch.cuda.current_stream().cuda_stream

    def step():
        for layer in range(NL):
            ses.attention(layer, ids, nq, 0, q, k_new[layer], v_new[layer], pos_d, None, 0.0, out, sh_)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    n0 = M.ms_launch_count(ses.cache)
    M.ms_profile_attention(ses.cache, args.steps, NL, NL)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    launches = (M.ms_launch_count(ses.cache) - n0) / (args.steps * NL)
    if args.calibrate_copy:
        calibrate_copy(torch, dev, gen)
    kern_ms = M.ms_profile_read(ses.cache, args.steps)
    M.ms_profile_attention(ses.cache, 0, 1, 1)
    lens = np.asarray(sh.lengths, dtype=np.int64)
    per_call_bytes = int(np.sum(2 * lens * Hkv * D * 2 + 4 * (-(-lens // 16)))) + B * nq * (2 * Hq + 2 * Hkv) * D * 2
    per_call_flops = 4.0 * float(lens.sum() + B * nq / 2) * Hq * nq * D
    call_ms = float(np.mean(kern_ms))
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    result = {
        "metric": f"wide_step_attn_hbm_gbps_b{B}_kv{args.kv}_q{nq}",
        "value": round(NL * per_call_bytes / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"wide_step_batch{B}_kv{args.kv}_layers{NL}_q{Hq}_kv{Hkv}_d{D}_causal_queries{nq}", "batch": B, "layers": NL,
                   "step": f"{NL} attention calls of {nq} causal queries per sequence"},
        "kernel_launches_per_call": launches,
        "call_us": round(call_ms * 1e3, 2),
        "matrix_core_tflops": round(per_call_flops / (call_ms * 1e-3) / 1e12, 1),
        "roofline": {"kernel": "pv_attn_mfma_wide" if launches >= 1 and (nq > 16 or nq * (Hq // Hkv) > 64) else "pv_attn_mfma_stream",
                     "bound": "hbm", "achieved": round(per_call_bytes / (call_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(per_call_bytes / (call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "avg_kernel_ms": round(call_ms, 5), "launches": len(kern_ms) * NL, "launches_per_event_pair": NL,
                     "algorithmic_bytes_per_launch": per_call_bytes},
        "cpu_baseline": None,
    }
    ses.close()
    print(json.dumps(result))


def compaction_bench(args):
    """Configuration 4: batch 16, 28 layers of 4 KV heads x 128, bf16.  Every sequence (2304 to 8448
    cached tokens, multiples of 16) closes its last 256 tokens into 8 memory tokens (c = 32): the
    segment's 16 pages are released, the memory-token rows are rotated at their UPL position ids and
    scattered into fresh pages, in every layer, in one call.  Timed per call (the caches are put
    back between calls, untimed, by freeing and re-importing the sequences); then 4 verify + 3
    foresight queries attend over the 2k-8k token caches that result, 28 layers per step."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    B, NL, Hq, Hkv, D = args.batch or 16, args.layers, args.q_heads, args.kv_heads, 128
    nv, nf, seg, c_ratio = 4, 3, 256, 32
    nq, n_mem = nv + nf, seg // c_ratio
    rng = W.make_rng(1004, B, NL)
    lens = [int(16 * x) for x in rng.integers(2304 // 16, 8448 // 16 + 1, size=B)]
    sh = W.AttnShape("config4", "bf16", B, Hq, Hkv, D, nv, nf, lens, 0.5, 1000000.0, n_layers=NL, slack_pages=0.02)
    page_tables = W.shuffled_page_tables(rng, sh.n_pages, lens)
    ses = S.Session(NL, Hq, Hkv, D, sh.n_pages, M.MS_BF16, sh.rope_base, max_seqs=B, max_pages_per_seq=max(len(p) for p in page_tables) + 8)
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED + 4)
    for layer in range(NL):
        ses.pool[layer].normal_(0.0, sh.sigma, generator=gen)

    def dev_normal(*shape):
        return torch.empty(*shape, dtype=torch.bfloat16, device=dev).normal_(0.0, sh.sigma, generator=gen)

    mem_k, mem_v = dev_normal(NL, B * n_mem, Hkv, D), dev_normal(NL, B * n_mem, Hkv, D)
    begin = [n - seg for n in lens]
    mpos = sum((M.ms_upl_positions(3 * n - seg + 1, seg, c_ratio) for n in lens), [])
    mpos_d = S.ints_dev(mpos)
    stream = torch.cuda.current_stream()

    def restore():
        for s_ in range(B):
            if live[0]:
                M.ms_seq_free(ses.cache, s_)
        ids_ = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(lens, page_tables)]
        live[0] = True
        return ids_

    live = [False]
    host_us, dev_us, launches = [], [], []
    for it in range(args.warmup + args.steps):
        ids = restore()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n0 = M.ms_launch_count(ses.cache)
        e0.record(stream)
        t0 = time.perf_counter()
        M.ms_compact_segment(ses.cache, ids, begin, [seg] * B, [n_mem] * B, mem_k, mem_v, mpos_d, stream=stream.cuda_stream)
        t1 = time.perf_counter()
        e1.record(stream)
        torch.cuda.synchronize()
        if it >= args.warmup:
            host_us.append((t1 - t0) * 1e6)
            dev_us.append(e0.elapsed_time(e1) * 1e3)
            launches.append(M.ms_launch_count(ses.cache) - n0)
    M.ms_check_integrity(ses.cache)
    new_lens = np.asarray(ses.lengths(ids), dtype=np.int64)
    assert new_lens.tolist() == [n - seg + n_mem for n in lens]
    rows_bytes = B * n_mem * NL * Hkv * D * 2 * 2            # K and V rows written into the pool (and as many read)

    # ---- attention over the compacted caches: 28 layers per step, one event pair per step ----
    q = dev_normal(B, nq, Hq, D)
    k_new, v_new = dev_normal(NL, B, nq, Hkv, D), dev_normal(NL, B, nq, Hkv, D)
    out = torch.empty_like(q)
    pos = M.ms_step_positions(np.asarray([3 * n + 1 for n in lens], np.int32), nv, nf)
    pos_d = S.ints_dev(pos).view(B, nq)
    ids_c = M.int_array(ids)
    ses.ensure_workspace(B, nq)
    sh_ = stream.cuda_stream

    def attn_step():
        for layer in range(NL):
            ses.attention(layer, ids_c, nv, nf, q, k_new[layer], v_new[layer], pos_d, None, 0.0, out, sh_)

    for _ in range(max(2, args.warmup)):
        attn_step()
    torch.cuda.synchronize()
    M.ms_profile_attention(ses.cache, args.steps, NL, NL)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        attn_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern_ms = M.ms_profile_read(ses.cache, args.steps)
    M.ms_profile_attention(ses.cache, 0, 1, 1)
    per_launch_bytes = int(np.sum(2 * new_lens * Hkv * D * 2 + 4 * (-(-new_lens // 16)))) + B * nq * (2 * Hq + 2 * Hkv) * D * 2
    kern_avg_ms = float(np.mean(kern_ms))
    achieved = per_launch_bytes / (kern_avg_ms * 1e-3) / 1e9
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gbps = NL * per_launch_bytes / (ms_per_step * 1e-3) / 1e9
    result = {
        "metric": f"predict_verify_attn_hbm_gbps_b{B}_after_compaction_256_to_8",
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"config4_batch{B}_layers{NL}_q{Hq}_kv{Hkv}_d{D}_segment{seg}_to_{n_mem}_then_verify{nv}_foresight{nf}",
                   "batch": B, "mean_kv_len": round(float(new_lens.mean()), 1), "layers": NL,
                   "step": f"{NL}-layer attention over the compacted caches (the compaction itself is timed per call, below)"},
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "compaction": {
            "calls": len(dev_us), "sequences_per_call": B, "layers": NL,
            "device_us_per_call": round(float(np.mean(dev_us)), 1), "device_us_min": round(float(np.min(dev_us)), 1),
            "host_us_per_call": round(float(np.mean(host_us)), 1),
            "kernel_launches_per_call": float(np.mean(launches)),
            "kv_row_bytes_written_per_call": rows_bytes,
            "pages_released_per_call": B * (seg // 16), "pages_taken_per_call": B * (-(-n_mem // 16)),
            "timing": "HIP events on the call's stream around one call (includes the launch latency); host = time inside the call",
        },
        "roofline": {"kernel": "pv_attn_mfma_stream", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None, "avg_kernel_ms": round(kern_avg_ms, 5),
                     "launches": len(kern_ms) * NL, "launches_per_event_pair": NL, "algorithmic_bytes_per_launch": per_launch_bytes},
        "cpu_baseline": None,
    }
    ses.close()
    print(json.dumps(result))


def decode_step_bench(args):
    """The whole model step of Algorithm 1's SpeculativeStep at Qwen2.5-7B shapes with random bf16
    weights: embedding, 28 x (RMSNorm, Q/K/V GEMMs, fused attention, output GEMM, RMSNorm, MLP GEMMs
    with SwiGLU), final norm, LM head GEMM, greedy tokens, acceptance against them, commit of the
    accepted rows; the next verify block is built on the device from the step's own predictions.
    Every kernel of the step is this library's."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import decoder as D
    from paper_2604_14889_amd import session as S

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = D.DecoderConfig.qwen2_5_7b()
    if args.layers != 28:
        cfg.n_layers = args.layers
    B = args.batch or 64
    L0, nv, nf = args.kv, 4, 3
    nq = nv + nf
    NL, Hq, Hkv, Dh = cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    lengths = [L0] * B
    pages_per_seq = -(-L0 // 16)
    room = max(16, -(-(args.warmup + args.steps) * nv // 16) + 1)    # pages a sequence can grow by while the bench runs
    n_pages = B * (pages_per_seq + room)
    rng = W.make_rng(1005, B, NL)
    page_tables = W.shuffled_page_tables(rng, n_pages, lengths)
    ses = S.Session(NL, Hq, Hkv, Dh, n_pages, M.MS_BF16, cfg.rope_base, max_seqs=B, max_pages_per_seq=pages_per_seq + max(64, room + 1))
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED + 5)
    for layer in range(NL):
        ses.pool[layer].normal_(0.0, 0.5, generator=gen)
    ids = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(lengths, page_tables)]
    weights = D.DecoderTensors.random(cfg, W.BASE_SEED + 6, dev)
    dec = D.Decoder(cfg, weights, ses, B * nq, fused_lm_head=args.fused_lm_head)
    ses.ensure_workspace(B, nq)

    foresight_id = cfg.vocab - 1                           # stands for the <f> token
    tokens = torch.randint(0, cfg.vocab - 1, (B, nq), dtype=torch.int32, device=dev, generator=gen)
    tokens[:, nv:] = foresight_id
    acc_d = torch.empty(B, dtype=torch.int32, device=dev)
    nxt_d = torch.empty(B, dtype=torch.int32, device=dev)
    acc_h = torch.empty(B, dtype=torch.int32, pin_memory=True)
    pos_h = torch.empty(B, nq, dtype=torch.int32, pin_memory=True)
    pos_d = torch.empty(B, nq, dtype=torch.int32, device=dev)
    pos_np, acc_np = pos_h.numpy(), acc_h.numpy()
    next_pid = np.asarray([3 * n + 1 for n in lengths], dtype=np.int32)
    first_pid_d = torch.from_numpy(next_pid.copy()).to(dev)
    total_steps = args.warmup + args.steps
    commit_log = torch.zeros(total_steps, B, dtype=torch.int32, device=dev)   # rows kept per step and sequence
    host_commit = args.host_commit
    cur_len = np.asarray(lengths, dtype=np.int64)
    stream = torch.cuda.current_stream()
    state = {"committed": 0, "kv_bytes": 0.0, "step": 0}

    def step():
        if host_commit:
            M.ms_step_positions(next_pid, nv, nf, pos_np)
            pos_d.copy_(pos_h, non_blocking=True)
        else:
            M.ms_step_positions_device(first_pid_d, nv, nf, pos_d)
        _, targets = dec.step(ids, tokens, pos_d, nv, nf)
        tg = targets.view(B, nq)
        M.ms_accept(B, nv - 1, tokens[:, 1:nv].contiguous(), tg[:, :nv - 1].contiguous(), None, acc_d, nxt_d)
        # next verify block: the token after the accepted ones, then the foresight rows' predictions
        tokens[:, 0] = torch.gather(tg, 1, acc_d.long().unsqueeze(1)).squeeze(1)
        tokens[:, 1:nv] = tg[:, nv:]
        k_new, v_new = dec.step_kv()
        n_commit_d = commit_log[state["step"]]
        torch.add(acc_d, 1, out=n_commit_d)                 # the block's first token is always kept
        state["step"] += 1
        if not host_commit:
            # the commit reads the counts on the device, takes pages in the host's order and advances the
            # lengths and the next position ids: no synchronisation in the step
            M.ms_commit_accepted_device(ses.cache, ids, n_commit_d, nq, nv, k_new, v_new, pos_d, first_pid_d)
            return
        acc_h.copy_(n_commit_d, non_blocking=True)
        stream.synchronize()
        M.ms_commit_accepted(ses.cache, ids, acc_np, nq, k_new, v_new, pos_d)
        next_pid[:] += acc_np

    gc.collect()
    gc.disable()    # a full collection in the middle of a step stalls the launch thread for tens of milliseconds
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # other kernels run between the layers' attention launches here: one launch per event pair
    # (as many events as spans: creating thousands of them would idle the GPU between warm-up and timing)
    ev_stride = args.event_stride or 29
    M.ms_profile_attention(ses.cache, -(-args.steps * NL // ev_stride), ev_stride, 1)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    kern_ms = M.ms_profile_read(ses.cache, args.steps * NL)
    M.ms_profile_attention(ses.cache, 0, 1, 1)
    M.ms_check_integrity(ses.cache)
    log = commit_log.cpu().numpy().astype(np.int64)
    cur_len = cur_len + log.sum(0)
    assert np.array_equal(np.asarray(ses.lengths(ids)), cur_len), "the cache's lengths differ from the logged commits"
    state["committed"] = int(log[args.warmup:].sum())
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # bytes of the timed launches: mean over the timed steps of the lengths they started from
    start_len = np.asarray(lengths, dtype=np.int64)[None, :] + np.cumsum(log, 0) - log
    mean_len = start_len[args.warmup:].mean(0)
    per_launch_bytes = int(np.sum(2 * mean_len * Hkv * Dh * 2 + 4 * np.ceil(mean_len / 16))) + B * nq * (2 * Hq + 2 * Hkv) * Dh * 2
    kern_avg_ms = float(np.mean(kern_ms)) if kern_ms else float("nan")
    achieved = per_launch_bytes / (kern_avg_ms * 1e-3) / 1e9
    attn_ms = kern_avg_ms * NL      # from the sampled launches (an event pair around every launch would stall the stream)
    n_params = sum(t.numel() for lw in weights.layers for t in vars(lw).values()) + weights.lm_head.numel() + weights.norm.numel()
    result = {
        "metric": f"full_decode_step_tokens_per_s_b{B}_kv{L0 // 1024}k",
        "value": round(state["committed"] / (t1 - t0), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": f"decode_step_qwen2.5-7b_shapes_batch{B}_kv{L0}_layers{NL}_verify{nv}_foresight{nf}",
            "batch": B, "mean_kv_len": round(float(cur_len.mean()), 1), "layers": NL,
            "step": f"embedding, {NL} blocks (norm, fused Q/K/V projection, attention, output projection, norm, gate/up projection with "
                    "SwiGLU, down projection with the residual add and the next norm), LM head, greedy tokens, accept, commit: every kernel is "
                    "this library's; random weights, so about one token per sequence is accepted per step; "
                    + ("accept lengths read back by the host before the commit" if host_commit else "commit on the device, no synchronisation in the step"),
            "projections": "few-row matrix-core kernel" if B * nq <= 16 else "tiled matrix-core GEMM",
        },
        "query_tokens_per_s": round(B * nq * args.steps / (t1 - t0), 1),
        "committed_per_step_per_seq": round(state["committed"] / args.steps / B, 3),
        "attention_ms_per_step": round(attn_ms, 4),
        "attention_share_of_step": round(attn_ms / ms_per_step, 4),
        "weight_bytes_streamed_per_step": int(n_params * 2),
        "roofline": {
            "kernel": "pv_attn_mfma_stream", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
            "avg_kernel_ms": round(kern_avg_ms, 5), "launches": len(kern_ms),
            "algorithmic_bytes_per_launch": per_launch_bytes,
        },
        "cpu_baseline": None,
    }
    ses.close()
    print(json.dumps(result))


def projections_bench(args):
    """The five dense projections of a decoder block and the LM head at Qwen2.5-7B widths (Algorithm 1,
    SpeculativeStep; Section 3.1), each as the decoder calls it (bias, K split, SwiGLU or residual add +
    RMSNorm in the same call), stand-alone with cold weights: every call takes the next of several
    weight copies that together exceed the chip's caches.  One HIP-event pair around `--steps` calls."""
    import torch

    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import decoder as D

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = D.DecoderConfig.qwen2_5_7b()
    rows = args.rows
    qd, kd, hid, inter = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.hidden, cfg.inter
    vocab = -(-cfg.vocab // 128) * 128
    # the decoder's K splits (decoder.py): one row tile up to 256 rows
    few = rows <= 256
    splits = {"qkv": 7 if few else 4, "out": 8 if few else 7, "down": 16 if few else 8}
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260414)

    def rand(*shape, scale=1.0):
        return (torch.randn(*shape, device=dev, dtype=torch.float32, generator=gen) * scale).to(torch.bfloat16)

    def copies(n, k):   # enough copies of an [n, k] weight to exceed 640 MB (L2 + the 256 MB memory-side cache twice over)
        return [rand(n, k, scale=k ** -0.5) for _ in range(max(2, min(24, -(-640_000_000 // (n * k * 2)))))]

    ws = torch.empty(max(M.ms_gemm_workspace_bytes(rows, qd + 2 * kd, hid, splits["qkv"]),
                         M.ms_gemm_add_rmsnorm_workspace_bytes(rows, hid, qd, splits["out"]),
                         M.ms_gemm_add_rmsnorm_workspace_bytes(rows, hid, inter, splits["down"]),
                         M.ms_gemm_workspace_bytes(rows, 2 * inter, hid, 1), M.ms_gemm_workspace_bytes(rows, vocab, hid, 1), 16),
                     dtype=torch.uint8, device=dev)
    x_h, x_q, x_i = rand(rows, hid), rand(rows, qd), rand(rows, inter, scale=0.1)
    h = torch.zeros(rows, hid, dtype=torch.float32, device=dev)
    norm_w = rand(hid)
    bias = rand(qd + 2 * kd, scale=0.1)
    q, k, v = (torch.empty(rows, n, dtype=torch.bfloat16, device=dev) for n in (qd, kd, kd))
    x_out = torch.empty(rows, hid, dtype=torch.bfloat16, device=dev)
    act = torch.empty(rows, inter, dtype=torch.bfloat16, device=dev)
    logits = torch.empty(rows, vocab, dtype=torch.bfloat16, device=dev)
    cases = [
        ("qkv", qd + 2 * kd, hid, f"bias, three outputs, K split {splits['qkv']}", lambda w: M.ms_gemm_bf16(x_h, w, bias, [q, k, v], splits["qkv"], ws), x_h),
        ("out+add+norm", hid, qd, f"K split {splits['out']}, residual add and RMSNorm in the reduction", lambda w: M.ms_gemm_add_rmsnorm_bf16(x_q, w, h, norm_w, 1e-6, x_out, splits["out"], ws), x_q),
        ("gate/up+SwiGLU", 2 * inter, hid, "SwiGLU in the epilogue", lambda w: M.ms_gemm_swiglu_bf16(x_h, w, act, ws), x_h),
        ("down+add+norm", hid, inter, f"K split {splits['down']}, residual add and RMSNorm in the reduction", lambda w: M.ms_gemm_add_rmsnorm_bf16(x_i, w, h, norm_w, 1e-6, x_out, splits["down"], ws), x_i),
        ("lm_head", vocab, hid, "logits", lambda w: M.ms_gemm_bf16(x_h, w, None, [logits], 1, ws), x_h),
    ]

    def timed(fn, weights):
        state = [0]

        def call():
            fn(weights[state[0] % len(weights)])
            state[0] += 1
        for _ in range(max(1, args.warmup)):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps * 1e3

    table, flops_total, us_total = [], 0.0, 0.0
    for name, n, kk, what, fn, xin in cases:
        weights = copies(n, kk)
        us = timed(fn, weights)
        flops = 2.0 * rows * n * kk
        row = {"projection": name, "rows": rows, "N": n, "K": kk, "call": what, "us": round(us, 1), "pflops": round(flops / us / 1e9, 3),
               "frac_of_2.5_pflops": round(flops / us / 1e9 / 2.5, 3), "weight_gbps": round(n * kk * 2 / us / 1e3, 1)}
        if args.library_reference:   # a reference, not on any path of the library: the bare product through torch.mm
            ref = torch.empty(rows, n, dtype=torch.bfloat16, device=dev)
            row["library_us_bare_product"] = round(timed(lambda w: torch.mm(xin, w.t(), out=ref), weights), 1)
            del ref
        table.append(row)
        flops_total += flops
        us_total += us
        del weights
    step_us = 28 * sum(r["us"] for r in table[:4]) + table[4]["us"]
    result = {
        "metric": f"decoder_projections_pflops_rows{rows}", "value": round(flops_total / us_total / 1e9, 3), "unit": "PFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(step_us / 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"qwen2.5-7b_projections_rows{rows}", "note": "ms_per_step = 28 blocks' four projections + the LM head, stand-alone times added up"},
        "projections": table,
        "roofline": {"kernel": "gemm_tn_bf16 (+ its reduction kernels)", "bound": "mfma", "achieved": round(flops_total / us_total / 1e6, 1),
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops_total / us_total / 1e6 / 2500.0, 4), "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(result))


def cpu_baseline(args, ses, sh, ids, lengths, q, k_new, v_new, pos_d, out, M, S, W):
    """The oracle as it stands, timed on the host cores over the first sequences of the batch
    (layer 0, all 9 x 28 query rows each), and compared with what the GPU produced for them.  The
    oracle's own code is single-threaded per call; here its per-sequence routine is called once per
    (sequence, KV head) -- the rows of that head's query heads -- from a pool of threads, one per
    core this process may run on (numpy releases the interpreter lock inside its kernels)."""
    import concurrent.futures as cf

    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits

    from oracle import memosight_oracle as O

    n = max(1, min(args.cpu_seqs, sh.batch))
    nproc = os.cpu_count() or 1
    usable = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else nproc
    # the GPU machines give one GPU's job 16 cores whatever nproc says
    threads = max(1, min(usable, 16, n * sh.n_kv_heads))
    nv, nf = sh.n_verify, sh.n_foresight
    group = sh.n_q_heads // sh.n_kv_heads
    # fresh GPU result for layer 0 with the final cache state
    ses.attention(0, ids, nv, nf, q, k_new[0], v_new[0], pos_d, None, 0.0, out)
    torch.cuda.synchronize()
    got = S.to_host_f32(out[:n])
    tables = ses.page_tables(ids[:n])
    used = sorted({p for t in tables for p in t})
    remap = {p: i for i, p in enumerate(used)}
    pool = S.to_host_f32(ses.pool[0, torch.tensor(used, device="cuda")])[None]
    ora = O.PagedCache(1, sh.n_kv_heads, sh.head_dim, len(used), dtype=O.BF16, rope_base=sh.rope_base,
                       max_seqs=n, pool=np.ascontiguousarray(pool))
    oids = [ora.seq_import(lengths[b], [remap[p] for p in tables[b]]) for b in range(n)]
    qh, kh, vh = S.to_host_f32(q[:n]), S.to_host_f32(k_new[0, :n]), S.to_host_f32(v_new[0, :n])
    pos = pos_d[:n].cpu().numpy()
    ctx = O.default_ctx_new(nv, nf)
    want = np.empty((n, nv + nf, sh.n_q_heads, sh.head_dim), np.float64)

    def one(task):
        b, g = task
        rows = [(i, h) for i in range(nv + nf) for h in range(g * group, (g + 1) * group)]
        res = O.attention_rows(ora, 0, oids[b], qh[b], kh[b], vh[b], pos[b], ctx, rows=rows)
        want[b, :, g * group:(g + 1) * group] = res[:, g * group:(g + 1) * group]

    tasks = [(b, g) for b in range(n) for g in range(sh.n_kv_heads)]
    with threadpool_limits(limits=1):       # one BLAS thread per worker: the workers are the parallelism
        t0 = time.perf_counter()
        with cf.ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, tasks))
        dt = time.perf_counter() - t0
    nbytes = sum(2 * lengths[b] * sh.n_kv_heads * sh.head_dim * 2 for b in range(n))
    # the same oracle on one thread: one sequence of 4096 cached tokens, 4 verify + 3 foresight queries, all heads
    c2 = W.config2()
    inp = W.attention_inputs(c2, 2)
    ora2 = O.PagedCache(1, c2.n_kv_heads, c2.head_dim, c2.n_pages, dtype=O.BF16, rope_base=c2.rope_base, max_seqs=1,
                        pool=np.ascontiguousarray(W.bits_as_f32(inp.pool)))
    oid2 = ora2.seq_import(c2.lengths[0], inp.page_tables[0])
    p0 = inp.first_pid[0]       # verify block at consecutive positions, the foresight tokens right after it (Section 2.1.1)
    pos2 = np.asarray(list(range(p0, p0 + c2.n_verify)) + O.foresight_pids(p0 + c2.n_verify - 1, c2.n_foresight), dtype=np.int64)
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        O.attention_rows(ora2, 0, oid2, W.bits_as_f32(inp.q[0]), W.bits_as_f32(inp.k_new[0]), W.bits_as_f32(inp.v_new[0]),
                         pos2, O.default_ctx_new(c2.n_verify, c2.n_foresight))
        dt2 = time.perf_counter() - t0
    bytes2 = 2 * c2.lengths[0] * c2.n_kv_heads * c2.head_dim * 2
    err = float(np.abs(got - want).max())
    rel = float(np.abs(got - want).mean() / np.abs(want).mean())
    return {
        "value": round(nbytes / dt / 1e9, 4),
        "unit": "GB/s",
        "cores": threads,
        "nproc": nproc,
        "cores_usable": usable,
        "kind": "oracle",
        "sample": f"{n} of {sh.batch} sequences, layer 0, all {nv + nf} x {sh.n_q_heads} query rows, one task per (sequence, KV head) "
                  f"on {threads} threads, {nbytes / 1e6:.1f} MB of KV in {dt:.2f} s (1 of {sh.n_layers} layers of one step)",
        "single_thread": {"workload": "one sequence, 4096 cached tokens, 4 verify + 3 foresight, 28 / 4 heads", "seconds": round(dt2, 3),
                          "value": round(bytes2 / dt2 / 1e9, 4), "unit": "GB/s", "cores": 1},
        "gpu_vs_oracle_max_abs": round(err, 6),
        "gpu_vs_oracle_mean_rel": round(rel, 6),
        "tolerance": {"max_abs": 2e-2, "mean_rel": 1e-2},
        "within_tolerance": bool(err <= 2e-2 and rel <= 1e-2),
    }


if __name__ == "__main__":
    main()
