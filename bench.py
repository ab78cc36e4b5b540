"""Benchmark of the batched verification step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 13b] [--no-cpu-baseline] [--no-per-config]

One step = one pass of the whole hot path over one synthetic batch that is already resident in
HBM: spin_decompose (when the configuration decomposes), spin_verify_attn (schedule, stream K/V,
QK^T, mask, online softmax, PV, join) for ONE attention layer, and spin_accept (rejection mode:
row statistics, first-reject scan, residual / bonus draw).  Prints one JSON line: the headline
workload (13b) timed over exactly K steps, the same region repeated for a spread, the other four
configurations each after a warm-up of its own (`per_config`), and the CPU oracle as a baseline.
"""
import argparse
import dataclasses
import gc
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
REPEATS = 5             # further timed regions of K steps after the one the headline value comes from


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_leg(cfg, batch, ab, budget_s):
    """Time the oracle on a bounded sample of the batch; returns (verified draft tokens/s for the whole batch
    by linear scaling, description of the sample, CPU seconds used per wall second, K/V GB/s of its attention)."""
    import numpy as np
    import spin_inputs as si
    from oracle import spin_oracle as orc
    t = batch.table
    rng = np.random.default_rng(0)
    n_tok = (t.prefix_len.astype(np.int64) + t.draft_len)
    total_cells = float((n_tok * cfg.n_q_heads).sum())
    kb, vb, qb = si.host_elems(batch.k_pool), si.host_elems(batch.v_pool), si.host_elems(batch.q)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    tl_all, dl_all = ab.target_logits.cpu().numpy(), ab.draft_logits.cpu().numpy()
    toks_all, ua_all, us_all = ab.draft_tokens.cpu().numpy(), ab.u_accept.cpu().numpy(), ab.u_sample.cpu().numpy()
    cpu0, wall0 = time.process_time(), time.perf_counter()
    done_cells, t_attn, n_pairs = 0.0, 0.0, 0
    while t_attn < budget_s * 0.7 and n_pairs < t.n_req * cfg.n_q_heads:
        i = int(rng.integers(t.n_req))
        h = int(rng.integers(cfg.n_q_heads))
        t0 = time.perf_counter()
        orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                             qb, kb, vb, cfg.n_q_heads, cfg.n_kv_heads, scale, requests=[i], heads=[h])
        t_attn += time.perf_counter() - t0
        done_cells += float(n_tok[i])
        n_pairs += 1
    attn_full = t_attn * total_cells / done_cells
    # acceptance: requests in order until the rest of the budget is used
    nreq, t_acc = 0, 0.0
    while nreq < t.n_req and t_acc < budget_s * 0.3:
        r0, r1 = int(t.q_offset[nreq]), int(t.q_offset[nreq + 1])
        t0 = time.perf_counter()
        orc.accept_rejection(t.draft_len[nreq:nreq + 1], toks_all[r0:r1], tl_all[r0 + nreq: r1 + nreq + 1], dl_all[r0:r1],
                             ua_all[r0:r1], us_all[nreq:nreq + 1])
        t_acc += time.perf_counter() - t0
        nreq += 1
    busy = (time.process_time() - cpu0) / max(time.perf_counter() - wall0, 1e-9)
    acc_full = t_acc * t.n_req / nreq
    sample = (f"attention: {n_pairs} random (request, head) pairs = {done_cells / total_cells:.3%} of the batch's "
              f"key-head rows in {t_attn:.1f} s; acceptance: first {nreq} of {t.n_req} requests in {t_acc:.2f} s; "
              f"both scaled linearly to the whole batch")
    kv_gbs = si.algorithmic_kv_bytes(t, cfg.n_kv_heads, cfg.head_dim) / attn_full / 1e9
    return t.n_rows / (attn_full + acc_full), sample, busy, kv_gbs


def cpu_baseline(cfg, batch, ab, budget_s=10.0):
    """The float64 oracle, as it stands, timed on this machine's host cores on a bounded sample of the same
    batch: once as it runs by default (numpy's BLAS pool free to use every core) and once held to one thread."""
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        pool = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits, pool = None, 1
    v_all, sample, busy_all, gbs_all = _oracle_leg(cfg, batch, ab, budget_s)
    res = {"value": v_all, "unit": "verified draft tokens/s", "cores": max(1, int(math.ceil(busy_all - 0.05))),
           "kind": "oracle", "sample": sample, "attention_kv_gbs": gbs_all,
           "nproc": os.cpu_count(), "cpus_allowed": len(os.sched_getaffinity(0)), "cpu_model": cpu_model(),
           "blas_threads_available": int(pool), "cpu_seconds_per_wall_second": round(busy_all, 2),
           "note": "cores = CPU seconds the oracle used per wall second, rounded up: its loops over requests and heads "
                   "are Python, only the small matrix products inside may use the BLAS pool"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            v_one, sample_one, busy_one, gbs_one = _oracle_leg(cfg, batch, ab, budget_s)
        res["one_thread"] = {"value": v_one, "unit": "verified draft tokens/s", "cores": 1, "sample": sample_one,
                             "attention_kv_gbs": gbs_one,
                             "cpu_seconds_per_wall_second": round(busy_one, 2)}
    return res


def calib_stream(args):
    """What a kernel that only reads reaches on this machine: 4 GiB in 4 KiB blocks, in order and shuffled, plain and
    non-temporal loads, one wavefront per workgroup with 16 KiB in flight (the attention kernel's way of loading)."""
    import ctypes as C
    import torch
    from paper_2503_15921_amd.build import PROBE_LIB
    lib = C.CDLL(PROBE_LIB)
    lib.spin_probe_read_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spin_probe_read_blocks.restype = C.c_int
    dev = "cuda:0"
    n_bytes = 4 << 30
    n_blocks = n_bytes // 4096
    buf = torch.ones(n_bytes // 4, dtype=torch.int32, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu").manual_seed(1)
    tables = {"linear": torch.arange(n_blocks, dtype=torch.int32),
              "shuffled": torch.randperm(n_blocks, generator=g).to(torch.int32)}
    out = {"bytes_per_launch": n_bytes, "block_bytes": 4096, "launches_timed": args.steps, "results": []}
    stream = C.c_void_p(torch._C._cuda_getCurrentRawStream(0))
    for order, tab in tables.items():
        tab = tab.to(dev)
        for per_wave in (1024, 256, 64):          # 1024 wavefronts (one per SIMD) ... 16384
            n_waves = n_blocks // per_wave
            for nt in (1, 0):
                def launch():
                    rc = lib.spin_probe_read_blocks(buf.data_ptr(), tab.data_ptr(), n_waves, per_wave, nt, sink.data_ptr(), stream)
                    if rc:
                        raise RuntimeError(f"probe launch failed: hipError {rc}")
                for _ in range(args.warmup):
                    launch()
                times = []
                for _ in range(args.steps):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(); launch(); e1.record()
                    e1.synchronize()
                    times.append(e0.elapsed_time(e1))
                med = statistics.median(times)
                out["results"].append({"order": order, "wavefronts": n_waves, "blocks_per_wavefront": per_wave,
                                       "nontemporal": bool(nt), "ms_median": med, "ms_min": min(times),
                                       "gbs_median": n_bytes / med / 1e6, "gbs_best": n_bytes / min(times) / 1e6})
    # What result rows written during the stream cost it: 1024 readers over the shuffled table, and beside them 256
    # writer wavefronts that spread 18.9 MB (the final rows of the 70b_gqa batch) over the stream's duration.
    lib.spin_probe_read_beside_writers.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_uint64,
                                                   C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spin_probe_read_beside_writers.restype = C.c_int
    tab = tables["shuffled"].to(dev)
    wbuf = torch.zeros((64 << 20) // 4, dtype=torch.int32, device=dev)
    out["writes_during_stream"] = []
    for name, writers, chunks, pause, mode in (("no writers", 0, 0, 0, 0), ("plain stores", 256, 18, 16, 0),
                                               ("non-temporal stores", 256, 18, 16, 1), ("write-through stores", 256, 18, 16, 2),
                                               ("plain stores to one cached chunk per writer", 256, 18, 16, 3)):
        def launch():
            rc = lib.spin_probe_read_beside_writers(buf.data_ptr(), tab.data_ptr(), 1024, n_blocks // 1024, wbuf.data_ptr(),
                                                    wbuf.numel() * 4, writers, chunks, pause, mode, sink.data_ptr(), stream)
            if rc:
                raise RuntimeError(f"probe launch failed: hipError {rc}")
        for _ in range(args.warmup):
            launch()
        times = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); launch(); e1.record()
            e1.synchronize()
            times.append(e0.elapsed_time(e1))
        out["writes_during_stream"].append({"writers": name, "mb_written": writers * chunks * 4096 / 1e6,
                                            "ms_median": statistics.median(times), "ms_min": min(times)})
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="13b")
    ap.add_argument("--seed", type=int, default=3)
    ap.add_argument("--page-size", type=int, default=0, help="tokens per KV page (0 = the configuration's, 16)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"], help="element type of Q, K, V and the output")
    ap.add_argument("--kv-layout", default="hnd", choices=["hnd", "nhd", "paired", "paired-head"],
                    help="memory order of a KV page: [head][token][dim] (default), [token][head][dim], or K and V pages of the first kind "
                         "paired in one allocation ([page][K|V][head][token][dim])")
    ap.add_argument("--pages-in-order", action="store_true",
                    help="every request's pages consecutive in the pool (default: a shuffled pool, as after long service)")
    ap.add_argument("--waves", type=int, default=0, help="wavefronts per attention launch (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the pass over the other four configurations")
    ap.add_argument("--repeats", type=int, default=REPEATS, help="further timed regions of K steps, for the spread")
    ap.add_argument("--append", action="store_true",
                    help="the step also puts the draft tokens' K/V rows into the cache first (spin_append_kv)")
    ap.add_argument("--tree", default="", help="drafts are token trees of this shape (random, star, wide, chain): "
                                               "spin_verify_attn_tree and spin_accept_tree instead of the linear calls "
                                               "(the acceptance kernels of the tree call are not timed separately)")
    ap.add_argument("--decomp", default="config",
                    help="decomposition of the batch: config (the configuration's own), none, q:<width>, kv:<length>, "
                         "search:<max sub-requests> (the padding-minimising length search of Sec. V-A)")
    ap.add_argument("--microbatches", type=int, default=1,
                    help="split the batch into this many micro-batches of about equal K/V volume, issued round-robin "
                         "on --streams streams (acceptance of one overlaps attention of the next)")
    ap.add_argument("--streams", type=int, default=2)
    ap.add_argument("--reuse-plan", action="store_true",
                    help="let the library launch from the tables of the previous step (what the other layers of "
                         "one step do); off by default: every timed step plans and uploads afresh")
    ap.add_argument("--profile-every", type=int, default=10,
                    help="the library's HIP events time every n-th step of the timed region")
    ap.add_argument("--calib-copy", action="store_true",
                    help="instead of the step, run a plain 1 GiB device copy per step (counter calibration)")
    ap.add_argument("--calib-stream", action="store_true",
                    help="instead of the step, measure the streaming-read ceiling of this box (4 GiB in 4 KiB blocks, "
                         "in order and shuffled, plain and non-temporal loads)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2503_15921_amd as spin
    import spin_inputs as si

    dev = "cuda:0"
    if args.calib_copy:
        # known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE: each step reads 1 GiB and writes 1 GiB
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes_read_per_step": 1 << 30, "calib_copy_bytes_written_per_step": 1 << 30,
                          "steps": args.warmup + args.steps}))
        return
    if args.calib_stream:
        calib_stream(args)
        return
    elem = torch.bfloat16 if args.dtype == "bf16" else torch.float16

    def run_config(cfg, repeats, keep_inputs=False, rho=None, decomp=None):
        """Warm up, then time 1 + repeats regions of args.steps steps of `cfg`'s batch.  Returns a dict of figures
        (region 0 is the one a headline is taken from) and, on request, the inputs for the CPU baseline."""
        batch = si.make_verify_batch(cfg, args.seed, device=dev, dtype=elem, shuffle_pages=not args.pages_in_order)
        if args.kv_layout == "nhd":
            # same logical [page][head][token][dim] tensors over [page][token][head][dim] memory: the library reads the strides
            batch.k_pool = batch.k_pool.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            batch.v_pool = batch.v_pool.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        if args.kv_layout == "paired":
            # one allocation, [page][K|V][head][token][dim]: the K and V of a (page, head) are 2 x 4 KiB side by side
            both = torch.stack([batch.k_pool, batch.v_pool], dim=1).contiguous()
            batch.k_pool, batch.v_pool = both[:, 0], both[:, 1]
        if args.kv_layout == "paired-head":
            # one allocation, [page][head][K|V][token][dim]: the K and V of a (page, head) are 8 KiB in one piece
            both = torch.stack([batch.k_pool, batch.v_pool], dim=2).contiguous()
            batch.k_pool, batch.v_pool = both[:, :, 0], both[:, :, 1]
        t = batch.table
        # Batches whose K/V is smaller than the chip's last-level cache would be flattered by it: every step reads another
        # copy of the pools, enough copies that 2 GB pass between two uses of the same bytes (one copy for 13b and 70b_gqa).
        kv_once = si.algorithmic_kv_bytes(t, cfg.n_kv_heads, cfg.head_dim)
        n_copies = max(1, min(16, -(-(2 << 30) // max(kv_once, 1))))
        if args.kv_layout == "paired":
            pools = [(batch.k_pool, batch.v_pool)] + [(b[:, 0], b[:, 1]) for b in (both.clone() for _ in range(n_copies - 1))]
        elif args.kv_layout == "paired-head":
            pools = [(batch.k_pool, batch.v_pool)] + [(b[:, :, 0], b[:, :, 1]) for b in (both.clone() for _ in range(n_copies - 1))]
        else:
            pools = [(batch.k_pool, batch.v_pool)] + [(batch.k_pool.clone(), batch.v_pool.clone()) for _ in range(n_copies - 1)]
        step_no = [0]
        ab = si.make_accept_batch(t.draft_len, cfg.vocab, cfg.logit_sigma, args.seed, device=dev, rho=rho)
        M = max(1, args.microbatches)
        S = 1 if M == 1 else max(1, min(args.streams, M))
        ctxs = [spin.SpinContext(0) for _ in range(S)]
        for c in ctxs:
            c.set_plan_reuse(args.reuse_plan)
            if args.waves:
                c.set_waves(args.waves)
        streams = [torch.cuda.current_stream()] if S == 1 else [torch.cuda.Stream() for _ in range(S)]
        out = torch.empty_like(batch.q)
        n_acc = torch.empty(t.n_req, dtype=torch.int32, device=dev)
        nxt = torch.empty_like(n_acc)
        k_new = v_new = None
        if args.append:
            g = torch.Generator(device="cpu").manual_seed(args.seed)
            shape = (t.n_rows, cfg.n_kv_heads, cfg.head_dim)
            k_new = torch.randn(shape, generator=g).to(elem).to(dev)
            v_new = torch.randn(shape, generator=g).to(elem).to(dev)

        parents, masks = si.random_trees(t.draft_len, np.random.default_rng(args.seed), args.tree) if args.tree else (None, None)
        path = torch.empty(t.n_rows, dtype=torch.int32, device=dev)
        # micro-batches: contiguous request ranges of about equal K/V volume
        tok = np.cumsum(t.prefix_len.astype(np.int64) + t.draft_len)
        cuts = [0] + [int(np.searchsorted(tok, tok[-1] * (m + 1) / M, side="left")) + 1 for m in range(M - 1)] + [t.n_req]
        cuts = sorted(set(min(c, t.n_req) for c in cuts))
        mbs = []
        for i0, i1 in zip(cuts[:-1], cuts[1:]):
            r0, r1 = int(t.q_offset[i0]), int(t.q_offset[i1])
            p0, p1 = int(t.pt_offset[i0]), int(t.pt_offset[i1])
            c = ctxs[len(mbs) % S]
            mbs.append(dict(
                ctx=c, stream=streams[len(mbs) % S], prefix=t.prefix_len[i0:i1], draft=t.draft_len[i0:i1],
                tab=c.make_table(t.prefix_len[i0:i1], t.draft_len[i0:i1], t.q_offset[i0:i1 + 1] - r0,
                                 t.pt_offset[i0:i1 + 1] - p0, t.page_table[p0:p1]),
                q=batch.q[r0:r1], out=out[r0:r1], tokens=ab.draft_tokens[r0:r1], target=ab.target_logits[r0 + i0:r1 + i1],
                dlogits=ab.draft_logits[r0:r1], u_acc=ab.u_accept[r0:r1], u_smp=ab.u_sample[i0:i1],
                n_acc=n_acc[i0:i1], nxt=nxt[i0:i1], masks=masks[r0:r1] if args.tree else None,
                parents=parents[r0:r1] if args.tree else None, path=path[r0:r1],
                k_new=k_new[r0:r1] if args.append else None, v_new=v_new[r0:r1] if args.append else None))

        def decomposition(prefix, draft):
            d = decomp or args.decomp
            if d == "config":
                d = f"q:{cfg.q_split_width}" if cfg.q_split_width else "none"
            if d == "none":
                return None
            kind, _, val = d.partition(":")
            if kind == "q":
                return spin.decompose(prefix, draft, spin.DECOMP_Q_SPLIT, q_width=int(val))[0]
            if kind == "kv":
                return spin.decompose(prefix, draft, spin.DECOMP_KV_SPLIT, kv_len=int(val))[0]
            if kind == "search":
                return spin.decompose(prefix, draft, spin.DECOMP_KV_SEARCH, max_subreq=int(val), l_min=64,
                                      l_max=int(prefix.max() + draft.max()), l_step=16)[0]
            raise SystemExit(f"unknown --decomp {args.decomp}")

        attn_done = [torch.cuda.Event() for _ in mbs]

        def step():
            k_pool, v_pool = pools[step_no[0] % n_copies]
            step_no[0] += 1
            for k, mb in enumerate(mbs):
                subs = decomposition(mb["prefix"], mb["draft"])
                with torch.cuda.stream(mb["stream"]):
                    if S > 1:
                        # attention kernels fill the chip: chain them, so that only the acceptance of one
                        # micro-batch runs beside the attention of the next
                        mb["stream"].wait_event(attn_done[k - 1])
                    if args.append:
                        mb["ctx"].append_kv(mb["tab"], k_pool, v_pool, mb["k_new"], mb["v_new"])
                    mb["ctx"].verify_attn(mb["tab"], k_pool, v_pool, mb["q"], mb["out"], cfg.n_q_heads, subs=subs,
                                          tree_mask=mb["masks"])
                    if S > 1:
                        attn_done[k].record(mb["stream"])
                    if args.tree:
                        mb["ctx"].accept_tree(spin.ACCEPT_REJECTION, mb["draft"], mb["parents"], mb["tokens"], mb["target"],
                                              mb["dlogits"], mb["u_acc"], mb["u_smp"], mb["n_acc"], mb["path"], mb["nxt"])
                    else:
                        mb["ctx"].accept(spin.ACCEPT_REJECTION, mb["draft"], mb["tokens"], mb["target"], mb["dlogits"],
                                         mb["u_acc"], mb["u_smp"], mb["n_acc"], mb["nxt"])

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        # The library's events time every tenth step of a timed region: three event records per timed call
        # cost about 27 us of stream time per step, which would otherwise be 4 % of the figure being measured
        # (0.4 % this way; the kernel averages do not depend on the sampling).
        regions = []
        for _ in range(1 + repeats):
            for c in ctxs:
                c.profile_begin(args.steps * len(mbs), every=args.profile_every)
            # (the interpreter's cyclic garbage collector stays out of the timed region, as in `timeit`: a full collection
            # over the tables and tensors this script holds takes 40 ms, more than sixty steps)
            gc.collect()
            gc.disable()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            gc.enable()
            ms = {"attn": 0.0, "join": 0.0, "accept_stats": 0.0, "accept_draw": 0.0}
            calls = [0, 0]
            for c in ctxs:
                m1, c1 = c.profile_end()
                for k in ms:
                    ms[k] += m1[k]
                calls = [calls[0] + c1[0], calls[1] + c1[1]]
            # kernel times are per timed step: the sum over the step's micro-batches
            n_a, n_c = max(calls[0] / len(mbs), 1), max(calls[1] / len(mbs), 1)
            regions.append({"ms_per_step": wall * 1e3 / args.steps, "timed_steps": calls[0] // len(mbs),
                            "kernel_ms": {"attn": ms["attn"] / n_a, "join": ms["join"] / n_a,
                                          "accept_stats": ms["accept_stats"] / n_c, "accept_draw": ms["accept_draw"] / n_c}})
        # the host's share of a step (decomposition, scheduling, staging, launches), measured apart from the timed
        # regions with an idle GPU in front of every step so that no call waits for a staging buffer
        host = 0.0
        for _ in range(10):
            torch.cuda.synchronize()
            h0 = time.perf_counter()
            step()
            host += time.perf_counter() - h0
        torch.cuda.synchronize()
        torch.cuda.synchronize()
        mean_accepted = float(n_acc.float().mean().item())
        for c in ctxs:
            c.close()
        kv_bytes = si.algorithmic_kv_bytes(t, cfg.n_kv_heads, cfg.head_dim)
        # strips of more than 32 (draft row x query head) rows run on the grouped-query kernel
        group = cfg.n_q_heads // cfg.n_kv_heads
        attn_kernel = "verify_attn_group_kernel" if min(int(t.draft_len.max()), 64 // group) * group > 32 else "verify_attn_kernel"
        res = dict(cfg=cfg, table=t, regions=regions, host_ms=host * 1e3 / 10, kv_bytes=kv_bytes, attn_kernel=attn_kernel,
                   n_mbs=len(mbs), n_streams=S, kv_pool_copies=n_copies, mean_accepted=mean_accepted)
        if keep_inputs:
            res["batch"], res["ab"] = batch, ab
        return res

    def spread(regions):
        steps = [r["ms_per_step"] for r in regions]
        attn = [r["kernel_ms"]["attn"] for r in regions]
        return {"regions": len(regions), "steps_per_region": args.steps, "ms_per_step_by_region": [round(x, 5) for x in steps],
                "ms_per_step_min": min(steps), "ms_per_step_median": statistics.median(steps), "ms_per_step_max": max(steps),
                "attn_kernel_ms_min": min(attn), "attn_kernel_ms_median": statistics.median(attn), "attn_kernel_ms_max": max(attn)}

    cfg = si.CONFIGS[args.config]
    if args.page_size:
        cfg = dataclasses.replace(cfg, page_size=args.page_size)
    head = run_config(cfg, args.repeats, keep_inputs=not args.no_cpu_baseline)
    t = head["table"]
    r0 = head["regions"][0]            # exactly K steps after W warm-up steps: the headline
    ms_per_step = r0["ms_per_step"]
    kv_bytes = head["kv_bytes"]
    attn_ms = r0["kernel_ms"]["attn"]
    achieved = kv_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms > 0 else 0.0
    with_join = kv_bytes / ((attn_ms + r0["kernel_ms"]["join"]) * 1e-3) / 1e9 if attn_ms > 0 else 0.0
    # measured HBM bytes per launch: the PMC summary of this workload as the default flags run it, else none
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{cfg.name}.json")
    as_profiled = (args.seed == 3 and args.decomp == "config" and not args.tree and not args.page_size and not args.append
                   and args.kv_layout == "hnd" and args.dtype == "bf16" and head["n_mbs"] == 1 and not args.waves)
    if as_profiled and os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
        traffic_source = (f"profiles/traffic_{cfg.name}.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this workload, "
                          f"a committed earlier measurement, not read by this run")
    res = {
        "metric": "verified draft tokens/sec + achieved KV HBM GB/s (% peak), batched verify step",
        "value": t.n_rows / (ms_per_step * 1e-3),
        "unit": "verified draft tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "host_ms_per_step": head["host_ms"], "steps_with_kernel_timing": r0["timed_steps"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_req} requests, {cfg.n_q_heads}q/{cfg.n_kv_heads}kv heads, "
                               f"head_dim {cfg.head_dim}, prefix {cfg.prefix_dist} {cfg.prefix_lo}-{cfg.prefix_hi}, "
                               f"draft {cfg.draft_dist} {cfg.draft_lo}-{cfg.draft_hi}, page {cfg.page_size}{' (token-major)' if args.kv_layout == 'nhd' else ''}, "
                               f"vocab {cfg.vocab}; " + ("KV append + " if args.append else "") + (f"{args.tree} draft trees, " if args.tree else "") +
                               "one attention layer + one rejection-sampling accept",
                   "decomposition": args.decomp, "microbatches": head["n_mbs"], "streams": head["n_streams"],
                   "plan_reuse": bool(args.reuse_plan),
                   "seed": args.seed, "draft_rows": t.n_rows, "kv_tokens": t.kv_tokens(),
                   "kv_gb_per_step": kv_bytes / 1e9, "kv_pool_copies": head["kv_pool_copies"], "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBS},
        "kernel_ms": r0["kernel_ms"],
        "kernel_ms_keys": "attn / join: attention and partial-join kernels; accept_stats: first acceptance kernel (row "
                          "statistics; the whole acceptance when the call is small enough for one kernel); accept_draw: "
                          "second acceptance kernel (accept scan + next-token draw)",
        "spread": spread(head["regions"]),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": head["attn_kernel"], "algorithmic_bytes_per_launch": kv_bytes,
                     "frac_attn_plus_join": with_join / HBM_PEAK_GBS},
    }
    if not args.no_per_config and not args.tree:
        # The literal configuration draws target and draft logits independently, so nearly every request is rejected at
        # its first row.  The same step once more with draft = 0.9 target + noise, where accepted lengths spread over
        # 0..gamma (a property of the synthetic data, reported for the acceptance kernels' sake).
        r = run_config(cfg, args.repeats, rho=0.9)
        sp = spread(r["regions"])
        res["correlated_logits"] = {"rho": 0.9, "ms_per_step": sp["ms_per_step_median"],
                                    "tokens_per_s": r["table"].n_rows / (sp["ms_per_step_median"] * 1e-3),
                                    "mean_accepted_per_request": r["mean_accepted"],
                                    "kernel_ms": {k: statistics.median(x["kernel_ms"][k] for x in r["regions"])
                                                  for k in ("attn", "join", "accept_stats", "accept_draw")}}
    if not args.no_per_config and args.config == "13b":
        # the other four configurations, each after a warm-up of its own, figures = medians over the timed regions
        per = {}
        # (skewed a second time, cut the paper's way: along the keys into rows of length L = 512, Sec. V-A)
        for name in list(si.CONFIG_ORDER) + ["skewed, KV-split L=512"]:
            if name == cfg.name:
                continue
            r = run_config(si.CONFIGS[name.split(",")[0]], args.repeats, decomp="kv:512" if "," in name else None)
            sp = spread(r["regions"])
            km = {k: statistics.median(x["kernel_ms"][k] for x in r["regions"]) for k in ("attn", "join", "accept_stats", "accept_draw")}
            gbs = r["kv_bytes"] / (km["attn"] * 1e-3) / 1e9 if km["attn"] > 0 else 0.0
            per[name] = {"ms_per_step": sp["ms_per_step_median"], "ms_per_step_min": sp["ms_per_step_min"],
                         "tokens_per_s": r["table"].n_rows / (sp["ms_per_step_median"] * 1e-3),
                         "attn_kernel": r["attn_kernel"], "attn_kernel_ms": km["attn"], "attn_kernel_ms_min": sp["attn_kernel_ms_min"],
                         "achieved_gbs": gbs, "frac": gbs / HBM_PEAK_GBS, "kernel_ms": km, "host_ms_per_step": r["host_ms"],
                         "draft_rows": r["table"].n_rows, "kv_gb_per_step": r["kv_bytes"] / 1e9,
                         "kv_pool_copies": r["kv_pool_copies"], "regions": sp["regions"], "steps_per_region": args.steps, "warmup": args.warmup}
        res["per_config"] = per
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, head["batch"], head["ab"])
    print(json.dumps(res))


if __name__ == "__main__":
    main()
