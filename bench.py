#!/usr/bin/env python3
"""Benchmark of the SPD decode-attention hot path on one MI355X.

A "step" is one pass of the whole path for one layer and one decode position: private partial attention for all
users, public batched partial attention, and the merge.  Inputs are synthetic (seeded N(0,1) caches of the named
workload) and already resident in HBM when the timed region starts.  Several copies of the KV set at distinct
addresses are cycled through so that consecutive steps do not re-read the same lines from the 256 MB last-level
cache.

Prints ONE JSON line: whole-step KV-read throughput (algorithmic K/V bytes of both owners / time per step), the
roofline position of the dominant kernel (the private partial-attention kernel) from HIP-event timing, and the fp64
CPU oracle timed on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E peak


def clone_side(side):
    import copy
    c = copy.copy(side)
    if side.paged:
        c.k_pool, c.v_pool = side.k_pool.clone(), side.v_pool.clone()
        c.block_table = side.block_table.clone()
    else:
        c.k = [t.clone() for t in side.k]
        c.v = [t.clone() for t in side.v]
    return c


def measured_traffic(config: int, kernel_name: str):
    """(bytes, source): HBM bytes per launch of the streaming kernel from the committed rocprofv3 --pmc summary of this
    workload (scaled FETCH_SIZE + WRITE_SIZE) and where that figure comes from.  bytes is None, and source says why, if
    there is no summary or it was made with another kernel instance than `kernel_name`, the one that just ran: the
    summary is a stored measurement, not one made by this run."""
    import re
    rel = os.path.join("profiles", f"partial_kernel_config{config}_pmc_traffic.txt")
    path = os.path.join(ROOT, rel)
    source = {"file": rel, "kind": "stored rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, scaled by a 256 MiB copy)",
              "kernel_that_ran": kernel_name}
    if not os.path.exists(path):
        source["why_null"] = "no summary for this workload"
        return None, source
    total, found, seen = 0.0, 0, set()
    for line in open(path):
        m = re.search(r"^\s+spd::(partial_mfma_kernel<[^>]*>).*->\s+([0-9.]+) MB scaled", line)
        if m:
            seen.add(m.group(1))
            if m.group(1) == kernel_name:
                total += float(m.group(2)) * 1e6
                found += 1
    source["kernel_in_summary"] = sorted(seen)
    if found != 2:
        source["why_null"] = "the summary was made with another kernel instance"
        return None, source
    return int(total), source


def masked_stream(torch, n_cus, wanted):
    """A HIP stream (default priority) whose kernels run only on the compute units cu with wanted(cu)."""
    import ctypes
    # the HIP runtime this process already uses (loading another copy by name would start a second runtime)
    with open("/proc/self/maps") as f:
        paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    assert len(paths) == 1, f"expected one HIP runtime in the process, found {sorted(paths)}"
    hip = ctypes.CDLL(paths.pop())
    words = (n_cus + 31) // 32
    mask = (ctypes.c_uint32 * words)()
    for cu in range(n_cus):
        if wanted(cu):
            mask[cu // 32] |= 1 << (cu % 32)
    handle = ctypes.c_void_p()
    hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                 ctypes.POINTER(ctypes.c_uint32)]
    hip.hipExtStreamCreateWithCUMask.restype = ctypes.c_int
    rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(handle), words, mask)
    assert rc == 0 and handle.value, f"hipExtStreamCreateWithCUMask failed ({rc})"
    return torch.cuda.ExternalStream(handle.value)


# ---- the users' side of --mode two_processes -------------------------------------------------------------------
# Host handshake between the service process and the users' processes: a few 64-bit counters in shared host memory.
FLAG_GO, FLAG_STOP, FLAG_DONE0 = 0, 1, 8      # done[i] / ready[i] of worker i at FLAG_DONE0 + 2 i, + 2 i + 1
SPIN_LIMIT_S = 120.0                           # every wait on a counter gives up after this long


def spin_until(flags, idx, value, also_stop=False, proc=None):
    """Waits until flags[idx] >= value (or, with also_stop, the stop flag is up); False on time-out, or when the
    process `proc` that should raise the counter has ended."""
    t0 = time.perf_counter()
    n = 0
    while flags[idx] < value:
        if also_stop and flags[FLAG_STOP]:
            return True
        n += 1
        if (n & 0x3fff) == 0:
            if time.perf_counter() - t0 > SPIN_LIMIT_S:
                return False
            if proc is not None and proc.poll() is not None:
                return bool(flags[idx] >= value)
    return True


def worker_main(args):
    """One users' process (section 4, step 3b): holds the private caches of its share of the users, maps the service's
    q / A_in / lse_in buffers, and answers every step with spd_partial_attn_private written in place."""
    import json as js
    import numpy as np
    import torch
    import paper_2409_19134_amd as spd
    import workloads
    from paper_2409_19134_amd import ipc

    idx, n_workers = (int(x) for x in args.worker.split("/"))
    flags = np.memmap(args.shm, dtype=np.int64, mode="r+", shape=(64,))     # the service's counters (a file in /dev/shm)
    dev = "cuda:0"
    shape = tuple(int(x) for x in args.shape.split(",")) if args.shape else None
    dtype = {None: None, "bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[args.dtype]
    len_ranges = tuple(int(x) for x in args.lens.split(",")) if args.lens else None
    wl = workloads.make_workload(args.config, dev, layout=args.layout, shape=shape, dtype=dtype, n_users=args.users,
                                 page_tokens=args.page_tokens, len_ranges=len_ranges)
    wl.public = None                               # the service's, not ours
    msg = js.loads(sys.stdin.readline())           # what the service shares
    copies = int(msg["copies"])
    U = wl.n_users
    u0, u1 = U * idx // n_workers, U * (idx + 1) // n_workers
    sides = [wl.private] + [clone_side(wl.private) for _ in range(copies - 1)]

    def view_of(side):
        if side.paged:
            return spd.KVView(side.lens[u0:u1], side.token_stride, side.head_stride, k_pool=side.k_pool, v_pool=side.v_pool,
                              block_table=side.block_table[u0:u1], block_size=side.page_tokens,
                              block_stride=side.block_stride)
        return spd.KVView(side.lens[u0:u1], side.token_stride, side.head_stride, k=side.k[u0:u1], v=side.v[u0:u1],
                          head_strides=None if side.head_strides is None else side.head_strides[u0:u1])
    views = [view_of(s) for s in sides]
    sh = spd.make_shape(wl.dtype, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.scale)
    q = ipc.MappedBuffer(bytes.fromhex(msg["q"]), (U, wl.n_q_heads, wl.head_dim), wl.dtype, dev)
    a_in = ipc.MappedBuffer(bytes.fromhex(msg["a_in"]), (U, wl.n_q_heads, wl.head_dim), torch.float32, dev)
    lse_in = ipc.MappedBuffer(bytes.fromhex(msg["lse_in"]), (U, wl.n_q_heads), torch.float32, dev)
    use_events = msg["sync"] == "events"
    ev_q = ipc.SharedEvent(bytes.fromhex(msg["ev_q"])) if use_events else None
    ev_done = ipc.SharedEvent() if use_events else None
    ctx = spd.Context(0)
    stream = torch.cuda.current_stream()
    qs, As, Ls = q.tensor[u0:u1], a_in.tensor[u0:u1], lse_in.tensor[u0:u1]
    scratch_a, scratch_l = torch.empty_like(As), torch.empty_like(Ls)
    for v in views:                                # every view's schedule is built before the first timed step
        ctx.spd_partial_attn_private(sh, qs, v, scratch_a, scratch_l, stream)
    torch.cuda.synchronize()
    print(js.dumps({"ev_done": ev_done.handle.hex() if use_events else None, "users": [u0, u1]}), flush=True)
    k = 1
    while True:
        if not spin_until(flags, FLAG_GO, k, also_stop=True) or flags[FLAG_STOP]:
            break
        if u1 > u0:
            if use_events:
                ev_q.wait(stream)                  # the service's previous merge has read A_in; q is in place
            ctx.spd_partial_attn_private(sh, qs, views[(k - 1) % copies], As, Ls, stream)
            if use_events:
                ev_done.record(stream)
            else:
                stream.synchronize()
        flags[FLAG_DONE0 + 2 * idx] = k            # enqueued (events) or finished (host)
        k += 1
    torch.cuda.synchronize()
    ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = Llama-3-8B shape, 16 users: the headline)")
    ap.add_argument("--copies", type=int, default=0, help="KV set copies cycled through (0 = enough for > 1 GB, at most 8)")
    ap.add_argument("--mode", default="fused", choices=["fused", "calls", "calls_public_first", "streams", "two_parties", "per_user_streams",
                                                        "two_processes"],
                    help="fused: spd_decode_step (both owners' pieces in one launch, one closing kernel); "
                         "calls: the three entry points in sequence on one stream (private, public, merge); "
                         "calls_public_first: the same with the public call first; "
                         "streams: private and public calls on two streams of equal priority, joined before the merge "
                         "(these three are the orderings of the paper's overlap study, section 5); "
                         "two_parties: the users' call (private partials) and the service's call (public partial + merge); "
                         "per_user_streams: as two_parties, but every user's private call is made on its own (one user, "
                         "own context, own stream, as the paper's per-user processes would), joined before the service's call; "
                         "two_processes: the paper's deployment on one GPU - the private partials are computed by "
                         "--user-procs other processes that hold the private caches and write (A_in, lse_in) into "
                         "buffers of this (the service's) process through HIP IPC memory handles; this process runs "
                         "the public partial beside them and merges")
    ap.add_argument("--user-procs", type=int, default=1, metavar="N",
                    help="two_processes mode: users' processes (each takes an equal share of the users; at most 8)")
    ap.add_argument("--ipc-sync", default="host", choices=["host", "events"],
                    help="two_processes mode: how the two sides' streams are ordered - host synchronisation of each "
                         "side's stream before the other side goes on (default), or IPC events recorded and waited for "
                         "on the GPU, the host only saying when they have been enqueued (the HIP runtime of this image "
                         "hands out IPC event handles but refuses to record such an event, so this form fails here)")
    ap.add_argument("--worker", default=None, help=argparse.SUPPRESS)     # i/N: this process is users' process i of N
    ap.add_argument("--shm", default=None, help=argparse.SUPPRESS)
    ap.add_argument("--public-cus", type=int, default=0, metavar="N",
                    help="streams mode only: give the public call's stream N compute units and the private call's "
                         "stream the others (HIP compute-unit masks; 0 = both streams may use every unit)")
    ap.add_argument("--graph", action="store_true",
                    help="fused and per_user_streams modes: record one step on every KV copy (think: the layers of a model, --copies N) "
                         "into one HIP graph after the warm-up and time replays of it; --steps must be a multiple of "
                         "the number of copies")
    ap.add_argument("--decode-loop", type=int, default=0, metavar="N",
                    help="fused mode only: a decode loop instead of one repeated step - every step appends a token per "
                         "user to the public cache (as --append) and the public lengths grow by one per step; after N "
                         "steps (at most 32) the loop starts over on the next KV copy.  Shows what a growing cache costs "
                         "(nothing, when the schedule of the first step serves the following ones); no oracle leg")
    ap.add_argument("--append", action="store_true",
                    help="fused mode only: also append one new token per user to the public cache in the same launch "
                         "(its slot is the cache's last token, rewritten every step)")
    ap.add_argument("--layout", default=None, choices=["hnd", "hnd_exact", "nhd"], help="contiguous KV layout override")
    ap.add_argument("--shape", default=None, metavar="HQ,HKV,D",
                    help="replace the configuration's head counts and head size (same users, lengths and seeds): other "
                         "model shapes, e.g. 32,8,64 or 32,32,128; not one of the five benchmark workloads")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16", "f32"], help="replace the configuration's element type")
    ap.add_argument("--users", type=int, default=None, help="replace the configuration's number of users (same length law)")
    ap.add_argument("--lens", default=None, metavar="PLO,PHI,OLO,OHI",
                    help="replace the configuration's length law: private lengths uniform in [PLO, PHI], public in "
                         "[OLO, OHI] (e.g. 64,512,1,256 with --users 32: the paper's own prompt lengths and batch size)")
    ap.add_argument("--page-tokens", type=int, default=16, choices=[16, 32, 64, 128, 256],
                    help="tokens per page of the paged workload (config 5; 16 is the benchmark's)")
    ap.add_argument("--pointer-tables", action="store_true",
                    help="contiguous layouts: also pass the per-user pointers in device arrays (address-independent "
                         "schedules, shared by the layers of a model; one more dependent scalar load per segment)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg altogether (its timing and the parity check made on its output)")
    ap.add_argument("--no-check", action="store_true", help="skip the comparison of the GPU result with the oracle's")
    ap.add_argument("--cpu-seconds", type=float, default=1.5,
                    help="wall-clock seconds of oracle passes in the cpu_baseline leg (times the cores it uses: CPU work)")
    ap.add_argument("--no-sub-records", action="store_true",
                    help="default workload only: skip the three_calls / two_parties legs (the same step through the "
                         "three named entry points, and as the users' call plus the service's call) and the short runs "
                         "of workloads 1, 3, 4 and 5 (\"other_workloads\")")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, so that a rocprofv3 --pmc run has a dispatch of known "
                         "traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if args.worker:
        return worker_main(args)

    out, parity_failed = run_once(args)
    plain_default = (args.config == 2 and args.mode == "fused" and not any(
        (args.graph, args.append, args.decode_loop, args.public_cus, args.layout, args.shape, args.dtype, args.users,
         args.lens, args.pointer_tables, args.copies)) and args.page_tokens == 16)
    if plain_default and not args.no_sub_records and not parity_failed:
        # The other benchmark workloads, after the timed region of the headline one and in the same process: fewer
        # steps (their steps are 15 to 55 times longer), the same fused step, the same clocks, the same parity check
        # (one query head of every (user, KV head) stream against the oracle).  Not part of `value`.
        import copy
        others = []
        for cfg in (1, 3, 4, 5):
            a = copy.copy(args)
            a.config = cfg
            a.steps = max(10, min(args.steps, 100 if cfg != 1 else 1000))
            a.warmup = max(2, min(args.warmup, 10))
            a.no_sub_records = True
            o, failed = run_once(a)
            parity_failed = parity_failed or failed
            r = o["roofline"]
            others.append({"workload": o["config"]["workload"], "layout": o["config"]["layout"], "dtype": o["dtype"],
                           "kv_bytes_per_step": o["config"]["kv_bytes_per_step"], "steps": o["steps"],
                           "us_per_step": o["us_per_step"], "us_per_step_median": o["us_per_step_distribution"]["median"],
                           "GBps": o["value"], "pct_of_hbm_peak": o["pct_of_hbm_peak"],
                           "kernel": r["kernel"], "kernel_mean_us": r["mean_us"], "roofline_frac": r["frac"],
                           "traffic": r["traffic"], "parity": o.get("parity")})
        out["other_workloads"] = others
    print(json.dumps(out))
    if parity_failed:
        sys.exit("bench.py: the GPU result is beyond the tolerance against the fp64 oracle (see \"parity\")")


def run_once(args):
    """One measurement as the arguments describe it: returns the JSON record and whether its parity check failed."""
    two_proc = None
    if args.mode == "two_processes":
        # the users' processes are started before this process touches the GPU; each initialises the GPU itself
        import subprocess
        import tempfile
        assert 1 <= args.user_procs <= 8 and not (args.graph or args.append or args.decode_loop or args.public_cus), \
            "two_processes wants 1..8 users' processes and none of --graph / --append / --decode-loop / --public-cus"
        shm_dir = "/dev/shm" if os.path.isdir("/dev/shm") else None
        fd, shm_path = tempfile.mkstemp(prefix="spd_bench_", dir=shm_dir)
        os.write(fd, bytes(64 * 8))
        os.close(fd)
        passed = ["--config", str(args.config), "--page-tokens", str(args.page_tokens)]
        for flag, val in (("--layout", args.layout), ("--shape", args.shape), ("--dtype", args.dtype),
                          ("--users", args.users), ("--lens", args.lens)):
            if val is not None:
                passed += [flag, str(val)]
        procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--worker", f"{i}/{args.user_procs}",
                                   "--shm", shm_path, *passed], stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)
                 for i in range(args.user_procs)]
        two_proc = {"shm_path": shm_path, "procs": procs}

    import numpy as np
    import torch
    import paper_2409_19134_amd as spd
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    shape = tuple(int(x) for x in args.shape.split(",")) if args.shape else None
    assert shape is None or len(shape) == 3, "--shape wants Hq,Hkv,d"
    dtype = {None: None, "bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[args.dtype]
    len_ranges = tuple(int(x) for x in args.lens.split(",")) if args.lens else None
    assert len_ranges is None or len(len_ranges) == 4, "--lens wants four integers"
    variant = (shape is not None or dtype is not None or args.users is not None or args.page_tokens != 16
               or len_ranges is not None or args.decode_loop > 0)
    wl = workloads.make_workload(args.config, dev, layout=args.layout, shape=shape, dtype=dtype, n_users=args.users,
                                 page_tokens=args.page_tokens, len_ranges=len_ranges,
                                 min_public_len=args.decode_loop)   # the loop grows every public cache up to its drawn length
    kv_bytes = wl.kv_bytes
    elt = 4 if wl.dtype == torch.float32 else 2
    per_token = 2 * wl.n_kv_heads * wl.head_dim * elt
    priv_bytes = wl.private.n_tokens * per_token
    pub_bytes = wl.public.n_tokens * per_token

    copies = args.copies or int(min(8, max(1, -(-1_200_000_000 // max(1, kv_bytes)))))
    ctx = spd.Context(0)
    steps_objs = []
    for i in range(copies):
        w = wl if i == 0 else None
        if w is None:
            import copy
            w = copy.copy(wl)
            w.private, w.public = clone_side(wl.private), clone_side(wl.public)
        steps_objs.append(spd.DecodeStep.from_workload(ctx, w, device_pointer_tables=args.pointer_tables))
        steps_objs[-1].workload = w
    q = wl.q

    if two_proc is not None:
        # q, A_in and lse_in live in allocations of their own that the users' processes map; every KV copy's step
        # writes the same A_in / lse_in (steps run one after the other)
        from paper_2409_19134_amd import ipc
        U, Hq, D = wl.n_users, wl.n_q_heads, wl.head_dim
        sq = ipc.SharedBuffer((U, Hq, D), wl.dtype, dev)
        sa = ipc.SharedBuffer((U, Hq, D), torch.float32, dev)
        sl = ipc.SharedBuffer((U, Hq), torch.float32, dev)
        sq.tensor.copy_(wl.q)
        q = sq.tensor
        for so in steps_objs:
            so.a_in, so.lse_in = sa.tensor, sl.tensor
        use_events = args.ipc_sync == "events"
        ev_q = ipc.SharedEvent() if use_events else None
        torch.cuda.synchronize()
        flags = np.memmap(two_proc["shm_path"], dtype=np.int64, mode="r+", shape=(64,))
        hello = json.dumps({"q": sq.handle.hex(), "a_in": sa.handle.hex(), "lse_in": sl.handle.hex(), "copies": copies,
                            "sync": args.ipc_sync, "ev_q": ev_q.handle.hex() if use_events else None})
        ev_done = []
        for p in two_proc["procs"]:
            p.stdin.write(hello + "\n")
            p.stdin.flush()
        for p in two_proc["procs"]:
            line = p.stdout.readline()
            assert line, "a users' process ended before it was ready"
            reply = json.loads(line)
            ev_done.append(ipc.SharedEvent(bytes.fromhex(reply["ev_done"])) if use_events else None)
        two_proc.update(flags=flags, ev_q=ev_q, ev_done=ev_done, step=0, bufs=(sq, sa, sl))

    stream_ptr = torch.cuda.current_stream().cuda_stream
    k_new = v_new = None
    if args.append:
        assert args.mode == "fused" and int(wl.public.lens.min()) >= 1, "--append needs --mode fused and no empty public part"
        gen = torch.Generator(device=dev).manual_seed(1000 * args.config + 10)
        k_new = torch.randn((wl.n_users, wl.n_kv_heads, wl.head_dim), generator=gen, device=dev).to(wl.dtype)
        v_new = torch.randn((wl.n_users, wl.n_kv_heads, wl.head_dim), generator=gen, device=dev).to(wl.dtype)
    for so in steps_objs:
        so.prepare(q, stream_ptr, k_new, v_new)

    loops = None
    if args.decode_loop:
        # per KV copy, N views of the same buffers whose public lengths grow by one token from step to step
        import copy
        N = args.decode_loop
        assert args.mode == "fused" and 1 <= N <= 32 and not args.append and not args.graph, \
            "--decode-loop wants --mode fused, 1 <= N <= 32, and neither --append nor --graph"
        gen = torch.Generator(device=dev).manual_seed(1000 * args.config + 10)
        k_new = torch.randn((wl.n_users, wl.n_kv_heads, wl.head_dim), generator=gen, device=dev).to(wl.dtype)
        v_new = torch.randn((wl.n_users, wl.n_kv_heads, wl.head_dim), generator=gen, device=dev).to(wl.dtype)
        # the buffers and block tables were made for the drawn lengths (all >= N): the loop's N steps end there, so that
        # no step reads or writes past what is allocated, whatever the layout
        first = wl.public.lens.astype(np.int64) - N
        assert int(first.min()) >= 0 and int((first + N).max()) <= int(wl.public.lens.max())
        assert all(int(first[u]) + N <= int(wl.public.lens[u]) for u in range(wl.n_users))
        loops = []
        for so in steps_objs:
            views = []
            for step in range(N):
                w = copy.copy(so.workload)
                w.public = copy.copy(so.workload.public)
                w.public.lens = (first + step + 1).astype(np.int32)
                views.append(spd.DecodeStep.from_workload(ctx, w, device_pointer_tables=args.pointer_tables))
            loops.append(views)
        kv_bytes = int(priv_bytes + (first + (N + 1) / 2).sum() * per_token)    # mean over the loop's steps

    fused = args.mode == "fused"

    side = torch.cuda.Stream() if args.mode == "streams" else None     # default priority
    if args.public_cus:
        # the owners on disjoint sets of compute units: the nearest a single process comes to the paper's separate
        # processes sharing a GPU (section 5)
        n_cus = torch.cuda.get_device_properties(0).multi_processor_count
        assert args.mode == "streams" and 0 < args.public_cus < n_cus, "--public-cus wants --mode streams and 0 < N < the GPU's units"
        side = masked_stream(torch, n_cus, lambda cu: cu < args.public_cus)
        torch.cuda.set_stream(masked_stream(torch, n_cus, lambda cu: cu >= args.public_cus))

    per_user = None
    if args.mode == "per_user_streams":
        U = wl.n_users
        assert not wl.private.paged and U <= 32, "per_user_streams wants a contiguous workload of at most 32 users"
        user_ctx = [spd.Context(0) for _ in range(U)]           # calls that overlap in time need a context each
        user_stream = [torch.cuda.Stream() for _ in range(U)]   # default priority
        per_user = []
        for so in steps_objs:
            side = so.workload.private
            per_user.append([spd.KVView(side.lens[u:u + 1], side.token_stride, side.head_stride, k=[side.k[u]], v=[side.v[u]],
                                        head_strides=None if side.head_strides is None else side.head_strides[u:u + 1])
                             for u in range(U)])

    def run_per_user(so, views):
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)
        for u, view in enumerate(views):
            st = user_stream[u]
            st.wait_event(fork)
            user_ctx[u].spd_partial_attn_private(so.shape, q[u:u + 1], view, so.a_in[u:u + 1], so.lse_in[u:u + 1], st)
            done = torch.cuda.Event()
            done.record(st)
            main.wait_event(done)
        so.ctx.spd_public_attn_merge(so.shape, q, so.public, so.a_in, so.lse_in, so.a_out, so.lse_out, so.y, so.lse,
                                     so.w_in, main)

    def run_two_processes(so):
        """One step with the users' processes: they are told to enqueue their private calls, this process runs the
        public partial beside them, waits (on the GPU) for their partials and merges (section 4, step 3b / 3c)."""
        main = torch.cuda.current_stream()
        tp = two_proc
        tp["step"] += 1
        k = tp["step"]
        if tp["ev_q"] is not None:
            tp["ev_q"].record(main)        # behind the previous step's merge, which reads A_in
        else:
            main.synchronize()
        tp["flags"][FLAG_GO] = k
        so.ctx.spd_partial_attn_public_batched(so.shape, q, so.public, so.a_out, so.lse_out, main)
        for i, ev in enumerate(tp["ev_done"]):
            if not spin_until(tp["flags"], FLAG_DONE0 + 2 * i, k, proc=tp["procs"][i]):
                raise RuntimeError(f"users' process {i} did not answer step {k}"
                                   + (f" (it ended with status {tp['procs'][i].poll()})"
                                      if tp["procs"][i].poll() is not None else ""))
            if ev is not None:
                ev.wait(main)
        so.ctx.spd_lse_merge(so.a_in, so.lse_in, so.a_out, so.lse_out, so.y, so.lse, so.w_in, main)

    def run(n, start=0):
        for i in range(n):
            if two_proc is not None:
                run_two_processes(steps_objs[(start + i) % copies])
                continue
            if per_user is not None:
                run_per_user(steps_objs[(start + i) % copies], per_user[(start + i) % copies])
                continue
            if loops is not None:
                N = args.decode_loop
                loops[((start + i) // N) % copies][(start + i) % N].run_fused(q, k_new=k_new, v_new=v_new)
                continue
            so = steps_objs[(start + i) % copies]
            if fused:
                so.run_prepared_fused()
            elif side is not None:
                so.run_streams(q, side)
            elif args.mode == "two_parties":
                so.run_two_parties(q)
            else:
                so.run_prepared(public_first=args.mode == "calls_public_first")

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # the first call on a KV set builds its split schedule on the host and uploads it (both owners) and grows the
    # scratch memory; timed on its own, on the host side: the schedule is valid for every layer of a decode step
    torch.cuda.synchronize()
    t_first = time.perf_counter()
    run(1)
    host_first_call_us = (time.perf_counter() - t_first) * 1e6
    torch.cuda.synchronize()
    # warm-up: builds and uploads every copy's schedule
    run(max(args.warmup, copies), start=1)
    torch.cuda.synchronize()
    # host time to enqueue one step once everything is cached (no synchronisation inside)
    n_enq = min(32, max(1, args.steps))
    t_enq = time.perf_counter()
    run(n_enq)
    host_enqueue_us = (time.perf_counter() - t_enq) * 1e6 / n_enq
    torch.cuda.synchronize()
    builds, hits = ctx.spd_get_schedule_stats()

    run_eager = run
    if args.graph:
        # every schedule exists by now, so the calls only launch kernels and can be captured
        assert (fused or per_user is not None) and not args.append and args.steps % copies == 0, \
            "--graph wants --mode fused or per_user_streams, and --steps a multiple of the copies"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            for i, so in enumerate(steps_objs):
                if per_user is not None:
                    run_per_user(so, per_user[i])       # the users' streams fork from and rejoin the captured stream
                else:
                    so.run_fused(q)

        def run(n, start=0):
            for _ in range(n // copies):
                graph.replay()
        run(copies)
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps between two synchronisations ----
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- distribution of the step time: the same steps in short chunks between event pairs on the launch stream ----
    chunk = max(1, min(10, K // 10))
    n_chunks = max(1, K // chunk)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_chunks)]
    torch.cuda.synchronize()
    for c, (e0, e1) in enumerate(ev):
        e0.record()
        run(chunk, start=c * chunk)
        e1.record()
    torch.cuda.synchronize()
    chunk_us = np.asarray([e0.elapsed_time(e1) * 1e3 / chunk for e0, e1 in ev], dtype=np.float64)
    step_dist = {"median": round(float(np.median(chunk_us)), 2), "p10": round(float(np.percentile(chunk_us, 10)), 2),
                 "p90": round(float(np.percentile(chunk_us, 90)), 2), "samples": n_chunks, "steps_per_sample": chunk,
                 "clock": "HIP events on the launch stream around each sample"}

    # ---- the same workload through the calls the paper's deployment makes (same K, same clock as `value`) ----
    sub_records = {}
    plain_default = (fused and not args.graph and not args.append and not args.decode_loop and not args.public_cus
                     and per_user is None)
    if plain_default and not args.no_sub_records:
        def timed(fn):
            fn(max(args.warmup, copies))
            torch.cuda.synchronize()
            a = time.perf_counter()
            fn(K)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - a) * 1e3 / K
            return {"us_per_step": round(ms * 1e3, 2), "GBps": round(kv_bytes / (ms * 1e-3) / 1e9, 1),
                    "pct_of_hbm_peak": round(100.0 * kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)}

        def three_calls(n, start=0):
            for i in range(n):
                steps_objs[(start + i) % copies].run_prepared()

        def two_parties(n, start=0):
            for i in range(n):
                steps_objs[(start + i) % copies].run_prepared_two_parties()
        sub_records["three_calls"] = dict(timed(three_calls), calls="spd_partial_attn_private, "
                                          "spd_partial_attn_public_batched, spd_lse_merge")
        sub_records["two_parties"] = dict(timed(two_parties), calls="spd_partial_attn_private (users), "
                                          "spd_public_attn_merge (service)")

    # ---- the same K steps again with HIP events around the partial kernels (on the launch stream) ----
    ctx.spd_set_kernel_timing(K)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    if per_user is None:
        run_eager(K)      # the events ride on the dispatches themselves, which a graph replay does not make anew
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    kernel_name = ctx.spd_last_kernel_name()
    def stats(samples):
        a = np.asarray(samples, dtype=np.float64)
        return (len(a), float(a.mean()), float(a.min()), [float(np.percentile(a, p)) for p in (10, 50, 90)]) if len(a) \
            else (0, 0.0, 0.0, [0.0, 0.0, 0.0])
    n_priv, priv_mean_us, priv_min_us, priv_pct = stats(ctx.spd_get_kernel_timing_samples(0))
    pub_samples = ctx.spd_get_kernel_timing_samples(1)
    n_pub, pub_mean_us, pub_min_us, _ = stats(pub_samples)
    ctx.spd_set_kernel_timing(0)
    ms_per_step_timed = (t3 - t2) * 1e3 / K
    # fused mode: one launch streams both owners' caches; calls mode: the private call's kernel is the dominant one
    launch_bytes = kv_bytes if fused else priv_bytes
    if two_proc is not None:    # the private kernel runs in the users' processes: this process can time its own only
        n_priv, priv_mean_us, priv_min_us, priv_pct = stats(pub_samples)
        launch_bytes = pub_bytes
    achieved = launch_bytes / (priv_mean_us * 1e-6) / 1e9 if n_priv else 0.0

    out = {
        "metric": "kv_read_hbm_GBps_per_spd_decode_step",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "us_per_step_distribution": step_dist,
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}[wl.dtype],
        "data": "synthetic",
        "host": {"first_call_us_incl_schedule_build_and_upload": round(host_first_call_us, 1),
                 "enqueue_us_per_step_cached": round(host_enqueue_us, 2),
                 "schedule_builds": builds, "schedule_cache_hits": hits},
        "config": {"workload": f"config{args.config}:{wl.name}", "n_users": wl.n_users, "n_q_heads": wl.n_q_heads,
                   "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "private_tokens": wl.private.n_tokens, "public_tokens": wl.public.n_tokens,
                   "kv_bytes_per_step": kv_bytes, "kv_copies_cycled": copies, "mode": args.mode, "public_cus": args.public_cus or None, "hip_graph": bool(args.graph), "decode_loop_steps": args.decode_loop or None, "kv_append": bool(args.append),
                   "layout": f"paged{wl.private.page_tokens}" if wl.private.paged else wl.private.layout,
                   "device_pointer_tables": bool(args.pointer_tables and not wl.private.paged),
                   "seeds": wl.seeds},
        "roofline": {"bound": "hbm",
                     "kernel": kernel_name + (" (both owners, spd_decode_step)" if fused else
                                              " (public call; the private kernel runs in the users' processes)"
                                              if two_proc is not None else " (private call)"),
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None, "traffic_source": None,
                     "bytes_per_launch": launch_bytes, "launches_timed": n_priv,
                     "mean_us": round(priv_mean_us, 2), "min_us": round(priv_min_us, 2),
                     "p10_p50_p90_us": [round(v, 2) for v in priv_pct],
                     "public_kernel": ({"bytes_per_launch": pub_bytes, "mean_us": round(pub_mean_us, 2),
                                        "GBps": round(pub_bytes / (pub_mean_us * 1e-6) / 1e9, 1)} if n_pub else None),
                     "us_per_step_while_timed": round(ms_per_step_timed * 1e3, 2)},
    }

    if fused and not variant:
        out["roofline"]["traffic"], out["roofline"]["traffic_source"] = measured_traffic(args.config, kernel_name)
    out.update(sub_records)

    parity_failed = False
    if not args.no_cpu_baseline and not args.decode_loop:   # (the loop's caches differ from step to step)
        # The cpu_baseline leg: the oracle as it stands, on the host cores of this machine, on a bounded sample of the same
        # workload.  Its output doubles as the parity check of the GPU result (--no-check skips the comparison).
        from oracle import spd_oracle as orc
        hw = orc.from_workload(wl)
        full = args.config in (1, 2) and not variant
        if full:
            rows, sample_desc = None, "whole workload, all rows"
            sample_bytes = kv_bytes
        else:   # big workloads: one query head of every (user, KV head) stream, the head rotating with the user
            G = wl.n_q_heads // wl.n_kv_heads
            rows = [(u, kvh * G + (u + kvh) % G) for u in range(wl.n_users) for kvh in range(wl.n_kv_heads)]
            # a row's share of the algorithmic bytes: its (user, kv head) K/V stream divided among the G query
            # heads that share it (the whole job is U*Hq rows and reads every stream once)
            toks = sum(int(wl.private.lens[u]) + int(wl.public.lens[u]) for u, _ in rows)
            sample_bytes = toks * 2 * wl.head_dim * elt // G
            sample_desc = (f"{len(rows)} (user, head) rows: one query head of every (user, KV head) stream; "
                           "bytes = their share of the K/V streams")
        times = []
        t_begin = time.perf_counter()
        while len(times) < (5 if full else 1) or (time.perf_counter() - t_begin) < args.cpu_seconds:
            a = time.perf_counter()
            Y, _ = orc.attention(hw, rows=rows)
            times.append(time.perf_counter() - a)
        med = float(np.median(times))
        cpu_model = None
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), None)
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(sample_bytes / med / 1e9, 4), "unit": "GB/s", "cores": orc.threads(),
                               "kind": "oracle", "sample": f"{sample_desc}; median of {len(times)} passes",
                               "seconds_per_pass": round(med, 4), "cpu_model": cpu_model}
        if not args.no_check:
            y = steps_objs[0].y.cpu().double().numpy().reshape(wl.n_users * wl.n_q_heads, -1)
            if rows is not None:
                y = y[[u * wl.n_q_heads + h for u, h in rows]]
            err = float(np.abs(y - Y).max())
            tol = {torch.float32: 1e-5, torch.bfloat16: 2e-3, torch.float16: 1e-4}[wl.dtype]
            out["parity"] = {"max_abs_err_vs_fp64_oracle": err, "tolerance": tol, "ok": bool(err <= tol),
                             "rows_checked": "all" if rows is None else len(rows)}
            parity_failed = not err <= tol
    if two_proc is not None:
        out["config"]["user_processes"] = args.user_procs
        out["config"]["ipc_sync"] = args.ipc_sync
        torch.cuda.synchronize()
        two_proc["flags"][FLAG_STOP] = 1
        for p in two_proc["procs"]:
            try:
                p.wait(timeout=60)
            except Exception:
                p.kill()
        del two_proc["flags"]
        os.unlink(two_proc["shm_path"])
    ctx.close()
    return out, parity_failed


if __name__ == "__main__":
    main()
