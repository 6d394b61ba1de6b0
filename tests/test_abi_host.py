"""Host-only checks of the C ABI: exported symbols, argument validation, the split schedule.  No GPU needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2409_19134_amd as spd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "spd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(spd_[a-z_]+)\s*\(", header))
    assert declared == set(spd.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(spd.lib, name), name


def test_abi_version_of_header_binding_and_library_agree():
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "spd.h")).read()
    in_header = int(re.search(r"#define SPD_ABI_VERSION (\d+)", header).group(1))
    from paper_2409_19134_amd import binding
    assert in_header == binding.SPD_ABI_VERSION == spd.lib.spd_abi_version()


def test_strerror_is_distinct_per_code():
    msgs = {spd.spd_strerror(c) for c in range(0, -8, -1)}
    assert len(msgs) == 8 and spd.spd_strerror(-99) == "unknown error code"


def _view(lens, token_stride=1024, head_stride=128, k=None, v=None, block_size=0, **kw):
    lens = np.asarray(lens, dtype=np.int32)
    n = len(lens)
    st = spd.spd_kv_view()
    st.n_users = n
    st.lens = lens.ctypes.data_as(C.POINTER(C.c_int32))
    st.token_stride, st.head_stride, st.block_size = token_stride, head_stride, block_size
    kp = (C.c_void_p * max(1, n))(*(k if k is not None else [0x10000] * n))
    vp = (C.c_void_p * max(1, n))(*(v if v is not None else [0x20000] * n))
    st.k_ptrs = C.cast(kp, C.POINTER(C.c_void_p))
    st.v_ptrs = C.cast(vp, C.POINTER(C.c_void_p))
    for key, val in kw.items():
        setattr(st, key, val)
    st._keep = (lens, kp, vp)
    return st


Q, OUT, LSE = 0x1000, 0x2000, 0x3000   # fake device addresses: validation never dereferences them


def _check(shape, view, q=Q, out=OUT, lse=LSE):
    return spd.spd_validate_partial(shape, q, view, out, lse)


def test_validation_accepts_good_arguments():
    sh = spd.make_shape(spd.SPD_BF16, 32, 8, 128, 0.0884)
    assert _check(sh, _view([5, 0, 9])) == spd.SPD_OK
    assert _check(sh, _view([0, 0], k=[0, 0], v=[0, 0])) == spd.SPD_OK          # empty users may have NULL buffers
    assert _check(sh, _view([])) == spd.SPD_OK
    paged = _view([40, 1], token_stride=128, head_stride=2048, block_size=16, k_pool=0x100000, v_pool=0x200000,
                  block_table=0x300000, max_blocks=3, block_stride=16384)
    assert _check(sh, paged) == spd.SPD_OK
    assert _check(spd.make_shape(spd.SPD_F32, 8, 8, 64, 0.125), _view([128], token_stride=512, head_stride=64)) == spd.SPD_OK
    assert _check(spd.make_shape(spd.SPD_F32, 6, 2, 128, 0.1), _view([128])) == spd.SPD_OK          # group of 3 heads
    assert _check(spd.make_shape(spd.SPD_BF16, 128, 8, 64, 0.125), _view([128], token_stride=512, head_stride=64)) == spd.SPD_OK
    assert _check(spd.make_shape(spd.SPD_F16, 128, 8, 128, 0.1), _view([128])) == spd.SPD_OK


@pytest.mark.parametrize("args,code", [
    (dict(dtype=7), spd.SPD_ERR_SHAPE),
    (dict(Hq=30), spd.SPD_ERR_SHAPE),                   # Hq % Hkv != 0
    (dict(d=96), spd.SPD_ERR_SHAPE),
    (dict(Hq=256, Hkv=8), spd.SPD_ERR_SHAPE),           # group of 32 heads
    (dict(Hq=136, Hkv=8, dtype=spd.SPD_F32), spd.SPD_ERR_SHAPE),  # group of 17 heads
    (dict(scale=float("nan")), spd.SPD_ERR_SHAPE),
])
def test_validation_rejects_bad_shapes(args, code):
    a = dict(dtype=spd.SPD_BF16, Hq=32, Hkv=8, d=128, scale=0.1)
    a.update(args)
    sh = spd.make_shape(a["dtype"], a["Hq"], a["Hkv"], a["d"], a["scale"])
    assert _check(sh, _view([5])) == code


def test_validation_rejects_bad_views_and_pointers():
    sh = spd.make_shape(spd.SPD_BF16, 32, 8, 128, 0.1)
    assert _check(sh, _view([5, -1])) == spd.SPD_ERR_LEN
    assert _check(sh, _view([5]), q=0) == spd.SPD_ERR_NULL
    assert _check(sh, _view([5]), out=0) == spd.SPD_ERR_NULL
    assert _check(sh, _view([5]), lse=0) == spd.SPD_ERR_NULL
    assert _check(sh, _view([5]), q=Q + 2) == spd.SPD_ERR_ALIGN
    assert _check(sh, _view([5], k=[0])) == spd.SPD_ERR_NULL
    assert _check(sh, _view([5], v=[0x20008])) == spd.SPD_ERR_ALIGN
    assert _check(sh, _view([5], token_stride=1028)) == spd.SPD_ERR_ALIGN       # rows no longer 16-byte aligned
    assert _check(sh, _view([5], token_stride=64)) == spd.SPD_ERR_ALIGN         # rows would overlap
    assert _check(sh, _view([5], head_stride=100)) == spd.SPD_ERR_ALIGN
    hs = (C.c_int64 * 2)(640, 100)
    assert _check(sh, _view([5, 9], token_stride=128, head_stride=0, head_strides=hs)) == spd.SPD_ERR_ALIGN
    hs = (C.c_int64 * 2)(640, 1152)
    assert _check(sh, _view([5, 9], token_stride=128, head_stride=0, head_strides=hs)) == spd.SPD_OK
    assert _check(sh, _view([5], block_size=24)) == spd.SPD_ERR_SHAPE           # pages hold 16, 32, 64, 128 or 256 tokens
    assert _check(sh, _view([5], block_size=8)) == spd.SPD_ERR_SHAPE
    assert _check(sh, _view([5], block_size=512)) == spd.SPD_ERR_SHAPE
    paged = dict(token_stride=128, head_stride=2048, block_size=16, k_pool=0x100000, v_pool=0x200000,
                 block_table=0x300000, max_blocks=3, block_stride=16384)
    assert _check(sh, _view([49], **paged)) == spd.SPD_ERR_LEN                   # needs 4 pages, table has 3
    assert _check(sh, _view([48], **dict(paged, block_table=0))) == spd.SPD_ERR_NULL
    assert _check(sh, _view([48], **dict(paged, block_stride=0))) == spd.SPD_ERR_ALIGN
    null_shape = C.POINTER(spd.spd_shape)()
    assert spd.lib.spd_validate_partial(null_shape, Q, C.byref(_view([5])), OUT, LSE) == spd.SPD_ERR_NULL


def test_lengths_beyond_two_to_the_thirty_are_rejected():
    sh = spd.make_shape(spd.SPD_BF16, 32, 8, 128, 0.1)
    assert _check(sh, _view([1 << 30])) == spd.SPD_OK
    assert _check(sh, _view([5, (1 << 30) + 1])) == spd.SPD_ERR_LEN
    assert _check(sh, _view([2 ** 31 - 1])) == spd.SPD_ERR_LEN
    with pytest.raises(spd.SpdError) as ei:
        spd.spd_build_schedule(sh, [2 ** 31 - 1], 256)
    assert ei.value.code == spd.SPD_ERR_LEN
    items, chunk = spd.spd_build_schedule(sh, [1 << 30], 256)       # the largest length still gets a schedule
    assert sum(it["t_end"] - it["t_begin"] for it in items) == 8 * (1 << 30)


def test_calls_reject_null_context_without_touching_the_gpu():
    sh = spd.make_shape(spd.SPD_BF16, 32, 8, 128, 0.1)
    v = _view([5])
    assert spd.lib.spd_partial_attn_private(None, C.byref(sh), Q, C.byref(v), OUT, LSE, None) == spd.SPD_ERR_NULL
    assert spd.lib.spd_partial_attn_public_batched(None, C.byref(sh), Q, C.byref(v), OUT, LSE, None) == spd.SPD_ERR_NULL
    assert spd.lib.spd_lse_merge(None, 4, 128, Q, Q, Q, Q, Q, None, None, None) == spd.SPD_ERR_NULL
    assert spd.lib.spd_destroy(None) == spd.SPD_ERR_NULL


@pytest.mark.parametrize("lens", [
    [0], [1], [31, 32, 33], [128, 129, 4096, 0, 513], [70000, 3, 40000], list(range(0, 700, 37)),
    [131072, 5, 40000], [2304] * 16, [100000] * 64,
])
@pytest.mark.parametrize("n_cus", [1, 256])
@pytest.mark.parametrize("plain", [True, False])
def test_schedule_covers_every_token_once(lens, n_cus, plain, monkeypatch):
    """plain: equal pieces (the options that make pieces unequal on purpose switched off); else the default options."""
    Hkv = 8
    seg_cost, skew = (0, 0) if plain else (2, 12)
    if plain:                                            # the host-only helper reads the SPD_* variables at every call
        monkeypatch.setenv("SPD_SEG_COST", "0")
        monkeypatch.setenv("SPD_HALF_SKEW", "0")
    sh = spd.make_shape(spd.SPD_BF16, 32, Hkv, 128, 0.1)
    items, chunk = spd.spd_build_schedule(sh, lens, n_cus)
    assert chunk % 32 == 0
    seen = {}
    slots = set()
    for it in items:
        assert 0 <= it["t_begin"] < it["t_end"] <= lens[it["user"]]
        assert it["t_begin"] % 32 == 0
        assert it["t_end"] % 32 == 0 or it["t_end"] == lens[it["user"]]
        seen.setdefault((it["user"], it["kv_head"]), []).append(it)
        assert it["slot"] not in slots
        slots.add(it["slot"])
    for u, L in enumerate(lens):
        for h in range(Hkv):
            row = sorted(seen.get((u, h), []), key=lambda x: x["t_begin"])
            if L == 0:
                assert not row
                continue
            assert row[0]["t_begin"] == 0 and row[-1]["t_end"] == L
            for a, b in zip(row, row[1:]):
                assert a["t_end"] == b["t_begin"]
            assert all(it["n_chunks"] == len(row) for it in row)
            assert [it["chunk"] for it in row] == list(range(len(row)))
            assert [it["slot"] for it in row] == list(range(row[0]["slot"], row[0]["slot"] + len(row)))
    # pieces: consecutive, equal to within one 32-token step, and no more than fit the machine at once
    # unless each already carries the maximum piece length
    pieces = [it["piece"] for it in items]
    assert pieces == sorted(pieces)
    if items:
        steps = {}
        for it in items:
            steps[it["piece"]] = steps.get(it["piece"], 0) + -(-(it["t_end"] - it["t_begin"]) // 32)
        assert sorted(steps) == list(range(len(steps)))
        short_chunks = sum(-(-(-(-L // 32)) // 4) for L in lens)
        if max(lens) <= 768 and short_chunks * Hkv <= 2 * n_cus:      # short rows that fit the machine at once:
            # chunks of 128 tokens, one per piece
            assert all(it["t_end"] - it["t_begin"] <= 128 for it in items)
            assert len(steps) == len(items)
            return
        sizes = [steps[i] for i in range(len(steps))]
        assert max(sizes) * 32 <= max(chunk, 128)
        resident = max(8, 2 * n_cus // 8 * 8)
        if plain:
            assert max(sizes) * 32 <= 16384
            assert max(sizes) - min(sizes) <= 1                    # equal pieces
        else:
            # a piece gives up seg_cost steps for every further row it reaches into (a cut that would land inside
            # that allowance moves to the row boundary, so a piece may come out up to seg_cost steps short or long)
            segs = {}
            for it in items:
                segs[it["piece"]] = segs.get(it["piece"], 0) + 1
            n_groups = len(sizes) // Hkv
            total_steps = sum(-(-L // 32) for L in lens)
            if total_steps > 64 * n_groups:                        # long pieces stay equal
                seg_cost = 0
            cost = [steps[i] + seg_cost * (segs[i] - 1) for i in range(len(steps))]
            halves = [cost]
            if len(sizes) == resident and n_groups >= 2 and 8 * n_groups <= total_steps <= 64 * n_groups:   # one resident round of short pieces: unequal halves
                h = n_groups // 2 * Hkv
                halves = [cost[:h], cost[h:]]
                m0, m1 = sum(halves[0]) / len(halves[0]), sum(halves[1]) / len(halves[1])
                assert abs(m0 / m1 - (100 + skew) / (100 - skew)) <= 0.12, (m0, m1)
            for part in halves:
                assert max(part) - min(part) <= 2 * seg_cost + 2, (min(part), max(part))
        if len(sizes) > resident:                              # several resident waves: a whole number of them
            assert len(sizes) % resident == 0


def test_schedule_fills_the_machine_for_the_headline_workload():
    import workloads
    lp, lo = workloads.draw_lengths(2, 16)
    sh = spd.make_shape(spd.SPD_BF16, 32, 8, 128, 0.1)
    items, chunk = spd.spd_build_schedule(sh, lp, 256)
    assert len({it["piece"] for it in items}) == 512      # the 2 workgroups per CU that are resident at once


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU only: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr


def test_bench_traffic_figure_names_its_source_and_its_kernel():
    """roofline.traffic is a stored measurement: the benchmark hands it out only for the kernel instance the stored
    summary was made with, and says which file it read."""
    import importlib.util
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    algorithmic = {2: 157405184, 3: 5299486720, 4: 2810568704, 5: 11444723712}   # 4096 B x the workload's tokens
    for config, want in algorithmic.items():
        rel = os.path.join("profiles", f"partial_kernel_config{config}_pmc_traffic.txt")
        names = set(re.findall(r"spd::(partial_mfma_kernel<[^>]*>)", open(os.path.join(root, rel)).read()))
        assert len(names) == 1, names
        name = names.pop()
        got, src = bench.measured_traffic(config, name)
        assert src["file"] == rel and src["kernel_that_ran"] == name and src["kernel_in_summary"] == [name]
        assert want <= got <= 1.05 * want, (config, got)          # every byte read once, little else
        other = name.replace("<1,", "<2,")
        got, src = bench.measured_traffic(config, other)
        assert got is None and "another kernel instance" in src["why_null"]
    got, src = bench.measured_traffic(1, "partial_mfma_kernel<0, 64, false, false, false, false>")
    assert got is None and "no summary" in src["why_null"]


def test_bench_handshake_wait_ends_when_the_other_process_has_ended():
    """The two-process benchmark's host handshake: a wait on a counter gives up as soon as the process that should
    raise it is gone (and not only at its time limit), and sees a counter that is already there."""
    import importlib.util
    import subprocess
    import sys
    import time
    import numpy as np
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    flags = np.zeros(64, dtype=np.int64)
    gone = subprocess.Popen([sys.executable, "-c", "pass"])
    gone.wait()
    t0 = time.perf_counter()
    assert bench.spin_until(flags, bench.FLAG_DONE0, 1, proc=gone) is False
    assert time.perf_counter() - t0 < 10.0 < bench.SPIN_LIMIT_S
    flags[bench.FLAG_DONE0] = 1
    assert bench.spin_until(flags, bench.FLAG_DONE0, 1, proc=gone) is True
    flags[bench.FLAG_STOP] = 1
    assert bench.spin_until(flags, bench.FLAG_GO, 5, also_stop=True) is True      # the stop flag ends a worker's wait


def test_product_package_does_not_reach_the_oracle():
    """The oracle is test infrastructure: nothing under the package imports or loads it."""
    pkg = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2409_19134_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "build.py", f"{f} mentions the oracle"


def test_device_pointer_tables_come_in_pairs_and_aligned():
    sh = spd.make_shape(spd.SPD_BF16, 8, 8, 128, 0.1)
    lens = np.asarray([5], dtype=np.int32)
    kp = (C.c_void_p * 1)(0x1000)
    st = spd.spd_kv_view()
    st.n_users, st.lens = 1, lens.ctypes.data_as(C.POINTER(C.c_int32))
    st.k_ptrs = C.cast(kp, C.POINTER(C.c_void_p))
    st.v_ptrs = C.cast(kp, C.POINTER(C.c_void_p))
    st.token_stride, st.head_stride = 1024, 128
    q = C.c_void_p(0x2000)
    out = C.c_void_p(0x3000)
    args = (C.byref(sh), q, C.byref(st), out, out)
    assert spd.lib.spd_validate_partial(*args) == spd.SPD_OK
    st.k_ptrs_dev = 0x4000
    assert spd.lib.spd_validate_partial(*args) == spd.SPD_ERR_NULL        # one table without the other
    st.v_ptrs_dev = 0x5004
    assert spd.lib.spd_validate_partial(*args) == spd.SPD_ERR_ALIGN       # pointers are 8 bytes
    st.v_ptrs_dev = 0x5008
    assert spd.lib.spd_validate_partial(*args) == spd.SPD_OK


def test_header_is_c99_and_library_links_from_c(tmp_path):
    """include/spd.h compiled by a C99 compiler with warnings as errors; the program links the library and calls the
    host-only entry points."""
    import subprocess
    lib_dir = os.path.join(ROOT, "paper_2409_19134_amd")
    exe = str(tmp_path / "abi_c99")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "host", "abi_c99.c"), "-o", exe,
                           "-L", lib_dir, "-l:libspd_hip.so", "-Wl,-rpath," + lib_dir])
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    assert "c99 ok" in res.stdout


@pytest.mark.parametrize("hpw,Hkv,w", [(1, 8, 8), (4, 8, 4), (2, 8, 2), (1, 12, 6), (4, 12, 4), (5, 12, 4), (8, 32, 8), (3, 9, 3)])
def test_head_per_wave_schedule_in_head_groups(hpw, Hkv, w):
    """Head-per-wave schedules: an item stands for w consecutive KV heads (w = the largest divisor of the KV head count
    up to the group size asked for); every token of every head is covered once and every head of every chunk has a
    partial slot of its own."""
    lens = [5000, 0, 33, 70000, 129]
    sh = spd.make_shape(spd.SPD_BF16, Hkv * 2, Hkv, 128, 0.1)
    items, _ = spd.spd_build_schedule(sh, lens, 256, head_per_wave=hpw)
    slots = set()
    cover = {}
    for it in items:
        assert it["kv_head"] % w == 0 and it["kv_head"] + w <= Hkv
        for j in range(w):
            slot = it["slot"] + j * it["n_chunks"]
            assert slot not in slots
            slots.add(slot)
            cover.setdefault((it["user"], it["kv_head"] + j), []).append((it["t_begin"], it["t_end"]))
    for u, L in enumerate(lens):
        for h in range(Hkv):
            row = sorted(cover.get((u, h), []))
            if L == 0:
                assert not row
                continue
            assert row[0][0] == 0 and row[-1][1] == L and all(a[1] == b[0] for a, b in zip(row, row[1:]))
    with pytest.raises(spd.SpdError):
        spd.spd_build_schedule(sh, lens, 256, head_per_wave=9)
