"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
function the header declares, and its pure-host entry points (plan construction, argument
validation) behave as documented."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1802_06058_amd import vgc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "vgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vgc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = vgc.load()
    names = _declared()
    assert {"vgc_sqgrad", "vgc_accumulate_select", "vgc_pack", "vgc_unpack_add"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in vgc.h but not exported"
    assert set(names) == set(vgc.EXPORTS), "binding and header disagree"


def _groups(sizes):
    arr = (vgc.Group * len(sizes))()
    off = 0
    for k, s in enumerate(sizes):
        arr[k].offset, arr[k].size, arr[k].reserved = off, s, 0
        off += s
    return arr, off


def test_plan_build_tiles_never_span_groups():
    lib = vgc.load()
    T = lib.vgc_tile_size()
    assert T == 2048
    S = 8192                                   # tiles per scan segment
    sizes = [1, T, T + 1, 5 * T - 3, 10, 2 * S * T + 7, S * T]
    arr, n = _groups(sizes)
    n_tiles = lib.vgc_tile_count(arr, len(sizes), n)
    assert n_tiles == sum((s + T - 1) // T for s in sizes)
    nbytes = lib.vgc_plan_bytes(arr, len(sizes), n)
    buf = np.zeros(nbytes, np.uint8)
    assert lib.vgc_plan_build(arr, len(sizes), n, buf.ctypes.data, nbytes) == 0
    hdr = buf[:64].view("<u8")
    assert hdr[1] == n and hdr[2] == n_tiles
    groups_off, tiles_off = int(buf[32:40].view("<u8")[0]), int(buf[40:48].view("<u8")[0])
    G = buf[groups_off:groups_off + 16 * len(sizes)].view(np.dtype([("offset", "<u8"), ("size", "<u4"), ("first", "<u4")]))
    Tt = buf[tiles_off:tiles_off + 16 * n_tiles].view(
        np.dtype([("group", "<u4"), ("start", "<u4"), ("seg", "<u4"), ("reserved", "<u4")]))
    segs_off, n_segs = int(buf[64:72].view("<u8")[0]), int(buf[72:80].view("<u8")[0])
    assert n_segs == sum(((s + T - 1) // T + S - 1) // S for s in sizes) == len(sizes) + 2
    Sg = buf[segs_off:segs_off + 16 * n_segs].view(
        np.dtype([("group", "<u4"), ("first_tile", "<u4"), ("seg_in_group", "<u4"), ("group_first_seg", "<u4")]))
    covered = np.zeros(n, np.int32)
    for t in range(n_tiles):
        k, start = int(Tt[t]["group"]), int(Tt[t]["start"])
        assert start % T == 0 and start < sizes[k]
        lo = int(G[k]["offset"]) + start
        covered[lo:lo + min(T, sizes[k] - start)] += 1
        if start == 0:
            assert int(G[k]["first"]) == t
        sg = Sg[int(Tt[t]["seg"])]
        in_group = start // T
        assert int(sg["group"]) == k and int(sg["first_tile"]) == in_group // S * S
        assert int(sg["seg_in_group"]) == in_group // S
        assert int(sg["group_first_seg"]) == int(Tt[t]["seg"]) - in_group // S
    assert np.all(covered == 1)
    assert lib.vgc_plan_build(arr, len(sizes), n, buf.ctypes.data, nbytes - 1) == -2
    assert lib.vgc_scratch_bytes(arr, len(sizes), n) >= n_tiles * (32 + T // 8 + 2 * T)
    assert lib.vgc_scratch_bitmap_offset(arr, len(sizes), n) % 256 == 0


def test_group_validation():
    lib = vgc.load()
    arr, n = _groups([10, 20])
    assert lib.vgc_tile_count(arr, 2, n) == 2
    assert lib.vgc_tile_count(arr, 2, n + 1) == 0 and b"cover" in lib.vgc_last_error()
    arr[1].offset = 11
    assert lib.vgc_tile_count(arr, 2, 31) == 0 and b"tile" in lib.vgc_last_error()
    arr, n = _groups([10, 0])
    assert lib.vgc_plan_bytes(arr, 2, 10) == 0 and b"empty" in lib.vgc_last_error()
    big = (vgc.Group * 1)()
    big[0].offset, big[0].size = 0, (1 << 28) + 1
    buf = np.zeros(64, np.uint8)
    assert lib.vgc_plan_build(big, 1, (1 << 28) + 1, buf.ctypes.data, 64) == -3
    big[0].size = 1 << 28
    assert lib.vgc_tile_count(big, 1, 1 << 28) == (1 << 28) // 2048
    assert lib.vgc_tile_count(None, 1, 5) == 0


def test_compute_calls_validate_before_touching_the_gpu():
    """Argument errors are detected on the host: these return without any HIP call."""
    lib = vgc.load()
    arr, n = _groups([100])
    one = C.c_void_p(256)          # non-NULL, aligned, never dereferenced on an argument error
    assert lib.vgc_accumulate_select(None, one, one, one, n, arr, 1, one, 1.0, 0.999, one, None) == -1
    assert lib.vgc_accumulate_select(one, one, one, one, n, arr, 1, one, float("nan"), 0.999, one, None) == -6
    assert lib.vgc_accumulate_select(one, one, one, one, n, arr, 1, one, 1.0, 0.0, one, None) == -6
    assert lib.vgc_accumulate_select(one, one, one, one, n + 1, arr, 1, one, 1.0, 0.999, one, None) == -2
    assert lib.vgc_accumulate_select(C.c_void_p(258), one, one, one, n, arr, 1, one, 1.0, 0.999, one, None) == -5
    assert lib.vgc_pack(n, arr, 1, one, one, None, 10, one, one, None) == -1
    assert lib.vgc_unpack_add(one, 5, one, arr, 1, one, float("inf"), one, n, None) == -6
    assert lib.vgc_sqgrad(2, 0, one, one, 1, 1, 1, 1, 1.0, None, one, None, 0, None) == -4
    assert lib.vgc_sqgrad(0, 0, one, one, 0, 1, 1, 1, 1.0, None, one, None, 0, None) == -2
    assert lib.vgc_sqgrad(0, 0, C.c_void_p(260), one, 1, 1, 1, 1, 1.0, None, one, None, 0, None) == -5


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(vgc, "_lib", None)
    monkeypatch.setattr(vgc, "LIB_PATH", str(tmp_path / "libvgc.so"))
    with pytest.raises(vgc.VgcError):
        vgc.load()


def test_conv2d_and_update_argument_checks_need_no_gpu():
    """Geometry and hyper-parameter validation happens on the host before anything is launched."""
    lib = vgc.load()
    fake = C.c_void_p(0x1000)                                     # never dereferenced: every call below is rejected first
    conv = lambda dtype, Cin, Cc, kh, ph: lib.vgc_sqgrad_conv2d(dtype, fake, fake, 2, 8, 8, Cin, Cc, kh, 3, 1, 1, ph, 1, 1.0,
                                                                 None, fake, None, 0, None)
    # input channels that are not a multiple of 16 bytes: a first layer's kernel takes them while kh kw Cin <= 160, with a workspace
    assert conv(vgc.BF16, 12, 8, 3, 1) == -2 and b"needs the workspace" in lib.vgc_last_error()
    assert conv(vgc.BF16, 12, 8, 5, 1) == -2 and b"multiple of 16 bytes" in lib.vgc_last_error()      # kh kw Cin = 180
    assert conv(vgc.F32, 6, 8, 3, 1) == -2
    assert lib.vgc_sqgrad_conv2d_workspace_bytes(vgc.BF16, 64, 224, 224, 3, 64, 3, 3, 1, 1, 1, 1) == 64 * 32 * 27 * 64 * 4    # 32 parts per sample
    assert conv(vgc.BF16, 8, 8, 3, 3) == -2 and b"pad" in lib.vgc_last_error()
    assert conv(9, 8, 8, 3, 1) == -4
    assert lib.vgc_sqgrad_conv2d(vgc.BF16, None, fake, 2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, None, fake, None, 0, None) == -1
    # the batch call checks every layer before it touches a stream
    ok = vgc.Conv2dLayer(vgc.BF16, 0x1000, 0x1000, 2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, None, 0x1000, None, 0)
    odd = vgc.Conv2dLayer(vgc.BF16, 0x1000, 0x1000, 2, 8, 8, 12, 8, 3, 3, 1, 1, 1, 1, 1.0, None, 0x1000, None, 0)
    arr2 = (vgc.Conv2dLayer * 2)(ok, odd)
    assert lib.vgc_sqgrad_conv2d_batch(C.cast(arr2, C.c_void_p), 2, None) == -2 and b"needs the workspace" in lib.vgc_last_error()
    assert lib.vgc_sqgrad_conv2d_batch(None, 2, None) == -1
    # the workspace query is pure host code: a layer with few tiles and many positions wants room for partial products
    assert lib.vgc_sqgrad_conv2d_workspace_bytes(vgc.BF16, 64, 224, 224, 64, 64, 3, 3, 1, 1, 1, 1) > 0
    assert lib.vgc_sqgrad_conv2d_workspace_bytes(vgc.BF16, 64, 224, 224, 6, 64, 7, 7, 1, 1, 1, 1) == 0     # unsupported shape: 6 channels, 7 x 7

    arr, n = _groups([100, 200])
    opt = vgc.Optimizer(vgc.MOMENTUM_SGD, 0.1, 1.5, 0.9, 0.999, 1e-8, 1)
    call = lambda o, p=0, s2=None: lib.vgc_unpack_apply(None, None, None, p, arr, 2, fake, 1.0, C.byref(o), fake, fake, s2, n, None)
    assert call(opt) == -6 and b"momentum" in lib.vgc_last_error()
    opt.kind, opt.momentum = 5, 0.9
    assert call(opt) == -6
    opt.kind = vgc.ADAM
    assert call(opt) == -1                                         # Adam without its second state array
    opt.step = 0
    assert call(opt, 0, fake) == -6
    opt.kind, opt.step = vgc.MOMENTUM_SGD, 1
    assert call(opt, 65) == -1                                     # message tables missing


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N above 1 exits with a message that says so,
    before anything touches a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_binding_checks_tensor_sizes_before_any_launch():
    """The C ABI sees raw pointers; the binding knows the tensors and refuses outputs, state or scratch that are
    too small or of the wrong type before anything is launched (CPU tensors here: nothing may reach the GPU)."""
    import torch
    from paper_1802_06058_amd import vgc
    vgc.load()
    act = torch.zeros(2, 6, 6, 8)
    D = torch.zeros(2, 6, 6, 16)
    ok = torch.zeros(72, 16)
    with pytest.raises(vgc.VgcError, match="s_out"):
        vgc.sqgrad_conv2d(act, D, 3, 3, (1, 1), (1, 1), 0.5, torch.zeros(71, 16))
    with pytest.raises(vgc.VgcError, match="g_out"):
        vgc.sqgrad_conv2d(act, D, 3, 3, (1, 1), (1, 1), 0.5, ok, torch.zeros(72, 16, dtype=torch.float64))
    with pytest.raises(vgc.VgcError, match="output gradient"):
        vgc.sqgrad_conv2d(act, torch.zeros(2, 5, 6, 16), 3, 3, (1, 1), (1, 1), 0.5, ok)
    with pytest.raises(vgc.VgcError, match="s_out"):
        vgc.sqgrad(vgc.FC, torch.zeros(4, 8), torch.zeros(4, 16), 0.25, torch.zeros(8, 15))
    with pytest.raises(vgc.VgcError, match="belong together"):
        vgc.sqgrad(vgc.CONV, torch.zeros(4, 5, 8), torch.zeros(4, 6, 16), 0.25, torch.zeros(8, 16))
    plan = vgc.Plan([(0, 5000), (5000, 3000)], "cpu")
    f = lambda k: torch.zeros(k)
    scratch = torch.zeros(plan.scratch_bytes, dtype=torch.uint8)
    with pytest.raises(vgc.VgcError, match="r:"):
        vgc.accumulate_select(f(8000), f(8000), f(7999), f(8000), plan, 1.0, 0.999, scratch)
    with pytest.raises(vgc.VgcError, match="scratch"):
        vgc.accumulate_select(f(8000), f(8000), f(8000), f(8000), plan, 1.0, 0.999, scratch[:-1])
    words, hdrs = torch.zeros(100, dtype=torch.int32), plan.new_headers()
    with pytest.raises(vgc.VgcError, match="words"):
        vgc.unpack_add(words, 101, hdrs, plan, 1.0, f(8000))
    with pytest.raises(vgc.VgcError, match="dense"):
        vgc.unpack_add(words, 100, hdrs, plan, 1.0, f(10))
    with pytest.raises(vgc.VgcError, match="headers"):
        vgc.unpack_add_batch([words], [10], [hdrs[:-1]], plan, 1.0, f(8000))
    with pytest.raises(vgc.VgcError, match="state1"):
        vgc.unpack_apply([words], [10], [hdrs], plan, 1.0, f(8000), f(3))


def test_binding_rejects_host_tensors_before_any_launch():
    """The kernels dereference data_ptr() as GPU memory, so the binding must refuse a tensor that lives in
    host memory (a forgotten .to(device)) before anything is launched.  Runs without a GPU: a plan whose
    table stays on the host is enough to reach the checks."""
    import torch
    from paper_1802_06058_amd import vgc
    plan = vgc.Plan([(0, 100), (100, 200)], device="cpu")
    t = torch.zeros(300, dtype=torch.float32)
    sc = torch.zeros(plan.scratch_bytes, dtype=torch.uint8)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.accumulate_select(t, t, t, t, plan, 1.0, 0.999, sc)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.accumulate_select_hybrid(t, t, t, t, plan, 1.0, 0.999, 0.1, sc)
    words = torch.zeros(300, dtype=torch.int32)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.pack(plan, sc, words, plan.new_headers(), plan.new_status())
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.unpack_add(words, 0, plan.new_headers(), plan, 1.0, t)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.unpack_add_batch([words], [0], [plan.new_headers()], plan, 1.0, t)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.unpack_apply([words], [0], [plan.new_headers()], plan, 1.0, t, t)
    X, D, s = torch.zeros(4, 8), torch.zeros(4, 8), torch.zeros(8, 8)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.sqgrad(vgc.FC, X, D, 1.0, s)
    a, d = torch.zeros(2, 8, 8, 8), torch.zeros(2, 8, 8, 8)
    with pytest.raises(vgc.VgcError, match="GPU memory"):
        vgc.sqgrad_conv2d(a, d, 3, 3, (1, 1), (1, 1), 1.0, torch.zeros(72, 8))


def test_noalloc_entry_point_refuses_oversized_shapes_on_the_host():
    """vgc_sqgrad_noalloc works inside a fixed static buffer: a shape whose partial sums would not fit is
    refused with VGC_ERR_SIZE before anything touches a GPU (fake pointers here, never dereferenced)."""
    lib = vgc.load()
    fake = C.c_void_p(0x1000)
    B, P, J, Cc = 8, 49, 9216, 1024
    assert lib.vgc_sqgrad_workspace_bytes(vgc.CONV, vgc.F32, B, P, J, Cc) > vgc.NOALLOC_SCRATCH_BYTES
    assert lib.vgc_sqgrad_noalloc(vgc.CONV, vgc.F32, fake, fake, B, P, J, Cc, 1.0, None, fake, None) == -2
    assert b"static buffer" in lib.vgc_last_error()
    assert lib.vgc_sqgrad_noalloc(vgc.CONV, 9, fake, fake, B, P, J, Cc, 1.0, None, fake, None) == -4
    assert lib.vgc_sqgrad_noalloc(vgc.CONV, vgc.F32, fake, fake, 0, P, J, Cc, 1.0, None, fake, None) == -2


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    """The library's host side (group validation, plan construction, argument checks, dispatch decisions) built
    with AddressSanitizer + UndefinedBehaviorSanitizer and driven by csrc/hostcheck/vgc_hostcheck.cpp: plans for
    group lists at every boundary the builder distinguishes are written into buffers allocated to the byte and
    re-derived, and every entry point is driven into each of its argument errors with fabricated device pointers.
    A finding of either sanitizer aborts the program."""
    import subprocess
    from paper_1802_06058_amd import build
    exe = build.build_hostcheck()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "hostcheck ok" in p.stdout
    assert "AddressSanitizer" not in p.stderr and "runtime error" not in p.stderr
    sym = subprocess.run(["nm", os.path.join(os.path.dirname(exe), "vgc_api_san.o")], capture_output=True, text=True).stdout
    assert "__asan_" in sym and "__ubsan_" in sym, "the API object was not instrumented"
