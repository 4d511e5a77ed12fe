"""ctypes binding of libvgc.so: same names as the C ABI in include/vgc.h, argument
marshalling only.  torch tensors supply device memory (`data_ptr()`) and the current
HIP stream; every step of the path runs in the library's kernels.

There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvgc.so")

F32, BF16 = 0, 1
FC, CONV = 0, 1


class VgcError(RuntimeError):
    pass


class Group(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("size", C.c_uint32), ("reserved", C.c_uint32)]


class GroupHdr(C.Structure):
    _fields_ = [("exp_field", C.c_uint32), ("count", C.c_uint32), ("word_offset", C.c_uint64)]


class PackStatus(C.Structure):
    _fields_ = [("total_words", C.c_uint64), ("overflow", C.c_uint32), ("plan_mismatch", C.c_uint32)]


class Optimizer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_uint32)]


class Conv2dLayer(C.Structure):
    _fields_ = [("dtype", C.c_int), ("act", C.c_void_p), ("D", C.c_void_p)] + \
               [(k, C.c_uint32) for k in ("B", "H", "W", "Cin", "C", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w")] + \
               [("c", C.c_float), ("g_out", C.c_void_p), ("s_out", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t)]


MOMENTUM_SGD, ADAM = 0, 1

HDR_DTYPE = np.dtype([("exp_field", "<u4"), ("count", "<u4"), ("word_offset", "<u8")])

EXPORTS = {
    # name: (restype, argtypes)
    "vgc_last_error": (C.c_char_p, []),
    "vgc_tile_size": (C.c_uint32, []),
    "vgc_tile_count": (C.c_uint64, [C.c_void_p, C.c_uint32, C.c_uint64]),
    "vgc_plan_bytes": (C.c_size_t, [C.c_void_p, C.c_uint32, C.c_uint64]),
    "vgc_scratch_bytes": (C.c_size_t, [C.c_void_p, C.c_uint32, C.c_uint64]),
    "vgc_scratch_bitmap_offset": (C.c_size_t, [C.c_void_p, C.c_uint32, C.c_uint64]),
    "vgc_plan_build": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_size_t]),
    "vgc_sqgrad_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]),
    "vgc_sqgrad": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                             C.c_uint32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "vgc_sqgrad_noalloc": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                                     C.c_uint32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]),
    "vgc_sqgrad_conv2d_workspace_bytes": (C.c_size_t, [C.c_int] + [C.c_uint32] * 11),
    "vgc_sqgrad_conv2d": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p] + [C.c_uint32] * 11 +
                          [C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "vgc_sqgrad_conv2d_batch": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p]),
    "vgc_accumulate_select": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                                        C.c_uint32, C.c_void_p, C.c_float, C.c_float, C.c_void_p, C.c_void_p]),
    "vgc_accumulate_select_hybrid": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                                               C.c_uint32, C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_void_p,
                                               C.c_void_p]),
    "vgc_accumulate_select_range": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                                              C.c_uint32, C.c_void_p, C.c_uint32, C.c_uint32, C.c_float, C.c_float,
                                              C.c_void_p, C.c_void_p]),
    "vgc_sqgrad_accumulate_select_workspace_bytes": (C.c_size_t, [C.c_int, C.c_uint32, C.c_uint32, C.c_uint32]),
    "vgc_sqgrad_accumulate_select": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_float,
                                               C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                               C.c_uint32, C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                               C.c_void_p, C.c_void_p, C.c_void_p]),
    "vgc_pack": (C.c_int, [C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                           C.c_void_p, C.c_void_p, C.c_void_p]),
    "vgc_run_count": (C.c_uint64, [C.c_void_p, C.c_uint32, C.c_uint64]),
    "vgc_pack_compact": (C.c_int, [C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "vgc_unpack_compact_add_batch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                               C.c_void_p, C.c_uint32, C.c_void_p, C.c_float, C.c_int, C.c_void_p,
                                               C.c_uint64, C.c_void_p]),
    "vgc_unpack_add": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                 C.c_float, C.c_void_p, C.c_uint64, C.c_void_p]),
    "vgc_unpack_add_batch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32,
                                       C.c_void_p, C.c_float, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
    "vgc_unpack_apply": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32,
                                   C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                   C.c_void_p]),
}

_lib = None


def load():
    """Load libvgc.so (built by `python -m paper_1802_06058_amd.build`)."""
    global _lib
    if _lib is None:
        # torch first: it brings its own HIP runtime, and the library must bind to that same copy
        # (device pointers and streams come from torch), not to a second one loaded before it
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise VgcError(f"{LIB_PATH} is not built; run `python -m paper_1802_06058_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(rc):
    if rc != 0:
        raise VgcError(f"vgc error {rc}: {load().vgc_last_error().decode()}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def tile_size():
    return int(load().vgc_tile_size())


class Plan:
    """Host group list + the device plan table built from it (shared by all worker
    states and by the decoder)."""

    def __init__(self, groups, device="cuda"):
        import torch
        lib = load()
        self.n_groups = len(groups)
        self.groups = [(int(o), int(s)) for o, s in groups]
        self.n = sum(s for _, s in self.groups)
        arr = (Group * self.n_groups)()
        for k, (o, s) in enumerate(self.groups):
            arr[k].offset, arr[k].size, arr[k].reserved = o, s, 0
        self.c_groups = arr
        nbytes = lib.vgc_plan_bytes(arr, self.n_groups, self.n)
        if nbytes == 0:
            raise VgcError(lib.vgc_last_error().decode())
        host = torch.empty(nbytes, dtype=torch.uint8)
        _check(lib.vgc_plan_build(arr, self.n_groups, self.n, C.c_void_p(host.data_ptr()), nbytes))
        self.plan_host = host
        self.plan = host.to(device)
        self.n_tiles = int(lib.vgc_tile_count(arr, self.n_groups, self.n))
        self.n_runs = int(lib.vgc_run_count(arr, self.n_groups, self.n))
        self.scratch_bytes = int(lib.vgc_scratch_bytes(arr, self.n_groups, self.n))
        self.bitmap_offset = int(lib.vgc_scratch_bitmap_offset(arr, self.n_groups, self.n))
        self.device = device

    def new_scratch(self):
        import torch
        return torch.empty(self.scratch_bytes, dtype=torch.uint8, device=self.device)

    def new_headers(self):
        import torch
        return torch.zeros(self.n_groups * C.sizeof(GroupHdr), dtype=torch.uint8, device=self.device)

    def new_status(self):
        import torch
        return torch.zeros(C.sizeof(PackStatus), dtype=torch.uint8, device=self.device)

    def send_mask(self, scratch):
        """Send bitmap of the last vgc_accumulate_select, reordered from tile order to
        the flat parameter order (host side; for inspection and tests)."""
        T = tile_size()
        raw = scratch[self.bitmap_offset:self.bitmap_offset + self.n_tiles * (T // 8)].cpu().numpy()
        bits = np.unpackbits(raw, bitorder="little").reshape(self.n_tiles, T).astype(bool)
        out = np.empty(self.n, dtype=bool)
        t = 0
        for off, size in self.groups:
            nt = (size + T - 1) // T
            out[off:off + size] = bits[t:t + nt].reshape(-1)[:size]
            t += nt
        return out


def read_headers(hdrs):
    """[(exp_field, count, word_offset)] from a device header tensor."""
    a = hdrs.cpu().numpy().view(HDR_DTYPE)
    return [(int(x["exp_field"]), int(x["count"]), int(x["word_offset"])) for x in a]


def read_status(status):
    """(total_words, overflow) from a device status tensor (synchronises).  Raises if the kernels found that the
    plan they were given was not built from the group list of the call (nothing was computed then)."""
    a = status.cpu().numpy()
    if int(a[12:16].view("<u4")[0]):
        raise VgcError("the device plan was not built from the group list passed with it: nothing was computed")
    return int(a[:8].view("<u8")[0]), int(a[8:12].view("<u4")[0])


def sqgrad_workspace_bytes(kind, dtype, B, P, J, Cc):
    return int(load().vgc_sqgrad_workspace_bytes(kind, dtype, B, P, J, Cc))


class _Args:
    """Checks of one call's tensors before anything is launched.  The library sees raw pointers, so a tensor
    of the wrong size, type or layout is caught here; and since the kernels dereference data_ptr() as GPU
    memory, so is a tensor in host memory (a forgotten .to(device)) or on another GPU than the call's.
    Sizes and types are reported first, devices last (`launchable`)."""

    def __init__(self, device=None):
        self.device = device
        self.seen = []

    def on_device(self, t, what):
        if t is not None:
            self.seen.append((t, what))

    def need(self, t, numel, dtype, what):
        if t is None:
            return
        self.seen.append((t, what))
        if t.dtype != dtype or t.numel() < numel or not t.is_contiguous():
            raise VgcError(f"{what}: need a contiguous {dtype} tensor of at least {numel} elements, "
                           f"got {t.dtype} with {t.numel()} (contiguous: {t.is_contiguous()})")

    def need_bytes(self, t, nbytes, what):
        if t is None:
            return
        self.seen.append((t, what))
        if t.numel() * t.element_size() < nbytes or not t.is_contiguous():
            raise VgcError(f"{what}: need a contiguous tensor of at least {nbytes} bytes, got {t.numel() * t.element_size()}")

    def need_state(self, plan, scratch=None, **arrays):
        import torch
        self.on_device(plan.plan, "plan")
        for name, t in arrays.items():
            self.need(t, plan.n, torch.float32, name)
        self.need_bytes(scratch, plan.scratch_bytes, "scratch")

    def need_messages(self, plan, words, n_words, hdrs):
        for w, k, h in zip(words, n_words, hdrs):
            if w.element_size() != 4:
                raise VgcError(f"words: need 32-bit elements, got {w.dtype}")
            self.need_bytes(w, 4 * int(k), "words")
            self.need_bytes(h, plan.n_groups * C.sizeof(GroupHdr), "headers")

    def launchable(self):
        """Every tensor seen lives in the memory of one GPU: the plan's, else the first tensor's."""
        import torch
        want = torch.device(self.device) if self.device is not None else None
        for t, what in self.seen:
            if not t.is_cuda:
                raise VgcError(f"{what}: need a tensor in GPU memory, got one on {t.device}")
            if want is None or want.type != "cuda":
                want = t.device
            elif want.index is None:
                want = torch.device("cuda", torch.cuda.current_device())
            if t.device != want:
                raise VgcError(f"{what}: tensor is on {t.device}, the call's other tensors on {want}")


def sqgrad(kind, X, D, c, s_out, g_out=None, workspace=None):
    """vgc_sqgrad.  X, D: float32 or bfloat16 tensors, [B, J]/[B, C] (FC) or [B, P, J]/[B, P, C] (CONV).
    workspace: optional uint8 tensor of sqgrad_workspace_bytes() bytes."""
    import torch
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(X.dtype)
    if dtype is None or D.dtype != X.dtype:
        raise VgcError(f"unsupported dtypes {X.dtype}, {D.dtype}")
    if kind == FC:
        B, J = X.shape
        P, Cc = 1, D.shape[1]
    else:
        B, P, J = X.shape
        Cc = D.shape[2]
    if D.shape[0] != B or (kind != FC and D.shape[1] != P) or not X.is_contiguous() or not D.is_contiguous():
        raise VgcError(f"X {tuple(X.shape)} and D {tuple(D.shape)} do not belong together (or are not contiguous)")
    a = _Args()
    a.on_device(X, "X"); a.on_device(D, "D")
    a.need(s_out, J * Cc, torch.float32, "s_out")
    a.need(g_out, J * Cc, torch.float32, "g_out")
    a.need(workspace, 0, torch.uint8, "workspace")
    a.launchable()
    _check(load().vgc_sqgrad(kind, dtype, _ptr(X), _ptr(D), B, P, J, Cc, float(c), _ptr(g_out), _ptr(s_out),
                             _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()))


NOALLOC_SCRATCH_BYTES = 128 << 20


def sqgrad_noalloc(kind, X, D, c, s_out, g_out=None):
    """vgc_sqgrad_noalloc: vgc_sqgrad with the library's own static working memory (no workspace argument)."""
    import torch
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(X.dtype)
    if dtype is None or D.dtype != X.dtype:
        raise VgcError(f"unsupported dtypes {X.dtype}, {D.dtype}")
    if kind == FC:
        B, J = X.shape
        P, Cc = 1, D.shape[1]
    else:
        B, P, J = X.shape
        Cc = D.shape[2]
    if D.shape[0] != B or (kind != FC and D.shape[1] != P) or not X.is_contiguous() or not D.is_contiguous():
        raise VgcError(f"X {tuple(X.shape)} and D {tuple(D.shape)} do not belong together (or are not contiguous)")
    a = _Args()
    a.on_device(X, "X"); a.on_device(D, "D")
    a.need(s_out, J * Cc, torch.float32, "s_out")
    a.need(g_out, J * Cc, torch.float32, "g_out")
    a.launchable()
    _check(load().vgc_sqgrad_noalloc(kind, dtype, _ptr(X), _ptr(D), B, P, J, Cc, float(c), _ptr(g_out), _ptr(s_out),
                                     _stream()))


def sqgrad_conv2d_workspace_bytes(dtype, B, H, W, Cin, Cc, kh, kw, stride, pad):
    return int(load().vgc_sqgrad_conv2d_workspace_bytes(dtype, B, H, W, Cin, Cc, kh, kw, stride[0], stride[1], pad[0], pad[1]))


def sqgrad_conv2d(act, D, kh, kw, stride, pad, c, s_out, g_out=None, workspace=None):
    """vgc_sqgrad_conv2d.  act [B, H, W, Cin], D [B, Ho, Wo, C] (NHWC, float32 or bfloat16); s_out, g_out float32
    [kh*kw*Cin, C]; workspace: optional uint8 tensor of sqgrad_conv2d_workspace_bytes() bytes."""
    import torch
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(act.dtype)
    if dtype is None or D.dtype != act.dtype:
        raise VgcError(f"unsupported dtypes {act.dtype}, {D.dtype}")
    B, H, W, Cin = act.shape
    Ho, Wo = (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1
    if tuple(D.shape[:3]) != (B, Ho, Wo) or not act.is_contiguous() or not D.is_contiguous():
        raise VgcError(f"D {tuple(D.shape)} is not the output gradient [B, {Ho}, {Wo}, C] of act {tuple(act.shape)} "
                       f"(or a tensor is not contiguous)")
    a = _Args()
    a.on_device(act, "act"); a.on_device(D, "D")
    a.need(s_out, kh * kw * Cin * D.shape[3], torch.float32, "s_out")
    a.need(g_out, kh * kw * Cin * D.shape[3], torch.float32, "g_out")
    a.need(workspace, 0, torch.uint8, "workspace")
    a.launchable()
    _check(load().vgc_sqgrad_conv2d(dtype, _ptr(act), _ptr(D), B, H, W, Cin, D.shape[3], kh, kw, stride[0], stride[1],
                                    pad[0], pad[1], float(c), _ptr(g_out), _ptr(s_out), _ptr(workspace),
                                    0 if workspace is None else workspace.numel(), _stream()))


def _conv2d_layer(a, act, D, kh, kw, stride, pad, c, s_out, g_out, workspace):
    """The checks of sqgrad_conv2d on one layer; its record for the batch call."""
    import torch
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(act.dtype)
    if dtype is None or D.dtype != act.dtype:
        raise VgcError(f"unsupported dtypes {act.dtype}, {D.dtype}")
    B, H, W, Cin = act.shape
    Ho, Wo = (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1
    if tuple(D.shape[:3]) != (B, Ho, Wo) or not act.is_contiguous() or not D.is_contiguous():
        raise VgcError(f"D {tuple(D.shape)} is not the output gradient [B, {Ho}, {Wo}, C] of act {tuple(act.shape)} "
                       f"(or a tensor is not contiguous)")
    a.on_device(act, "act"); a.on_device(D, "D")
    a.need(s_out, kh * kw * Cin * D.shape[3], torch.float32, "s_out")
    a.need(g_out, kh * kw * Cin * D.shape[3], torch.float32, "g_out")
    a.need(workspace, 0, torch.uint8, "workspace")
    addr = lambda t: None if t is None else t.data_ptr()
    return Conv2dLayer(dtype, addr(act), addr(D), B, H, W, Cin, D.shape[3], kh, kw, stride[0], stride[1], pad[0], pad[1],
                       float(c), addr(g_out), addr(s_out), addr(workspace), 0 if workspace is None else workspace.numel())


def sqgrad_conv2d_batch(layers):
    """vgc_sqgrad_conv2d_batch.  layers: sequence of dicts with the arguments of sqgrad_conv2d (act, D, kh, kw, stride,
    pad, c, s_out and optionally g_out, workspace); every layer needs outputs and a workspace of its own."""
    a = _Args()
    recs = [_conv2d_layer(a, L["act"], L["D"], L["kh"], L["kw"], L["stride"], L["pad"], L["c"], L["s_out"], L.get("g_out"),
                          L.get("workspace")) for L in layers]
    a.launchable()
    arr = (Conv2dLayer * len(recs))(*recs)
    _check(load().vgc_sqgrad_conv2d_batch(C.cast(arr, C.c_void_p), len(recs), _stream()))


def accumulate_select(g, s, r, v, plan, alpha, zeta, scratch):
    a = _Args(plan.device)
    a.need_state(plan, scratch, g=g, s=s, r=r, v=v)
    a.launchable()
    _check(load().vgc_accumulate_select(_ptr(g), _ptr(s), _ptr(r), _ptr(v), plan.n, plan.c_groups, plan.n_groups,
                                        _ptr(plan.plan), float(alpha), float(zeta), _ptr(scratch), _stream()))


def accumulate_select_hybrid(g, s, r, v, plan, alpha, zeta, tau, scratch):
    a = _Args(plan.device)
    a.need_state(plan, scratch, g=g, s=s, r=r, v=v)
    a.launchable()
    _check(load().vgc_accumulate_select_hybrid(_ptr(g), _ptr(s), _ptr(r), _ptr(v), plan.n, plan.c_groups,
                                               plan.n_groups, _ptr(plan.plan), float(alpha), float(zeta), float(tau),
                                               _ptr(scratch), _stream()))


def accumulate_select_range(g, s, r, v, plan, first_group, group_count, alpha, zeta, scratch):
    """vgc_accumulate_select_range: the pass over groups [first_group, first_group + group_count) only."""
    a = _Args(plan.device)
    a.need_state(plan, scratch, g=g, s=s, r=r, v=v)
    a.launchable()
    _check(load().vgc_accumulate_select_range(_ptr(g), _ptr(s), _ptr(r), _ptr(v), plan.n, plan.c_groups, plan.n_groups,
                                              _ptr(plan.plan), int(first_group), int(group_count), float(alpha), float(zeta),
                                              _ptr(scratch), _stream()))


def sqgrad_accumulate_select_workspace_bytes(dtype, B, J, Cc):
    return int(load().vgc_sqgrad_accumulate_select_workspace_bytes(dtype, B, J, Cc))


def sqgrad_accumulate_select(X, D, c, r, v, plan, group, alpha, zeta, scratch, workspace, g_out=None, s_out=None):
    """vgc_sqgrad_accumulate_select: the FC statistic of X [B, J], D [B, C] fused into the accumulate pass of
    group `group` (whose size is J * C).  workspace: uint8 tensor of sqgrad_accumulate_select_workspace_bytes()."""
    import torch
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(X.dtype)
    if dtype is None or D.dtype != X.dtype:
        raise VgcError(f"unsupported dtypes {X.dtype}, {D.dtype}")
    if X.dim() != 2 or D.dim() != 2 or D.shape[0] != X.shape[0] or not X.is_contiguous() or not D.is_contiguous():
        raise VgcError(f"X {tuple(X.shape)} and D {tuple(D.shape)} do not belong together (or are not contiguous)")
    B, J = X.shape
    Cc = D.shape[1]
    a = _Args(plan.device)
    a.on_device(X, "X"); a.on_device(D, "D")
    a.need_state(plan, scratch, r=r, v=v)
    a.need(g_out, J * Cc, torch.float32, "g_out")
    a.need(s_out, J * Cc, torch.float32, "s_out")
    a.need(workspace, sqgrad_accumulate_select_workspace_bytes(dtype, B, J, Cc), torch.uint8, "workspace")
    a.launchable()
    _check(load().vgc_sqgrad_accumulate_select(dtype, _ptr(X), _ptr(D), B, J, Cc, float(c), _ptr(r), _ptr(v), plan.n,
                                               plan.c_groups, plan.n_groups, _ptr(plan.plan), int(group), float(alpha),
                                               float(zeta), _ptr(scratch), _ptr(workspace),
                                               0 if workspace is None else workspace.numel(), _ptr(g_out), _ptr(s_out),
                                               _stream()))


def pack(plan, scratch, words, hdrs, status):
    if words.element_size() != 4:
        raise VgcError(f"words: need 32-bit elements, got {words.dtype}")
    a = _Args(plan.device)
    a.on_device(plan.plan, "plan")
    a.need_bytes(words, 0, "words")
    a.need_bytes(scratch, plan.scratch_bytes, "scratch")
    a.need_bytes(hdrs, plan.n_groups * C.sizeof(GroupHdr), "headers")
    a.need_bytes(status, C.sizeof(PackStatus), "status")
    a.launchable()
    _check(load().vgc_pack(plan.n, plan.c_groups, plan.n_groups, _ptr(plan.plan), _ptr(scratch), _ptr(words),
                           words.numel(), _ptr(hdrs), _ptr(status), _stream()))


def unpack_add(words, n_words, hdrs, plan, scale, dense):
    a = _Args(plan.device)
    a.need_messages(plan, [words], [n_words], [hdrs])
    a.need_state(plan, dense=dense)
    a.launchable()
    _check(load().vgc_unpack_add(_ptr(words), int(n_words), _ptr(hdrs), plan.c_groups, plan.n_groups,
                                 _ptr(plan.plan), float(scale), _ptr(dense), plan.n, _stream()))


def _message_tables(words, n_words, hdrs):
    p = len(words)
    wp = (C.c_void_p * max(p, 1))(*[w.data_ptr() for w in words])
    hp = (C.c_void_p * max(p, 1))(*[h.data_ptr() for h in hdrs])
    nw = (C.c_uint64 * max(p, 1))(*[int(x) for x in n_words])
    return wp, nw, hp


def unpack_add_batch(words, n_words, hdrs, plan, scale, dense, overwrite=False):
    """vgc_unpack_add_batch: lists of word tensors, counts and header tensors, one per message."""
    p = len(words)
    if len(n_words) != p or len(hdrs) != p:
        raise VgcError("words, n_words and hdrs must have one entry per message")
    a = _Args(plan.device)
    a.need_messages(plan, words, n_words, hdrs)
    a.need_state(plan, dense=dense)
    a.launchable()
    wp, nw, hp = _message_tables(words, n_words, hdrs)
    _check(load().vgc_unpack_add_batch(wp, nw, hp, p, plan.c_groups, plan.n_groups, _ptr(plan.plan), float(scale),
                                       1 if overwrite else 0, _ptr(dense), plan.n, _stream()))


def unpack_apply(words, n_words, hdrs, plan, scale, param, state1, state2=None, *, kind=MOMENTUM_SGD, lr=0.0,
                 momentum=0.0, beta1=0.9, beta2=0.999, eps=1e-8, step=1):
    """vgc_unpack_apply: decode the messages and take one optimizer step on (param, state1[, state2]) in place."""
    p = len(words)
    if len(n_words) != p or len(hdrs) != p:
        raise VgcError("words, n_words and hdrs must have one entry per message")
    a = _Args(plan.device)
    a.need_messages(plan, words, n_words, hdrs)
    a.need_state(plan, param=param, state1=state1, state2=state2)
    a.launchable()
    wp, nw, hp = _message_tables(words, n_words, hdrs)
    opt = Optimizer(kind, lr, momentum, beta1, beta2, eps, step)
    _check(load().vgc_unpack_apply(wp, nw, hp, p, plan.c_groups, plan.n_groups, _ptr(plan.plan), float(scale),
                                   C.byref(opt), _ptr(param), _ptr(state1), _ptr(state2), plan.n, _stream()))


def pack_compact(plan, scratch, stream_out, tile_bytes, run_offsets, hdrs, status):
    """vgc_pack_compact: the staged result of accumulate_select as a message with compressed indexes.
    stream_out: uint8 tensor; tile_bytes: int16/uint16 tensor [n_tiles]; run_offsets: int64 tensor [n_runs]."""
    a = _Args(plan.device)
    a.on_device(plan.plan, "plan")
    if stream_out.element_size() != 1:
        raise VgcError(f"stream: need 8-bit elements, got {stream_out.dtype}")
    a.need_bytes(stream_out, 0, "stream")
    a.need_bytes(scratch, plan.scratch_bytes, "scratch")
    a.need_bytes(tile_bytes, 2 * plan.n_tiles, "tile_bytes")
    a.need_bytes(run_offsets, 8 * plan.n_runs, "run_offsets")
    a.need_bytes(hdrs, plan.n_groups * C.sizeof(GroupHdr), "headers")
    a.need_bytes(status, C.sizeof(PackStatus), "status")
    a.launchable()
    _check(load().vgc_pack_compact(plan.n, plan.c_groups, plan.n_groups, _ptr(plan.plan), _ptr(scratch), _ptr(stream_out),
                                   stream_out.numel(), _ptr(tile_bytes), _ptr(run_offsets), _ptr(hdrs), _ptr(status), _stream()))


def unpack_compact_add_batch(streams, stream_bytes, tile_bytes, run_offsets, hdrs, plan, scale, dense, overwrite=False):
    """vgc_unpack_compact_add_batch: lists (one entry per message) of stream tensors, their lengths in bytes,
    tile_bytes tensors, run_offsets tensors and header tensors."""
    p = len(streams)
    if not (len(stream_bytes) == len(tile_bytes) == len(run_offsets) == len(hdrs) == p):
        raise VgcError("streams, stream_bytes, tile_bytes, run_offsets and hdrs must have one entry per message")
    a = _Args(plan.device)
    for s, nb, tb, ro, h in zip(streams, stream_bytes, tile_bytes, run_offsets, hdrs):
        if s.element_size() != 1:
            raise VgcError(f"stream: need 8-bit elements, got {s.dtype}")
        a.need_bytes(s, int(nb), "stream")
        a.need_bytes(tb, 2 * plan.n_tiles, "tile_bytes")
        a.need_bytes(ro, 8 * plan.n_runs, "run_offsets")
        a.need_bytes(h, plan.n_groups * C.sizeof(GroupHdr), "headers")
    a.need_state(plan, dense=dense)
    a.launchable()
    arr = lambda ts: (C.c_void_p * max(p, 1))(*[t.data_ptr() for t in ts])
    nb = (C.c_uint64 * max(p, 1))(*[int(x) for x in stream_bytes])
    _check(load().vgc_unpack_compact_add_batch(arr(streams), nb, arr(tile_bytes), arr(run_offsets), arr(hdrs), p, plan.c_groups,
                                               plan.n_groups, _ptr(plan.plan), float(scale), 1 if overwrite else 0, _ptr(dense),
                                               plan.n, _stream()))
