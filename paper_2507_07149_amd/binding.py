"""ctypes binding of libdaf.so: same names as the C ABI, argument marshalling only."""
import ctypes
import os
from typing import Optional, Sequence

import torch

F32, F16, BF16 = 0, 1, 2
_DTYPE_ID = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdaf.so")
_lib = None


class DafError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().daf_status_string(status).decode()
        super().__init__(f"{where}: {msg} ({status})")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libdaf.so.  Fails loudly if it has not been built (python -m paper_2507_07149_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2507_07149_amd.build`; "
                          "there is no fallback path")
    L = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i64, i32, u64 = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64
    L.daf_rand_bits.restype = c.c_int
    L.daf_status_string.argtypes = [c.c_int]
    L.daf_status_string.restype = c.c_char_p
    L.daf_plan.argtypes = [c.POINTER(i64), c.c_int, i32, vp, i64, vp, c.POINTER(vp)]
    L.daf_plan.restype = c.c_int
    for name, res in (("daf_plan_num_elements", i64), ("daf_plan_num_groups", i64),
                      ("daf_plan_packed_words", i64), ("daf_plan_group_size", i32),
                      ("daf_plan_uniform_bits", i32)):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = res
    L.daf_plan_update.argtypes = [vp, vp, vp]
    L.daf_plan_update.restype = c.c_int
    L.daf_plan_finish.argtypes = [vp, vp]
    L.daf_plan_finish.restype = c.c_int
    L.daf_plan_packed_words_bound.argtypes = [vp]
    L.daf_plan_packed_words_bound.restype = i64
    L.daf_plan_copy_offsets.argtypes = [vp, vp]
    L.daf_plan_copy_offsets.restype = c.c_int
    L.daf_plan_quantize_route.argtypes = [vp, c.c_int]
    L.daf_plan_quantize_route.restype = c.c_int
    L.daf_plan_set_output_cached.argtypes = [vp, c.c_int]
    L.daf_plan_set_output_cached.restype = c.c_int
    L.daf_plan_destroy.argtypes = [vp]
    L.daf_plan_destroy.restype = None
    L.daf_quantize_pack.argtypes = [vp, vp, c.c_int, u64, vp, vp, vp, vp]
    L.daf_quantize_pack.restype = c.c_int
    L.daf_quantize_pack_static.argtypes = [vp, vp, c.c_int, u64, vp, vp, vp, vp]
    L.daf_quantize_pack_static.restype = c.c_int
    L.daf_unpack_dequantize.argtypes = [vp, vp, vp, vp, vp, vp, c.c_int, vp]
    L.daf_unpack_dequantize.restype = c.c_int
    L.daf_quantize_pack_metrics.argtypes = [vp, vp, c.c_int, u64, vp, vp, vp, vp, vp]
    L.daf_quantize_pack_metrics.restype = c.c_int
    L.daf_quantize_pack_batch.argtypes = [vp, i32, c.c_int, vp]
    L.daf_quantize_pack_batch.restype = c.c_int
    L.daf_unpack_dequantize_batch.argtypes = [vp, i32, c.c_int, vp]
    L.daf_unpack_dequantize_batch.restype = c.c_int
    L.daf_relu_quantize_pack.argtypes = [vp, vp, c.c_int, u64, vp, vp, vp, vp, vp]
    L.daf_relu_quantize_pack.restype = c.c_int
    L.daf_linear_quantize_pack.argtypes = [vp, vp, vp, i64, i64, c.c_int, u64, vp, vp, vp, vp, vp]
    L.daf_linear_quantize_pack.restype = c.c_int
    L.daf_linear_tile_of_workgroup.argtypes = [i32, i32, i32, vp, vp]
    L.daf_linear_tile_of_workgroup.restype = c.c_int
    L.daf_unpack_relu_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, c.c_int, vp]
    L.daf_unpack_relu_backward.restype = c.c_int
    L.daf_unpack_matmul_workspace_bytes.argtypes = [vp, i64, i64]
    L.daf_unpack_matmul_workspace_bytes.restype = i64
    L.daf_unpack_matmul_grad_weight.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, c.c_int, vp, vp, vp]
    L.daf_unpack_matmul_grad_weight.restype = c.c_int
    L.daf_group_minmax.argtypes = [vp, vp, c.c_int, vp, vp, vp]
    L.daf_group_minmax.restype = c.c_int
    L.daf_select_bits_workspace_bytes.argtypes = [i64]
    L.daf_select_bits_workspace_bytes.restype = i64
    L.daf_select_bits.argtypes = [vp, vp, i64, vp, i32, vp, vp, vp]
    L.daf_select_bits.restype = c.c_int
    L.daf_select_bits_from_scale.argtypes = [vp, vp, i32, i64, vp, i32, vp, vp, vp]
    L.daf_select_bits_from_scale.restype = c.c_int
    L.daf_minmax_workspace_bytes.restype = i64
    L.daf_minmax_workspace_init.argtypes = [vp, vp]
    L.daf_minmax_workspace_init.restype = c.c_int
    L.daf_minmax.argtypes = [vp, c.c_int, i64, c.c_int, vp, vp, vp]
    L.daf_minmax.restype = c.c_int
    _lib = L
    return L


def rand_bits() -> int:
    return int(load_library().daf_rand_bits())


def dtype_id(dtype: torch.dtype) -> int:
    return _DTYPE_ID[dtype]


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


# The C ABI takes bare pointers and cannot see sizes, so a tensor that is too small, on the host,
# strided or of the wrong dtype would make a kernel read or write out of bounds.  These checks are
# the only place where that can be caught; they raise ValueError before anything is launched.
_ELEM_DTYPES = (torch.float32, torch.float16, torch.bfloat16)


class _Args:
    """Checks the tensors of one call: type, dtype, layout and size as each is named, and that
    all of them live on the device once every size has passed (`on_device`)."""

    def __init__(self, plan=None):
        self.plan = plan
        self.seen = []

    def tensor(self, name: str, t, dtype, numel: int, exact: bool = False) -> None:
        if not isinstance(t, torch.Tensor):
            raise ValueError(f"{name}: expected a torch.Tensor, got {type(t).__name__}")
        if not t.is_contiguous():
            raise ValueError(f"{name}: must be contiguous")
        if isinstance(dtype, tuple):
            if t.dtype not in dtype:
                raise ValueError(f"{name}: dtype {t.dtype} not in {dtype}")
        elif t.dtype != dtype:
            raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
        if (t.numel() != numel) if exact else (t.numel() < numel):
            raise ValueError(f"{name}: {t.numel()} elements, expected {'' if exact else 'at least '}{numel}")
        self.seen.append((name, t))

    def activation(self, name: str, t) -> None:
        self.tensor(name, t, _ELEM_DTYPES, self.plan.num_elements, exact=True)

    def packed(self, words, mn, scale, prefix: str = "") -> None:
        self.tensor(prefix + "words", words, torch.int32, self.plan.packed_words)
        self.tensor(prefix + "min", mn, torch.float32, self.plan.num_groups)
        self.tensor(prefix + "scale", scale, torch.float32, self.plan.num_groups)

    def bits(self, bits) -> None:
        if bits is not None:
            self.tensor("bits", bits, torch.uint8, self.plan.num_groups)

    def on_device(self) -> None:
        for name, t in self.seen:
            if not t.is_cuda:
                raise ValueError(f"{name}: must be a device (cuda) tensor")


class Plan:
    """Owns a daf_plan_t*.  `bits` (a device uint8 tensor for per-group widths) is kept alive."""

    def __init__(self, handle: int, bits_keepalive=None):
        self._h = handle
        self._keep = bits_keepalive
        # the plan's sizes never change: read them once, so that the argument checks of every
        # call cost no foreign-function calls
        L = load_library()
        self.num_elements = int(L.daf_plan_num_elements(handle))
        self.num_groups = int(L.daf_plan_num_groups(handle))
        self.packed_words = int(L.daf_plan_packed_words(handle))
        self.group_size = int(L.daf_plan_group_size(handle))
        self.uniform_bits = int(L.daf_plan_uniform_bits(handle))

    @property
    def handle(self) -> int:
        if not self._h:
            raise ValueError("plan already destroyed")
        return self._h

    def update(self, bits: torch.Tensor, stream=None) -> None:
        """daf_plan_update: new per-group widths (device uint8[G]) for this plan, enqueued on `stream`
        without synchronizing; `packed_words` reads as the 8-bit bound until `finish()`."""
        a = _Args(self)
        a.tensor("bits", bits, torch.uint8, self.num_groups, exact=True)
        a.on_device()
        rc = load_library().daf_plan_update(self.handle, bits.data_ptr(), _stream_handle(stream))
        if rc != 0:
            raise DafError(rc, "daf_plan_update")
        self._keep = bits
        self.packed_words = int(load_library().daf_plan_packed_words(self.handle))

    def finish(self, stream=None) -> None:
        """daf_plan_finish: one synchronization; the exact packed size, and DafError if the last
        update contained a width outside {1,2,4,8}."""
        rc = load_library().daf_plan_finish(self.handle, _stream_handle(stream))
        self.packed_words = int(load_library().daf_plan_packed_words(self.handle))
        if rc != 0:
            raise DafError(rc, "daf_plan_finish")

    @property
    def packed_words_bound(self) -> int:
        return int(load_library().daf_plan_packed_words_bound(self.handle))

    ROUTES = ("tile", "units", "long", "two_pass", "group")

    def quantize_route(self, dtype: torch.dtype) -> str:
        rc = load_library().daf_plan_quantize_route(self.handle, _DTYPE_ID[dtype])
        if rc < 0:
            raise DafError(rc, "daf_plan_quantize_route")
        return Plan.ROUTES[rc]

    def set_output_cached(self, cached: bool) -> None:
        rc = load_library().daf_plan_set_output_cached(self.handle, 1 if cached else 0)
        if rc != 0:
            raise DafError(rc, "daf_plan_set_output_cached")

    def offsets(self) -> torch.Tensor:
        out = torch.empty(self.num_groups, dtype=torch.int32)
        rc = load_library().daf_plan_copy_offsets(self.handle, out.data_ptr())
        if rc != 0:
            raise DafError(rc, "daf_plan_copy_offsets")
        return out

    def destroy(self):
        if self._h:
            load_library().daf_plan_destroy(self._h)
            self._h = 0

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def daf_plan(shape: Sequence[int], group_size: int, bits, stream=None) -> Plan:
    """bits: an int (one width for all groups) or a device uint8 tensor with one width per group."""
    L = load_library()
    shp = (ctypes.c_int64 * len(shape))(*[int(s) for s in shape])
    out = ctypes.c_void_p()
    if isinstance(bits, int):
        b = (ctypes.c_uint8 * 1)(bits)
        rc = L.daf_plan(shp, len(shape), group_size, ctypes.cast(b, ctypes.c_void_p), 1, None, ctypes.byref(out))
        keep = None
    else:
        if bits.dtype != torch.uint8 or not bits.is_cuda or not bits.is_contiguous():
            raise TypeError("per-group bits must be a contiguous uint8 device tensor")
        rc = L.daf_plan(shp, len(shape), group_size, bits.data_ptr(), bits.numel(), _stream_handle(stream),
                        ctypes.byref(out))
        keep = bits
    if rc != 0:
        raise DafError(rc, "daf_plan")
    return Plan(out.value, keep)


def daf_quantize_pack(plan: Plan, x: torch.Tensor, seed: int, out_words: torch.Tensor, out_min: torch.Tensor,
                      out_scale: torch.Tensor, stream=None) -> None:
    a = _Args(plan)
    a.activation("x", x)
    a.packed(out_words, out_min, out_scale, "out_")
    a.on_device()
    rc = load_library().daf_quantize_pack(plan.handle, x.data_ptr(), _DTYPE_ID[x.dtype], seed,
                                          out_words.data_ptr(), out_min.data_ptr(), out_scale.data_ptr(),
                                          _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_quantize_pack")


STATIC_SCRATCH_BYTES = 2 << 20      # DAF_STATIC_SCRATCH_BYTES of daf.h


def daf_quantize_pack_static(plan: Plan, x: torch.Tensor, seed: int, out_words: torch.Tensor, out_min: torch.Tensor,
                             out_scale: torch.Tensor, stream=None) -> None:
    """daf_quantize_pack that allocates nothing: the two-pass route's scratch is the library's static buffer."""
    a = _Args(plan)
    a.activation("x", x)
    a.packed(out_words, out_min, out_scale, "out_")
    a.on_device()
    rc = load_library().daf_quantize_pack_static(plan.handle, x.data_ptr(), _DTYPE_ID[x.dtype], seed,
                                                 out_words.data_ptr(), out_min.data_ptr(), out_scale.data_ptr(),
                                                 _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_quantize_pack_static")


def daf_unpack_dequantize(plan: Plan, words: torch.Tensor, mn: torch.Tensor, scale: torch.Tensor,
                          out_x: torch.Tensor, bits: Optional[torch.Tensor] = None, stream=None) -> None:
    a = _Args(plan)
    a.packed(words, mn, scale)
    a.bits(bits)
    a.activation("out_x", out_x)
    a.on_device()
    rc = load_library().daf_unpack_dequantize(plan.handle, words.data_ptr(), mn.data_ptr(), scale.data_ptr(),
                                              bits.data_ptr() if bits is not None else None,
                                              out_x.data_ptr(), _DTYPE_ID[out_x.dtype], _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_unpack_dequantize")


class _QuantizeItem(ctypes.Structure):
    _fields_ = [("plan", ctypes.c_void_p), ("x", ctypes.c_void_p), ("seed", ctypes.c_uint64),
                ("out_words", ctypes.c_void_p), ("out_min", ctypes.c_void_p), ("out_scale", ctypes.c_void_p)]


class _DequantizeItem(ctypes.Structure):
    _fields_ = [("plan", ctypes.c_void_p), ("words", ctypes.c_void_p), ("min", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("bits", ctypes.c_void_p), ("out_x", ctypes.c_void_p)]


def quantize_items(items):
    """Marshals [(plan, x, seed, out_words, out_min, out_scale), ...] once; the result can be passed to
    daf_quantize_pack_batch any number of times while the tensors stay alive."""
    arr = (_QuantizeItem * len(items))()
    chk = _Args()
    for it, (plan, x, seed, words, mn, sc) in zip(arr, items):
        chk.plan = plan
        chk.activation("x", x)
        chk.packed(words, mn, sc, "out_")
        if x.dtype != items[0][1].dtype:
            raise ValueError("all tensors of a list call must have one dtype")
        it.plan, it.x, it.seed = plan.handle, x.data_ptr(), seed
        it.out_words, it.out_min, it.out_scale = words.data_ptr(), mn.data_ptr(), sc.data_ptr()
    chk.on_device()
    arr.dtype_id = _DTYPE_ID[items[0][1].dtype]
    return arr


def dequantize_items(items):
    """Marshals [(plan, words, min, scale, out_x, bits or None), ...] for daf_unpack_dequantize_batch."""
    arr = (_DequantizeItem * len(items))()
    chk = _Args()
    for it, (plan, words, mn, sc, out_x, bits) in zip(arr, items):
        chk.plan = plan
        chk.packed(words, mn, sc)
        chk.bits(bits)
        chk.activation("out_x", out_x)
        if out_x.dtype != items[0][4].dtype:
            raise ValueError("all tensors of a list call must have one dtype")
        it.plan, it.words, it.min, it.scale = plan.handle, words.data_ptr(), mn.data_ptr(), sc.data_ptr()
        it.bits = bits.data_ptr() if bits is not None else None
        it.out_x = out_x.data_ptr()
    chk.on_device()
    arr.dtype_id = _DTYPE_ID[items[0][4].dtype]
    return arr


def daf_quantize_pack_batch(items, stream=None) -> None:
    """items: a list of (plan, x, seed, out_words, out_min, out_scale), or the result of quantize_items."""
    arr = items if isinstance(items, ctypes.Array) else quantize_items(items)
    rc = load_library().daf_quantize_pack_batch(ctypes.cast(arr, ctypes.c_void_p), len(arr), arr.dtype_id,
                                                _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_quantize_pack_batch")


def daf_unpack_dequantize_batch(items, stream=None) -> None:
    """items: a list of (plan, words, min, scale, out_x, bits or None), or the result of dequantize_items."""
    arr = items if isinstance(items, ctypes.Array) else dequantize_items(items)
    rc = load_library().daf_unpack_dequantize_batch(ctypes.cast(arr, ctypes.c_void_p), len(arr), arr.dtype_id,
                                                    _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_unpack_dequantize_batch")


def daf_unpack_relu_backward(plan: Plan, words: torch.Tensor, mn: torch.Tensor, scale: torch.Tensor,
                             grad_y: torch.Tensor, out_grad_z: torch.Tensor, bits: Optional[torch.Tensor] = None,
                             stream=None) -> None:
    a = _Args(plan)
    a.packed(words, mn, scale)
    a.bits(bits)
    a.activation("grad_y", grad_y)
    a.activation("out_grad_z", out_grad_z)
    if out_grad_z.dtype != grad_y.dtype:
        raise ValueError("out_grad_z must have the dtype of grad_y")
    a.on_device()
    rc = load_library().daf_unpack_relu_backward(plan.handle, words.data_ptr(), mn.data_ptr(), scale.data_ptr(),
                                                 bits.data_ptr() if bits is not None else None, grad_y.data_ptr(),
                                                 out_grad_z.data_ptr(), _DTYPE_ID[grad_y.dtype],
                                                 _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_unpack_relu_backward")


def daf_unpack_matmul_workspace_bytes(plan: Plan, N: int, K: int) -> int:
    return int(load_library().daf_unpack_matmul_workspace_bytes(plan.handle, N, K))


def daf_unpack_matmul_grad_weight(plan: Plan, words: torch.Tensor, mn: torch.Tensor, scale: torch.Tensor,
                                  grad_y: torch.Tensor, out_grad_w: torch.Tensor,
                                  workspace: Optional[torch.Tensor] = None, bits: Optional[torch.Tensor] = None,
                                  stream=None) -> None:
    """grad_y is [M, N]; out_grad_w is float32 [N, K]; the plan's tensor is read as [M, K]."""
    a = _Args(plan)
    a.packed(words, mn, scale)
    a.bits(bits)
    if out_grad_w.dim() != 2 or grad_y.dim() != 2:
        raise ValueError("grad_y must be [M, N] and out_grad_w [N, K]")
    if plan.num_elements % out_grad_w.shape[1] != 0:
        raise ValueError("K = out_grad_w.shape[1] must divide the plan's element count")
    a.tensor("grad_y", grad_y, _ELEM_DTYPES, (plan.num_elements // out_grad_w.shape[1]) * out_grad_w.shape[0], exact=True)
    a.tensor("out_grad_w", out_grad_w, torch.float32, out_grad_w.numel())
    need = daf_unpack_matmul_workspace_bytes(plan, out_grad_w.shape[0], out_grad_w.shape[1])
    if need > 0 and workspace is not None:          # a missing workspace is the library's DAF_EINVAL
        a.tensor("workspace", workspace, workspace.dtype, -(-need // workspace.element_size()))
    N, K = out_grad_w.shape
    if grad_y.shape[-1] != N:
        raise ValueError("out_grad_w must be float32 [N, K] with N = grad_y.shape[-1]")
    a.on_device()
    rc = load_library().daf_unpack_matmul_grad_weight(
        plan.handle, words.data_ptr(), mn.data_ptr(), scale.data_ptr(), bits.data_ptr() if bits is not None else None,
        grad_y.data_ptr(), N, K, _DTYPE_ID[grad_y.dtype], out_grad_w.data_ptr(),
        workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_unpack_matmul_grad_weight")


REDUCE_TWO_PASS, REDUCE_ATOMIC = 0, 1


def daf_minmax_workspace(device="cuda:0", stream=None) -> torch.Tensor:
    """Allocates and prepares a workspace for daf_minmax (reusable across calls that do not overlap)."""
    L = load_library()
    ws = torch.empty(int(L.daf_minmax_workspace_bytes()), dtype=torch.uint8, device=device)
    rc = L.daf_minmax_workspace_init(ws.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_minmax_workspace_init")
    return ws


def daf_minmax(x: torch.Tensor, method: int, workspace: torch.Tensor, out_minmax: torch.Tensor, stream=None) -> None:
    a = _Args()
    a.tensor("x", x, _ELEM_DTYPES, 1)
    a.tensor("workspace", workspace, torch.uint8, int(load_library().daf_minmax_workspace_bytes()))
    a.tensor("out_minmax", out_minmax, torch.float32, 2)
    a.on_device()
    rc = load_library().daf_minmax(x.data_ptr(), _DTYPE_ID[x.dtype], x.numel(), method, workspace.data_ptr(),
                                   out_minmax.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_minmax")


def daf_group_minmax(plan: Plan, x: torch.Tensor, out_min: torch.Tensor, out_max: torch.Tensor, stream=None) -> None:
    a = _Args(plan)
    a.activation("x", x)
    a.tensor("out_min", out_min, torch.float32, plan.num_groups)
    a.tensor("out_max", out_max, torch.float32, plan.num_groups)
    a.on_device()
    rc = load_library().daf_group_minmax(plan.handle, x.data_ptr(), _DTYPE_ID[x.dtype], out_min.data_ptr(),
                                         out_max.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_group_minmax")


def daf_select_bits_workspace(num_groups: int, device="cuda:0") -> torch.Tensor:
    nbytes = int(load_library().daf_select_bits_workspace_bytes(num_groups))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def daf_select_bits(group_min: torch.Tensor, group_max: torch.Tensor, classes: Sequence[int], out_bits: torch.Tensor,
                    workspace: torch.Tensor, stream=None) -> None:
    G = group_min.numel() if isinstance(group_min, torch.Tensor) else 0
    a = _Args()
    a.tensor("group_min", group_min, torch.float32, max(G, 1))
    a.tensor("group_max", group_max, torch.float32, G, exact=True)
    a.tensor("out_bits", out_bits, torch.uint8, G)
    a.tensor("workspace", workspace, torch.uint8, int(load_library().daf_select_bits_workspace_bytes(G)))
    a.on_device()
    cl = (ctypes.c_uint8 * len(classes))(*[int(c) for c in classes])
    rc = load_library().daf_select_bits(group_min.data_ptr(), group_max.data_ptr(), group_min.numel(),
                                        ctypes.cast(cl, ctypes.c_void_p), len(classes), out_bits.data_ptr(),
                                        workspace.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_select_bits")


def daf_select_bits_from_scale(group_scale: torch.Tensor, prev_bits, classes: Sequence[int], out_bits: torch.Tensor,
                               workspace: torch.Tensor, stream=None) -> None:
    """Widths for the next iteration from the scales (and widths: a uint8 tensor, or one int for
    all groups) of an earlier daf_quantize_pack: no pass over the activation."""
    G = group_scale.numel() if isinstance(group_scale, torch.Tensor) else 0
    a = _Args()
    a.tensor("group_scale", group_scale, torch.float32, max(G, 1))
    uniform = 0
    if isinstance(prev_bits, torch.Tensor):
        a.tensor("prev_bits", prev_bits, torch.uint8, G, exact=True)
    else:
        uniform = int(prev_bits)
    a.tensor("out_bits", out_bits, torch.uint8, G)
    a.tensor("workspace", workspace, torch.uint8, int(load_library().daf_select_bits_workspace_bytes(G)))
    a.on_device()
    cl = (ctypes.c_uint8 * len(classes))(*[int(c) for c in classes])
    rc = load_library().daf_select_bits_from_scale(
        group_scale.data_ptr(), prev_bits.data_ptr() if isinstance(prev_bits, torch.Tensor) else None, uniform, G,
        ctypes.cast(cl, ctypes.c_void_p), len(classes), out_bits.data_ptr(), workspace.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_select_bits_from_scale")


def daf_relu_quantize_pack(plan: Plan, z: torch.Tensor, seed: int, out_y: torch.Tensor, out_words: torch.Tensor,
                           out_min: torch.Tensor, out_scale: torch.Tensor, stream=None) -> None:
    a = _Args(plan)
    a.activation("z", z)
    a.activation("out_y", out_y)
    a.packed(out_words, out_min, out_scale, "out_")
    if out_y.dtype != z.dtype:
        raise ValueError("out_y must have the dtype of z")
    a.on_device()
    rc = load_library().daf_relu_quantize_pack(plan.handle, z.data_ptr(), _DTYPE_ID[z.dtype], seed, out_y.data_ptr(),
                                               out_words.data_ptr(), out_min.data_ptr(), out_scale.data_ptr(),
                                               _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_relu_quantize_pack")


def daf_linear_quantize_pack(plan: Plan, x: torch.Tensor, weight: torch.Tensor, seed: int, out_y: torch.Tensor,
                             out_words: torch.Tensor, out_min: torch.Tensor, out_scale: torch.Tensor, stream=None) -> None:
    """y = x @ weight.T with the quantize+pack of y in the product's epilogue; `plan` describes y.
    With out_words, out_min and out_scale all None: the product alone."""
    if x.dim() != 2 or weight.dim() != 2 or x.shape[1] != weight.shape[1]:
        raise ValueError("x must be [M, K] and weight [N, K]")
    M, K = x.shape
    N = weight.shape[0]
    if M * N != plan.num_elements:
        raise ValueError(f"the plan describes {plan.num_elements} elements, y has {M * N}")
    a = _Args(plan)
    a.tensor("x", x, x.dtype, M * K, exact=True)
    a.tensor("weight", weight, x.dtype, N * K, exact=True)
    a.activation("out_y", out_y)
    product_only = out_words is None and out_min is None and out_scale is None
    if not product_only:
        a.packed(out_words, out_min, out_scale, "out_")
    if out_y.dtype != x.dtype:
        raise ValueError("out_y must have the dtype of x")
    a.on_device()
    ptr = (lambda t: None) if product_only else (lambda t: t.data_ptr())
    rc = load_library().daf_linear_quantize_pack(plan.handle, x.data_ptr(), weight.data_ptr(), N, K, _DTYPE_ID[x.dtype],
                                                 seed, out_y.data_ptr(), ptr(out_words), ptr(out_min),
                                                 ptr(out_scale), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_linear_quantize_pack")


def daf_quantize_pack_metrics(plan: Plan, x: torch.Tensor, seed: int, out_words: torch.Tensor, out_min: torch.Tensor,
                              out_scale: torch.Tensor, out_metrics: torch.Tensor, stream=None) -> None:
    a = _Args(plan)
    a.activation("x", x)
    a.packed(out_words, out_min, out_scale, "out_")
    a.tensor("out_metrics", out_metrics, torch.float32, 3 * plan.num_groups)
    a.on_device()
    rc = load_library().daf_quantize_pack_metrics(plan.handle, x.data_ptr(), _DTYPE_ID[x.dtype], seed,
                                                  out_words.data_ptr(), out_min.data_ptr(), out_scale.data_ptr(),
                                                  out_metrics.data_ptr(), _stream_handle(stream))
    if rc != 0:
        raise DafError(rc, "daf_quantize_pack_metrics")
