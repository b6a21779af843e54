"""ctypes binding with the same names as include/bitstack.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbitstack.so")
_lib = None

KERNEL_AUTO, KERNEL_REFERENCE, KERNEL_DECODE, KERNEL_PANEL, KERNEL_MATERIALISE = 0, 1, 2, 3, 4
Y_F16, Y_F32 = 0, 1
OPT_DECODE_BGROUPS, OPT_DECODE_TILES, OPT_DECODE_KS_CHUNKS, OPT_DECODE_EARLY, OPT_DENSE_TILE = 3, 4, 5, 6, 7


class BitStackError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().bitstack_strerror(code).decode()
        if code == -7:
            msg += f" (hipError {lib().bitstack_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Loads libbitstack.so; builds it first only if it is not there.  Fails loudly
    (no fallback of any kind) when the library cannot be loaded."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    L = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    L.bitstack_block_bytes.restype = sz
    L.bitstack_block_bytes.argtypes = [i32, i32, i32]
    L.bitstack_packed_bytes.restype = sz
    L.bitstack_packed_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.bitstack_pack_signs_from_f32.argtypes = [i32, i32, vp, vp]
    L.bitstack_pack_image_host.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz]
    L.bitstack_unpack_image_host.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, vp, vp]
    L.bitstack_pack_blocks.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, C.POINTER(vp)]
    L.bitstack_unpack_blocks.argtypes = [vp, i32, vp, vp, vp, vp]
    L.bitstack_linear.argtypes = [vp, vp, i32, vp, vp]
    L.bitstack_linear_batched.argtypes = [vp, i32, vp, i32, vp, i32, vp]
    L.bitstack_linear_select.argtypes = [vp, i32, vp, i32, vp, i32, i32, vp]
    L.bitstack_weight_shape.argtypes = [vp] + [C.POINTER(i32)] * 5
    L.bitstack_linear_many.argtypes = [vp, i32, i32, vp]
    L.bitstack_linear_many.restype = i32
    L.bitstack_linear_static.argtypes = [vp, vp, i32, vp, vp]
    L.bitstack_linear_static.restype = i32
    L.bitstack_static_workspace_bytes.restype = sz
    L.bitstack_static_workspace_bytes.argtypes = []
    L.bitstack_set_option.argtypes = [i32, i32]
    L.bitstack_probe_read.argtypes = [vp, sz, vp, i32, vp]
    L.bitstack_probe_read.restype = i32
    L.bitstack_block_staging_bytes.restype = sz
    L.bitstack_block_staging_bytes.argtypes = [i32, i32, i32]
    L.bitstack_stage_block_host.argtypes = [i32, i32, i32, vp, vp, vp, vp, sz]
    L.bitstack_stage_block_host.restype = i32
    L.bitstack_create_stack.argtypes = [i32, i32, i32, i32, i32, vp, vp, sz, vp, C.POINTER(vp)]
    L.bitstack_create_stack.restype = i32
    L.bitstack_push_block.argtypes = [vp, vp, vp]
    L.bitstack_push_block.restype = i32
    L.bitstack_push_block_device.argtypes = [vp, vp, vp, vp, vp]
    L.bitstack_push_block_device.restype = i32
    L.bitstack_pop_block.argtypes = [vp]
    L.bitstack_pop_block.restype = i32
    L.bitstack_resident_blocks.argtypes = [vp]
    L.bitstack_resident_blocks.restype = i32
    L.bitstack_resident_bytes.argtypes = [vp]
    L.bitstack_resident_bytes.restype = sz
    L.bitstack_dense_bytes.restype = sz
    L.bitstack_dense_bytes.argtypes = [i32, i32]
    L.bitstack_restore_max_blocks.restype = i32
    L.bitstack_restore_max_blocks.argtypes = []
    L.bitstack_restore_weight.argtypes = [vp, i32, vp, sz, vp]
    L.bitstack_restore_weight.restype = i32
    L.bitstack_linear_dense.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.bitstack_linear_dense.restype = i32
    L.bitstack_linear_materialised.argtypes = [vp, i32, vp, i32, vp, sz, vp, i32, vp]
    L.bitstack_linear_materialised.restype = i32
    L.bitstack_linear_batched_ws.argtypes = [vp, i32, vp, i32, vp, i32, vp, sz, vp]
    L.bitstack_linear_batched_ws.restype = i32
    L.bitstack_choose_kernel.argtypes = [i32, i32, i32, i32, i32, i32, sz]
    L.bitstack_choose_kernel.restype = i32
    L.bitstack_decompose_workspace_bytes.restype = sz
    L.bitstack_decompose_workspace_bytes.argtypes = [i32, i32, i32]
    L.bitstack_decompose.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.bitstack_decompose.restype = i32
    L.bitstack_order_check.argtypes = [i32, vp, vp, i32]
    L.bitstack_order_check.restype = i32
    L.bitstack_budget_position.argtypes = [i32, vp, vp, i32, sz, C.POINTER(i32), C.POINTER(sz)]
    L.bitstack_budget_position.restype = i32
    L.bitstack_manager_create.argtypes = [i32, vp, C.POINTER(vp)]
    L.bitstack_manager_create.restype = i32
    L.bitstack_manager_release.argtypes = [vp]
    L.bitstack_manager_release.restype = None
    L.bitstack_manager_set_block.argtypes = [vp, i32, i32, vp]
    L.bitstack_manager_set_block.restype = i32
    L.bitstack_manager_set_order.argtypes = [vp, vp, i32]
    L.bitstack_manager_set_order.restype = i32
    L.bitstack_manager_set_budget.argtypes = [vp, sz, vp, C.POINTER(i32), C.POINTER(i32)]
    L.bitstack_manager_set_budget.restype = i32
    L.bitstack_manager_position.argtypes = [vp]
    L.bitstack_manager_position.restype = i32
    L.bitstack_manager_resident_bytes.argtypes = [vp]
    L.bitstack_manager_resident_bytes.restype = sz
    L.bitstack_manager_n_loaded.argtypes = [vp, i32]
    L.bitstack_manager_n_loaded.restype = i32
    L.bitstack_plan_create.argtypes = [vp, i32, C.POINTER(vp)]
    L.bitstack_plan_create.restype = i32
    L.bitstack_plan_launch.argtypes = [vp, vp]
    L.bitstack_plan_launch.restype = i32
    L.bitstack_plan_steps.argtypes = [vp]
    L.bitstack_plan_steps.restype = i32
    L.bitstack_plan_release.argtypes = [vp]
    L.bitstack_plan_release.restype = None
    L.bitstack_release.argtypes = [vp]
    L.bitstack_release.restype = None
    L.bitstack_strerror.restype = C.c_char_p
    L.bitstack_strerror.argtypes = [i32]
    L.bitstack_last_hip_error.restype = i32
    for name in ("bitstack_pack_signs_from_f32", "bitstack_pack_image_host", "bitstack_unpack_image_host",
                 "bitstack_pack_blocks", "bitstack_unpack_blocks", "bitstack_linear",
                 "bitstack_linear_batched", "bitstack_linear_select", "bitstack_weight_shape",
                 "bitstack_set_option"):
        getattr(L, name).restype = i32
    _lib = L
    return L


class Job(C.Structure):
    _fields_ = [("x", C.c_void_p), ("blocks", C.c_void_p), ("n_loaded", C.c_int), ("y", C.c_void_p)]


def make_jobs(items):
    """items: iterable of (x tensor, PackedStack, n_loaded, y tensor) -> ctypes job array."""
    items = list(items)
    arr = (Job * len(items))()
    for j, (x, ps, nl, y) in zip(arr, items):
        j.x, j.blocks, j.n_loaded, j.y = x.data_ptr(), ps.handle.value, int(nl), y.data_ptr()
    arr._keepalive = items
    return arr


def linear_many(jobs, repeat: int = 1, stream=None):
    """bitstack_linear_many on a job array from make_jobs (current torch stream by default)."""
    import torch
    st = C.c_void_p((stream or torch.cuda.current_stream()).cuda_stream)
    _check(lib().bitstack_linear_many(jobs, len(jobs), repeat, st), "bitstack_linear_many")


class TokenPlan:
    """bitstack_plan_*: a job array from make_jobs prepared once, launched once per token."""

    def __init__(self, jobs):
        self._jobs = jobs   # keeps the tensors and stacks alive
        self._h = C.c_void_p()
        _check(lib().bitstack_plan_create(jobs, len(jobs), C.byref(self._h)), "bitstack_plan_create")

    @property
    def steps(self) -> int:
        return int(lib().bitstack_plan_steps(self._h))

    def launch(self, stream=None):
        import torch
        st = C.c_void_p((stream or torch.cuda.current_stream()).cuda_stream)
        _check(lib().bitstack_plan_launch(self._h, st), "bitstack_plan_launch")

    def release(self):
        if self._h:
            lib().bitstack_plan_release(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass


def _check(rc: int, where: str):
    if rc != 0:
        raise BitStackError(rc, where)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def strerror(code: int) -> str:
    return lib().bitstack_strerror(code).decode()


def block_bytes(out: int, inn: int, k: int = 16) -> int:
    return int(lib().bitstack_block_bytes(out, inn, k))


def packed_bytes(out: int, inn: int, k: int, n: int, max_batch: int = 1) -> int:
    return int(lib().bitstack_packed_bytes(out, inn, k, n, max_batch))


def set_option(option: int, value: int):
    _check(lib().bitstack_set_option(option, value), "bitstack_set_option")


def probe_read(buf, sink, workgroups: int = 4096, stream=None):
    """bitstack_probe_read on a torch uint8 tensor."""
    import torch
    st = C.c_void_p((stream or torch.cuda.current_stream(buf.device)).cuda_stream)
    _check(lib().bitstack_probe_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), workgroups, st),
           "bitstack_probe_read")


def pack_signs_from_f32(residual: np.ndarray) -> np.ndarray:
    r = np.ascontiguousarray(residual, dtype=np.float32)
    out, inn = r.shape
    words = np.empty((out, max(inn // 32, 0)), dtype=np.uint32)
    _check(lib().bitstack_pack_signs_from_f32(out, inn, _ptr(r), _ptr(words)), "bitstack_pack_signs_from_f32")
    return words


def _canon(sign_words, U, V, s):
    sw = np.ascontiguousarray(sign_words, dtype=np.uint32)
    U = np.ascontiguousarray(U, dtype=np.float16)
    V = np.ascontiguousarray(V, dtype=np.float16)
    s = np.ascontiguousarray(s, dtype=np.float32)
    n, out, k = U.shape
    inn = V.shape[1]
    assert sw.shape == (n, out, inn // 32) and V.shape == (n, inn, k) and s.shape == (inn,)
    return sw, U, V, s, n, out, inn, k


def pack_image_host(sign_words, U, V, s, max_batch: int = 1) -> np.ndarray:
    sw, U, V, s, n, out, inn, k = _canon(sign_words, U, V, s)
    nbytes = packed_bytes(out, inn, k, n, max_batch)
    if nbytes == 0:
        raise BitStackError(-2, "bitstack_packed_bytes")
    img = np.empty(nbytes, dtype=np.uint8)
    _check(lib().bitstack_pack_image_host(out, inn, k, n, max_batch, _ptr(sw), _ptr(U), _ptr(V), _ptr(s),
                                          _ptr(img), nbytes), "bitstack_pack_image_host")
    return img


def dense_bytes(out: int, inn: int) -> int:
    return int(lib().bitstack_dense_bytes(out, inn))


def choose_kernel(out: int, inn: int, n_slots: int, max_batch: int, batch: int, n_loaded: int,
                  workspace_bytes: int = 0) -> int:
    rc = int(lib().bitstack_choose_kernel(out, inn, n_slots, max_batch, batch, n_loaded, workspace_bytes))
    if rc < 0:
        raise BitStackError(rc, "bitstack_choose_kernel")
    return rc


def decompose(W, s, n: int, k: int = 16, iterations: int = 0, stream=None):
    """bitstack_decompose: W is a device fp32 tensor [out][in], s a host array [in].  Returns device
    tensors (sign_words int32 [n][out][in/32], U fp16 [n][out][k], V fp16 [n][in][k])."""
    import torch
    out, inn = W.shape
    s = np.ascontiguousarray(s, dtype=np.float32)
    dev = W.device
    sw = torch.empty((n, out, inn // 32), dtype=torch.int32, device=dev)
    U = torch.empty((n, out, k), dtype=torch.float16, device=dev)
    V = torch.empty((n, inn, k), dtype=torch.float16, device=dev)
    nbytes = int(lib().bitstack_decompose_workspace_bytes(out, inn, k))
    if nbytes == 0:
        raise BitStackError(-2, "bitstack_decompose_workspace_bytes")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    _check(lib().bitstack_decompose(W.data_ptr(), _ptr(s), out, inn, k, n, iterations, sw.data_ptr(), U.data_ptr(),
                                    V.data_ptr(), ws.data_ptr(), nbytes, C.c_void_p(stream.cuda_stream)),
           "bitstack_decompose")
    stream.synchronize()   # the workspace is released when this function returns
    return sw, U, V


def order_check(slots, order) -> int:
    """bitstack_order_check (host only): 0 if `order` is a valid universal stack, else the error code."""
    sl = np.ascontiguousarray(slots, dtype=np.int32)
    od = np.ascontiguousarray(order, dtype=np.int32)
    return int(lib().bitstack_order_check(len(sl), _ptr(sl), _ptr(od), len(od)))


def budget_position(block_bytes_per_stack, order, budget: int):
    """bitstack_budget_position (host only) -> (position, bytes)."""
    bb = np.ascontiguousarray(block_bytes_per_stack, dtype=np.uint64)
    od = np.ascontiguousarray(order, dtype=np.int32)
    pos, tot = C.c_int(), C.c_size_t()
    _check(lib().bitstack_budget_position(len(bb), _ptr(bb), _ptr(od), len(od), int(budget), C.byref(pos), C.byref(tot)),
           "bitstack_budget_position")
    return pos.value, tot.value


class BlockManager:
    """bitstack_manager_*: empty stacks (PackedStack.empty), their blocks staged in pinned host
    memory, a universal stack, a byte budget."""

    def __init__(self, stacks):
        self.stacks = list(stacks)
        arr = (C.c_void_p * len(self.stacks))(*[ps.handle.value for ps in self.stacks])
        self._h = C.c_void_p()
        self._pinned = []
        _check(lib().bitstack_manager_create(len(self.stacks), arr, C.byref(self._h)), "bitstack_manager_create")

    def stage_block(self, stack: int, block: int, sign_words, U, V):
        import torch
        ps = self.stacks[stack]
        pinned = torch.empty(block_staging_bytes(ps.out, ps.inn, ps.k), dtype=torch.uint8, pin_memory=True)
        stage_block_host(sign_words, U, V, pinned.numpy())
        self._pinned.append(pinned)
        _check(lib().bitstack_manager_set_block(self._h, stack, block, pinned.data_ptr()), "bitstack_manager_set_block")

    def set_order(self, order):
        od = np.ascontiguousarray(order, dtype=np.int32)
        _check(lib().bitstack_manager_set_order(self._h, _ptr(od), len(od)), "bitstack_manager_set_order")

    def set_budget(self, budget: int, stream=None):
        """-> (blocks loaded, blocks offloaded)"""
        up, down = C.c_int(), C.c_int()
        _check(lib().bitstack_manager_set_budget(self._h, int(budget), self.stacks[0]._stream(stream), C.byref(up),
                                                 C.byref(down)), "bitstack_manager_set_budget")
        return up.value, down.value

    @property
    def position(self) -> int:
        return int(lib().bitstack_manager_position(self._h))

    @property
    def resident_bytes(self) -> int:
        return int(lib().bitstack_manager_resident_bytes(self._h))

    def n_loaded(self, stack: int) -> int:
        return int(lib().bitstack_manager_n_loaded(self._h, stack))

    def release(self):
        if self._h:
            lib().bitstack_manager_release(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass


def restore_max_blocks() -> int:
    return int(lib().bitstack_restore_max_blocks())


def block_staging_bytes(out: int, inn: int, k: int = 16) -> int:
    return int(lib().bitstack_block_staging_bytes(out, inn, k))


def stage_block_host(sign_words, U, V, staging: np.ndarray | None = None) -> np.ndarray:
    """bitstack_stage_block_host: one block (canonical words [out][in/32], U [out][k], V [in][k]) in
    device form, in `staging` (uint8 array, e.g. a view of pinned memory) or a new array."""
    sw = np.ascontiguousarray(sign_words, dtype=np.uint32)
    U = np.ascontiguousarray(U, dtype=np.float16)
    V = np.ascontiguousarray(V, dtype=np.float16)
    out, k = U.shape
    inn = V.shape[0]
    nbytes = block_staging_bytes(out, inn, k)
    if nbytes == 0:
        raise BitStackError(-2, "bitstack_block_staging_bytes")
    if staging is None:
        staging = np.empty(nbytes, dtype=np.uint8)
    _check(lib().bitstack_stage_block_host(out, inn, k, _ptr(sw), _ptr(U), _ptr(V), _ptr(staging), staging.nbytes),
           "bitstack_stage_block_host")
    return staging


def unpack_image_host(img: np.ndarray, out: int, inn: int, k: int, n: int, max_batch: int, block: int):
    sw = np.empty((out, inn // 32), dtype=np.uint32)
    U = np.empty((out, k), dtype=np.float16)
    V = np.empty((inn, k), dtype=np.float16)
    _check(lib().bitstack_unpack_image_host(out, inn, k, n, max_batch, _ptr(img), block, _ptr(sw), _ptr(U), _ptr(V)),
           "bitstack_unpack_image_host")
    return sw, U, V


class PackedStack:
    """A weight stack resident in device memory (a torch uint8 tensor owned here)."""

    def __init__(self, sign_words, U, V, s, max_batch: int = 1, device="cuda:0", stream=None):
        import torch
        sw, U, V, s, n, out, inn, k = _canon(sign_words, U, V, s)
        self.out, self.inn, self.k, self.n, self.max_batch = out, inn, k, n, max_batch
        nbytes = packed_bytes(out, inn, k, n, max_batch)
        if nbytes == 0:
            raise BitStackError(-2, "bitstack_packed_bytes")
        self.device = torch.device(device)
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        st = self._stream(stream)
        _check(lib().bitstack_pack_blocks(out, inn, k, n, max_batch, _ptr(sw), _ptr(U), _ptr(V), _ptr(s),
                                          self.buf.data_ptr(), nbytes, st, C.byref(self._h)),
               "bitstack_pack_blocks")

    @classmethod
    def empty(cls, out: int, inn: int, n_slots: int, s, k: int = 16, max_batch: int = 1, device="cuda:0", stream=None):
        """bitstack_create_stack: room for n_slots blocks, none loaded."""
        import torch
        self = cls.__new__(cls)
        s = np.ascontiguousarray(s, dtype=np.float32)
        self.out, self.inn, self.k, self.n, self.max_batch = out, inn, k, n_slots, max_batch
        nbytes = packed_bytes(out, inn, k, n_slots, max_batch)
        if nbytes == 0:
            raise BitStackError(-2, "bitstack_packed_bytes")
        self.device = torch.device(device)
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        self._staged = []
        _check(lib().bitstack_create_stack(out, inn, k, n_slots, max_batch, _ptr(s), self.buf.data_ptr(), nbytes,
                                           self._stream(stream), C.byref(self._h)), "bitstack_create_stack")
        return self

    @classmethod
    def from_dense(cls, W, s, n: int, k: int = 16, iterations: int = 0, max_batch: int = 1, stream=None):
        """Compress a device fp32 weight [out][in] into a packed stack without leaving the device:
        bitstack_create_stack, bitstack_decompose, bitstack_push_block_device per block."""
        out, inn = W.shape
        self = cls.empty(out, inn, n, s, k=k, max_batch=max_batch, device=W.device, stream=stream)
        sw, U, V = decompose(W, s, n, k=k, iterations=iterations, stream=stream)
        for i in range(n):
            self.push_block_device(sw[i], U[i], V[i], stream=stream)
        import torch
        (stream or torch.cuda.current_stream(W.device)).synchronize()   # sw, U, V are released on return
        return self

    def push_block(self, sign_words, U, V, stream=None):
        """Stages the block in pinned host memory (kept alive here) and enqueues its load."""
        import torch
        pinned = torch.empty(block_staging_bytes(self.out, self.inn, self.k), dtype=torch.uint8, pin_memory=True)
        stage_block_host(sign_words, U, V, pinned.numpy())
        _check(lib().bitstack_push_block(self._h, pinned.data_ptr(), self._stream(stream)), "bitstack_push_block")
        if not hasattr(self, "_staged"):
            self._staged = []
        self._staged.append(pinned)

    def push_block_device(self, sign_words, U, V, stream=None):
        """bitstack_push_block_device: one block from device tensors in the canonical layout."""
        _check(lib().bitstack_push_block_device(self._h, sign_words.data_ptr(), U.data_ptr(), V.data_ptr(),
                                                self._stream(stream)), "bitstack_push_block_device")

    def pop_block(self):
        _check(lib().bitstack_pop_block(self._h), "bitstack_pop_block")

    @property
    def resident_blocks(self) -> int:
        return int(lib().bitstack_resident_blocks(self._h))

    @property
    def resident_bytes(self) -> int:
        return int(lib().bitstack_resident_bytes(self._h))

    def _stream(self, stream):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        return C.c_void_p(stream.cuda_stream)

    @property
    def handle(self):
        return self._h

    @property
    def block_bytes(self) -> int:
        return block_bytes(self.out, self.inn, self.k)

    def unpack_block(self, block: int, stream=None):
        sw = np.empty((self.out, self.inn // 32), dtype=np.uint32)
        U = np.empty((self.out, self.k), dtype=np.float16)
        V = np.empty((self.inn, self.k), dtype=np.float16)
        _check(lib().bitstack_unpack_blocks(self._h, block, _ptr(sw), _ptr(U), _ptr(V), self._stream(stream)),
               "bitstack_unpack_blocks")
        return sw, U, V

    def linear(self, x, n_loaded: int, y=None, stream=None):
        """bitstack_linear: one token, fp16 in, fp16 out."""
        import torch
        if y is None:
            y = torch.empty(self.out, dtype=torch.float16, device=self.device)
        _check(lib().bitstack_linear(x.data_ptr(), self._h, n_loaded, y.data_ptr(), self._stream(stream)),
               "bitstack_linear")
        return y

    def linear_static(self, x, n_loaded: int, y=None, stream=None):
        """bitstack_linear_static: one token, workspace in the library's static device array."""
        import torch
        if y is None:
            y = torch.empty(self.out, dtype=torch.float16, device=self.device)
        _check(lib().bitstack_linear_static(x.data_ptr(), self._h, n_loaded, y.data_ptr(), self._stream(stream)),
               "bitstack_linear_static")
        return y

    def linear_batched(self, x, n_loaded: int, y=None, out_dtype=None, kernel: int = KERNEL_AUTO, stream=None):
        import torch
        batch = x.shape[0]
        out_dtype = out_dtype or (y.dtype if y is not None else torch.float16)
        if y is None:
            y = torch.empty((batch, self.out), dtype=out_dtype, device=self.device)
        yd = Y_F32 if out_dtype == torch.float32 else Y_F16
        _check(lib().bitstack_linear_select(x.data_ptr(), batch, self._h, n_loaded, y.data_ptr(), yd, kernel,
                                            self._stream(stream)), "bitstack_linear_select")
        return y

    def restore_weight(self, n_loaded: int, w_dense=None, stream=None):
        """bitstack_restore_weight: the loaded prefix as a dense fp16 [out][in] matrix (1/s folded in)."""
        import torch
        if w_dense is None:
            w_dense = torch.empty((self.out, self.inn), dtype=torch.float16, device=self.device)
        _check(lib().bitstack_restore_weight(self._h, n_loaded, w_dense.data_ptr(),
                                             w_dense.numel() * w_dense.element_size(), self._stream(stream)),
               "bitstack_restore_weight")
        return w_dense

    def _y_for(self, x, y, out_dtype):
        import torch
        out_dtype = out_dtype or (y.dtype if y is not None else torch.float16)
        if y is None:
            y = torch.empty((x.shape[0], self.out), dtype=out_dtype, device=self.device)
        return y, (Y_F32 if out_dtype == torch.float32 else Y_F16)

    def linear_dense(self, x, w_dense, y=None, out_dtype=None, stream=None):
        """bitstack_linear_dense: y = x w_dense^T with a weight restored earlier."""
        y, yd = self._y_for(x, y, out_dtype)
        _check(lib().bitstack_linear_dense(x.data_ptr(), x.shape[0], self._h, w_dense.data_ptr(), y.data_ptr(), yd,
                                           self._stream(stream)), "bitstack_linear_dense")
        return y

    def linear_materialised(self, x, n_loaded: int, w_dense, y=None, out_dtype=None, stream=None):
        """bitstack_linear_materialised: restore into w_dense, then the dense product."""
        y, yd = self._y_for(x, y, out_dtype)
        _check(lib().bitstack_linear_materialised(x.data_ptr(), x.shape[0], self._h, n_loaded, w_dense.data_ptr(),
                                                  w_dense.numel() * w_dense.element_size(), y.data_ptr(), yd,
                                                  self._stream(stream)), "bitstack_linear_materialised")
        return y

    def linear_batched_ws(self, x, n_loaded: int, workspace=None, y=None, out_dtype=None, stream=None):
        """bitstack_linear_batched_ws: kernel chosen by the library, scratch buffer optional."""
        y, yd = self._y_for(x, y, out_dtype)
        wp = workspace.data_ptr() if workspace is not None else None
        wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
        _check(lib().bitstack_linear_batched_ws(x.data_ptr(), x.shape[0], self._h, n_loaded, y.data_ptr(), yd, wp, wb,
                                                self._stream(stream)), "bitstack_linear_batched_ws")
        return y

    def release(self):
        if self._h:
            lib().bitstack_release(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass
