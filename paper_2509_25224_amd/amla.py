"""ctypes binding of the C-ABI library (`include/amla.h`): argument marshalling only.

Every step of the decode path runs in the HIP kernels inside `libamla.so`; PyTorch is used
for device memory and the stream handle.  There is no CPU or PyTorch fallback: importing
this module raises if the library has not been built (run `__graft_entry__.build()`).
"""
from __future__ import annotations

import ctypes
import os

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libamla.so")

AMLA_OK = 0
AMLA_ERR_NULL_ARG = -1
AMLA_ERR_UNSUPPORTED = -2
AMLA_ERR_WORKSPACE = -3
AMLA_ERR_LAUNCH = -4
AMLA_RESCALE_MUL = 0
AMLA_RESCALE_ADD = 1
AMLA_RESCALE_ADD_COMP = 2
AMLA_RESCALE_ADD_LDEXP = 3
AMLA_FLAG_NO_SKIP = 1
AMLA_FLAG_LAZY_RESCALE = 2
AMLA_FLAG_BALANCED = 8
AMLA_FLAG_CAUSAL = 16
AMLA_FLAG_ITERATION_512 = 32
AMLA_FLAG_TRANSPOSED_ACC = 128

EXPORTS = ("amla_decode", "amla_decode_static_workspace", "amla_static_workspace_limit", "amla_workspace_bytes", "amla_effective_splits", "amla_exponent_add",
           "amla_mfma_probe", "amla_device_info", "amla_plan_segments", "amla_preload_rotation", "amla_status_string")


class AmlaDesc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("s_q", ctypes.c_int32), ("num_heads", ctypes.c_int32),
        ("d_qk", ctypes.c_int32), ("d_v", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("variant", ctypes.c_int32), ("num_splits", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("q_lens", ctypes.c_void_p),
    ]


if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build() "
                      "(hipcc --offload-arch=gfx950); there is no fallback path")

lib = ctypes.CDLL(_LIB_PATH)
lib.amla_decode.restype = ctypes.c_int
lib.amla_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                            ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(AmlaDesc)]
lib.amla_decode_static_workspace.restype = ctypes.c_int
lib.amla_decode_static_workspace.argtypes = lib.amla_decode.argtypes
lib.amla_static_workspace_limit.restype = ctypes.c_size_t
lib.amla_static_workspace_limit.argtypes = []
lib.amla_workspace_bytes.restype = ctypes.c_size_t
lib.amla_workspace_bytes.argtypes = [ctypes.POINTER(AmlaDesc)]
lib.amla_device_info.restype = ctypes.c_int
lib.amla_device_info.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
lib.amla_effective_splits.restype = ctypes.c_int
lib.amla_effective_splits.argtypes = [ctypes.POINTER(AmlaDesc)]
lib.amla_exponent_add.restype = ctypes.c_int
lib.amla_exponent_add.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                  ctypes.c_void_p]
lib.amla_mfma_probe.restype = ctypes.c_int
lib.amla_mfma_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
lib.amla_plan_segments.restype = ctypes.c_int
lib.amla_plan_segments.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                   ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
lib.amla_preload_rotation.restype = ctypes.c_int
lib.amla_preload_rotation.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32] + [ctypes.POINTER(ctypes.c_int32)] * 3
lib.amla_status_string.restype = ctypes.c_char_p
lib.amla_status_string.argtypes = [ctypes.c_int]


class AmlaError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"amla status {status}: {amla_status_string(status)}")


def amla_status_string(status: int) -> str:
    return lib.amla_status_string(int(status)).decode()


def make_desc(batch, s_q, num_heads, num_blocks, max_blocks_per_seq, variant=AMLA_RESCALE_ADD,
              num_splits=0, flags=0, d_qk=576, d_v=512, block_size=64) -> AmlaDesc:
    d = AmlaDesc()
    d.batch, d.s_q, d.num_heads = int(batch), int(s_q), int(num_heads)
    d.d_qk, d.d_v, d.block_size = int(d_qk), int(d_v), int(block_size)
    d.num_blocks, d.max_blocks_per_seq = int(num_blocks), int(max_blocks_per_seq)
    d.variant, d.num_splits, d.flags, d.reserved = int(variant), int(num_splits), int(flags), 0
    d.workspace, d.workspace_bytes, d.stream, d.q_lens = None, 0, None, None
    return d


def amla_workspace_bytes(desc: AmlaDesc) -> int:
    return int(lib.amla_workspace_bytes(ctypes.byref(desc)))


def amla_effective_splits(desc: AmlaDesc) -> int:
    return int(lib.amla_effective_splits(ctypes.byref(desc)))


def amla_decode(q, kv_cache, block_table, seqlens, softmax_scale, out=None, lse=None, *,
                variant=AMLA_RESCALE_ADD, num_splits=0, flags=0, workspace=None, want_lse=True, q_lens=None):
    """Decode attention on torch CUDA tensors.

    q bf16 [B, s_q, H, 576]; kv_cache bf16 [num_blocks, 64, 576]; block_table int32
    [B, max_blocks]; seqlens int32 [B].  Returns (out bf16 [B, s_q, H, 512], lse f32 [B, s_q, H]).
    `out`, `lse` and `workspace` (a uint8 tensor) are allocated with torch when not given.
    `q_lens` (int32 CUDA tensor [B], optional): query tokens each sequence really has.
    The call is enqueued on torch's current stream.
    """
    import torch

    for t, dt in ((q, torch.bfloat16), (kv_cache, torch.bfloat16), (block_table, torch.int32),
                  (seqlens, torch.int32)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dt):
            raise ValueError("inputs must be contiguous CUDA tensors of the documented dtypes")
    B, T, H, D = q.shape
    nblk, bs, D2 = kv_cache.shape
    if block_table.shape[0] != B or seqlens.shape[0] != B:
        raise ValueError("block_table / seqlens batch mismatch")
    if D2 != D:
        raise ValueError("q and kv_cache row widths differ")
    desc = make_desc(B, T, H, nblk, block_table.shape[1], variant, num_splits, flags, D, 512, bs)
    if q_lens is not None:
        if not (q_lens.is_cuda and q_lens.is_contiguous() and q_lens.dtype == torch.int32 and q_lens.shape == (B,)):
            raise ValueError("q_lens must be a contiguous int32 CUDA tensor of shape [batch]")
        desc.q_lens = q_lens.data_ptr()
    if out is None:
        out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, T, H), dtype=torch.float32, device=q.device)
    need = amla_workspace_bytes(desc)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if workspace is not None:
        desc.workspace = workspace.data_ptr()
        desc.workspace_bytes = workspace.numel() * workspace.element_size()
    desc.stream = torch.cuda.current_stream(q.device).cuda_stream
    st = lib.amla_decode(q.data_ptr(), kv_cache.data_ptr(), block_table.data_ptr(), seqlens.data_ptr(),
                         float(softmax_scale), out.data_ptr(), lse.data_ptr() if lse is not None else None,
                         ctypes.byref(desc))
    if st != AMLA_OK:
        raise AmlaError(st)
    return out, lse


def amla_decode_static_workspace(q, kv_cache, block_table, seqlens, softmax_scale, out, lse=None, *,
                                 variant=AMLA_RESCALE_ADD, num_splits=0, flags=0, q_lens=None):
    """amla_decode through the entry point that allocates nothing: `out` (and `lse` if wanted) are the
    caller's, and the partial results go to the library's static device array."""
    import torch

    B, T, H, D = q.shape
    nblk, bs, _ = kv_cache.shape
    desc = make_desc(B, T, H, nblk, block_table.shape[1], variant, num_splits, flags, D, 512, bs)
    if q_lens is not None:
        desc.q_lens = q_lens.data_ptr()
    desc.stream = torch.cuda.current_stream(q.device).cuda_stream
    st = lib.amla_decode_static_workspace(q.data_ptr(), kv_cache.data_ptr(), block_table.data_ptr(),
                                          seqlens.data_ptr(), float(softmax_scale), out.data_ptr(),
                                          lse.data_ptr() if lse is not None else None, ctypes.byref(desc))
    if st != AMLA_OK:
        raise AmlaError(st)
    return out, lse


def amla_static_workspace_limit() -> int:
    return int(lib.amla_static_workspace_limit())


def amla_exponent_add(x, delta: int, y=None):
    """y[i] = guarded exponent add of delta (<= 0) on float32 CUDA tensor x (Lemma 3.1)."""
    import torch

    if not (x.is_cuda and x.is_contiguous() and x.dtype == torch.float32):
        raise ValueError("x must be a contiguous float32 CUDA tensor")
    if y is None:
        y = torch.empty_like(x)
    st = lib.amla_exponent_add(x.data_ptr(), y.data_ptr(), x.numel(), int(delta),
                               torch.cuda.current_stream(x.device).cuda_stream)
    if st != AMLA_OK:
        raise AmlaError(st)
    return y


def amla_device_info():
    """(compute units, maximum engine clock in kHz) of the current device."""
    cus, khz = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib.amla_device_info(ctypes.byref(cus), ctypes.byref(khz))
    if st != AMLA_OK:
        raise AmlaError(st)
    return int(cus.value), int(khz.value)


def amla_mfma_probe(iters: int, workgroups: int) -> float:
    """Enqueue the register-resident MFMA loop on torch's current stream; returns its FLOP count."""
    import torch

    flops = ctypes.c_double(0.0)
    st = lib.amla_mfma_probe(int(iters), int(workgroups), ctypes.byref(flops),
                             torch.cuda.current_stream().cuda_stream)
    if st != AMLA_OK:
        raise AmlaError(st)
    return flops.value


def amla_plan_segments(seqlens, workers: int):
    """Host view of the balanced decomposition for the given lengths (any int sequence): returns
    (pieces int32 [n, 6]: worker, sequence, first block, end block, slot, full; seq_workers int32
    [batch, 2]: first and last worker meeting each sequence, -1 for an empty one)."""
    import numpy as np

    lens = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    batch = int(lens.shape[0])
    cap = int(workers) + batch
    pieces = np.zeros((cap, 6), dtype=np.int32)
    seq_workers = np.zeros((batch, 2), dtype=np.int32)
    n = ctypes.c_int32(0)
    st = lib.amla_plan_segments(lens.ctypes.data, batch, int(workers), pieces.ctypes.data, cap, ctypes.byref(n),
                                seq_workers.ctypes.data)
    if st != AMLA_OK:
        raise AmlaError(st)
    return pieces[:n.value].copy(), seq_workers


def amla_preload_rotation(cube, vec):
    """Cycle rotation of the Preload Pipeline for stage durations `cube`, `vec` (int sequences of equal
    length): returns (first matrix stage of the Cycle, pair whose C -> V edge crosses Cycles, Preload
    count), stage numbers 1-based."""
    import numpy as np

    c = np.ascontiguousarray(np.asarray(cube, dtype=np.int64))
    v = np.ascontiguousarray(np.asarray(vec, dtype=np.int64))
    if c.ndim != 1 or c.shape != v.shape:
        raise ValueError("cube and vec must be one-dimensional and of equal length")
    out = [ctypes.c_int32(0) for _ in range(3)]
    st = lib.amla_preload_rotation(c.ctypes.data, v.ctypes.data, int(c.shape[0]), *[ctypes.byref(o) for o in out])
    if st != AMLA_OK:
        raise AmlaError(st)
    return tuple(o.value for o in out)
