"""ctypes binding of libperq.so -- argument marshalling only; every step runs in the library.

Function names and argument order mirror include/perq.h.  Device buffers are PyTorch tensors
(PyTorch is used for device memory and streams, nothing else); host buffers are NumPy arrays.
There is no fallback: if the library is not built or cannot be loaded, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libperq.so")

PERQ_OK, PERQ_ERR_INVALID_ARG, PERQ_ERR_UNSUPPORTED, PERQ_ERR_LAUNCH, PERQ_ERR_INTERNAL = 0, 1, 2, 3, 4
PERQ_FMT_INT4_SYM_TOKEN, PERQ_FMT_MXFP4, PERQ_FMT_INT4_ASYM_TOKEN, PERQ_FMT_FP4_TOKEN = 0, 1, 2, 3
PERQ_FMT_FP4_TOKEN_AMAX7 = 4
PERQ_ALGO_AUTO, PERQ_ALGO_BUTTERFLY, PERQ_ALGO_MFMA = 0, 1, 2
FMT = {"int4": PERQ_FMT_INT4_SYM_TOKEN, "mxfp4": PERQ_FMT_MXFP4, "int4_asym": PERQ_FMT_INT4_ASYM_TOKEN,
       "fp4_token": PERQ_FMT_FP4_TOKEN, "fp4_token7": PERQ_FMT_FP4_TOKEN_AMAX7}
ALGO = {"auto": PERQ_ALGO_AUTO, "butterfly": PERQ_ALGO_BUTTERFLY, "mfma": PERQ_ALGO_MFMA}

EXPORTS = ["perq_status_string", "perq_colabs_mean_workspace_bytes", "perq_colabs_mean",
           "perq_massdiff_perm", "perq_perm_validate", "perq_permute_rotate_quant",
           "perq_permute_rotate_quant_algo", "perq_permute_rotate_f32", "perq_w4a4_gemm_ref",
           "perq_colabs_absmax", "perq_perm_sorted", "perq_perm_zigzag", "perq_block_diagnostics",
           "perq_hadamard_base", "perq_perm_random", "perq_w4a4_mxfp4_gemm_ref", "perq_perm_arrange",
           "perq_perm_gather_cost", "perq_schedule_set", "perq_reset_schedule", "perq_schedule_selftest",
           "perq_colabs_mean_static", "perq_quant_error", "perq_perm_prepared_bytes", "perq_perm_prepare",
           "perq_perm_prepared_validate", "perq_permute_rotate_quant_prepared"]

_lib = None


class PerqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


def load(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libperq.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise RuntimeError(f"{LIB_PATH} is not built; run paper_2601_22347_amd.build.build()")
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.perq_status_string.restype = ctypes.c_char_p
    lib.perq_status_string.argtypes = [ctypes.c_int]
    lib.perq_colabs_mean_workspace_bytes.restype = sz
    lib.perq_colabs_mean_workspace_bytes.argtypes = [i64, i32]
    lib.perq_colabs_mean.restype = ctypes.c_int
    lib.perq_colabs_mean.argtypes = [vp, i64, i32, i64, vp, vp, sz, vp]
    lib.perq_massdiff_perm.restype = ctypes.c_int
    lib.perq_massdiff_perm.argtypes = [vp, i32, i32, vp]
    lib.perq_perm_validate.restype = ctypes.c_int
    lib.perq_perm_validate.argtypes = [vp, i32]
    lib.perq_perm_arrange.restype = ctypes.c_int
    lib.perq_perm_arrange.argtypes = [vp, i32, i32, i32, vp]
    lib.perq_perm_gather_cost.restype = ctypes.c_int
    lib.perq_perm_gather_cost.argtypes = [vp, i32, i32, vp, vp]
    lib.perq_permute_rotate_quant.restype = ctypes.c_int
    lib.perq_permute_rotate_quant.argtypes = [vp, i64, i32, i64, vp, i32, ctypes.c_int, vp, vp, vp]
    lib.perq_permute_rotate_quant_algo.restype = ctypes.c_int
    lib.perq_permute_rotate_quant_algo.argtypes = [vp, i64, i32, i64, vp, i32, ctypes.c_int, ctypes.c_int,
                                                   vp, vp, vp]
    lib.perq_permute_rotate_f32.restype = ctypes.c_int
    lib.perq_permute_rotate_f32.argtypes = [vp, i64, i32, i64, vp, i32, ctypes.c_int, vp, vp]
    lib.perq_w4a4_gemm_ref.argtypes = [vp, vp, i64, vp, vp, i32, i32, vp, i64, vp]
    lib.perq_w4a4_gemm_ref.restype = ctypes.c_int
    lib.perq_w4a4_mxfp4_gemm_ref.argtypes = [vp, vp, i64, vp, vp, i32, i32, vp, i64, vp]
    lib.perq_w4a4_mxfp4_gemm_ref.restype = ctypes.c_int
    lib.perq_colabs_absmax.argtypes = [vp, i64, i32, i64, vp, vp, sz, vp]
    lib.perq_colabs_absmax.restype = ctypes.c_int
    lib.perq_perm_sorted.argtypes = [vp, i32, vp]
    lib.perq_perm_sorted.restype = ctypes.c_int
    lib.perq_perm_zigzag.argtypes = [vp, i32, i32, vp]
    lib.perq_perm_zigzag.restype = ctypes.c_int
    lib.perq_hadamard_base.argtypes = [i32, vp]
    lib.perq_hadamard_base.restype = ctypes.c_int
    lib.perq_perm_random.argtypes = [i32, ctypes.c_uint64, vp]
    lib.perq_perm_random.restype = ctypes.c_int
    lib.perq_block_diagnostics.argtypes = [vp, i64, i32, i64, vp, i32, vp, vp]
    lib.perq_block_diagnostics.restype = ctypes.c_int
    lib.perq_colabs_mean_static.argtypes = [vp, i64, i32, i64, vp, vp]
    lib.perq_colabs_mean_static.restype = ctypes.c_int
    lib.perq_quant_error.argtypes = [vp, i64, i32, vp, vp, ctypes.c_int, vp, vp]
    lib.perq_quant_error.restype = ctypes.c_int
    lib.perq_perm_prepared_bytes.argtypes = [i32]
    lib.perq_perm_prepared_bytes.restype = sz
    lib.perq_perm_prepare.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.perq_perm_prepare.restype = ctypes.c_int
    lib.perq_perm_prepared_validate.argtypes = [vp, vp, i32]
    lib.perq_perm_prepared_validate.restype = ctypes.c_int
    lib.perq_permute_rotate_quant_prepared.argtypes = [vp, i64, i32, i64, vp, vp, i32, ctypes.c_int, vp, vp, vp]
    lib.perq_permute_rotate_quant_prepared.restype = ctypes.c_int
    lib.perq_schedule_set.argtypes = [vp]
    lib.perq_schedule_set.restype = ctypes.c_int32
    lib.perq_reset_schedule.argtypes = [vp]
    lib.perq_reset_schedule.restype = ctypes.c_int
    lib.perq_schedule_selftest.argtypes = [i64, i32, i32, ctypes.c_uint64, i32]
    lib.perq_schedule_selftest.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().perq_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != PERQ_OK:
        raise PerqError(status, where)


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _check_x(x):
    import torch
    if not x.is_cuda or x.dim() != 2 or x.stride(1) != 1 or x.element_size() != 2:
        raise ValueError("x must be a 2-D CUDA tensor of 16-bit elements with unit column stride")
    if x.dtype not in (torch.bfloat16, torch.int16, torch.uint16):
        raise ValueError("x must hold bf16 values (dtype bfloat16, or int16/uint16 bit patterns)")
    return x.shape[0], x.shape[1], x.stride(0)


# ---- host entry points --------------------------------------------------------------------
def perq_massdiff_perm(colabs_mean: np.ndarray, b: int) -> np.ndarray:
    a = np.ascontiguousarray(colabs_mean, dtype=np.float32)
    perm = np.empty(a.shape[0], dtype=np.int32)
    st = load().perq_massdiff_perm(a.ctypes.data_as(ctypes.c_void_p), a.shape[0], int(b),
                                   perm.ctypes.data_as(ctypes.c_void_p))
    _check(st, "perq_massdiff_perm")
    return perm


def perq_perm_sorted(stat: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(stat, dtype=np.float32)
    perm = np.empty(a.shape[0], dtype=np.int32)
    _check(load().perq_perm_sorted(a.ctypes.data_as(ctypes.c_void_p), a.shape[0], perm.ctypes.data_as(ctypes.c_void_p)),
           "perq_perm_sorted")
    return perm


def perq_perm_random(d: int, seed: int) -> np.ndarray:
    """Reproducible random permutation of d channels (host)."""
    perm = np.empty(max(int(d), 1), dtype=np.int32)
    _check(load().perq_perm_random(int(d), int(seed) & ((1 << 64) - 1), perm.ctypes.data_as(ctypes.c_void_p)),
           "perq_perm_random")
    return perm[:max(int(d), 0)]


def perq_hadamard_base(m: int) -> np.ndarray:
    """The m x m base matrix (+-1, int8) of the non-power-of-two rotation."""
    out = np.empty((max(int(m), 1), max(int(m), 1)), dtype=np.int8)
    _check(load().perq_hadamard_base(int(m), out.ctypes.data_as(ctypes.c_void_p)), "perq_hadamard_base")
    return out


def perq_perm_zigzag(stat: np.ndarray, b: int) -> np.ndarray:
    a = np.ascontiguousarray(stat, dtype=np.float32)
    perm = np.empty(a.shape[0], dtype=np.int32)
    _check(load().perq_perm_zigzag(a.ctypes.data_as(ctypes.c_void_p), a.shape[0], int(b),
                                   perm.ctypes.data_as(ctypes.c_void_p)), "perq_perm_zigzag")
    return perm


def perq_perm_arrange(perm: np.ndarray, b: int, head: int = -1) -> np.ndarray:
    """perm with the channels of every block reordered for the kernel's LDS gather (same blocks);
    the first `head` positions of every block stay as given (-1: 64 for b >= 512, else 0)."""
    p = np.ascontiguousarray(perm, dtype=np.int32)
    out = np.empty_like(p)
    st = load().perq_perm_arrange(p.ctypes.data_as(ctypes.c_void_p), p.size, int(b), int(head),
                                  out.ctypes.data_as(ctypes.c_void_p))
    _check(st, "perq_perm_arrange")
    return out


def perq_perm_gather_cost(perm: np.ndarray, b: int):
    """(passes, reads) of the element-wise LDS gather for this permutation; passes == reads: conflict free."""
    p = np.ascontiguousarray(perm, dtype=np.int32)
    passes, reads = ctypes.c_int64(0), ctypes.c_int64(0)
    st = load().perq_perm_gather_cost(p.ctypes.data_as(ctypes.c_void_p), p.size, int(b), ctypes.byref(passes),
                                      ctypes.byref(reads))
    _check(st, "perq_perm_gather_cost")
    return passes.value, reads.value


def perq_perm_prepare(perm: np.ndarray, b: int):
    """(prepared uint8 [perq_perm_prepared_bytes(d)], passes_before, passes_after, reads): the permutation
    in the form the fused call's LDS staging wants it."""
    p = np.ascontiguousarray(perm, dtype=np.int32)
    lib = load()
    table = np.zeros(lib.perq_perm_prepared_bytes(p.size), dtype=np.uint8)
    pb, pa, rd = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    st = lib.perq_perm_prepare(p.ctypes.data_as(ctypes.c_void_p), p.size, int(b), table.ctypes.data_as(ctypes.c_void_p),
                               ctypes.byref(pb), ctypes.byref(pa), ctypes.byref(rd))
    _check(st, "perq_perm_prepare")
    return table, pb.value, pa.value, rd.value


def prepared_parts(prepared: np.ndarray, d: int):
    """(place of every position int32 [d], piece of the row in every slot uint16 [d/8], operand offsets in
    lane order uint16 [2][tiles][8][64][8]) of a prepared form."""
    raw = np.ascontiguousarray(prepared, dtype=np.uint8)
    at = 4 * d + d // 4
    tiles = (d + 4095) // 4096
    return (raw[:4 * d].view(np.int32), raw[4 * d:at].view(np.uint16),
            raw[at:at + 2 * tiles * 8192].view(np.uint16).reshape(2, tiles, 8, 64, 8))


def perq_perm_prepared_validate(prepared: np.ndarray, perm: np.ndarray) -> bool:
    p = np.ascontiguousarray(perm, dtype=np.int32)
    t = np.ascontiguousarray(prepared, dtype=np.uint8)
    if t.size != load().perq_perm_prepared_bytes(p.size):
        return False
    return load().perq_perm_prepared_validate(t.ctypes.data_as(ctypes.c_void_p), p.ctypes.data_as(ctypes.c_void_p),
                                              p.size) == PERQ_OK


def perq_perm_validate(perm: np.ndarray) -> bool:
    p = np.ascontiguousarray(perm, dtype=np.int32)
    return load().perq_perm_validate(p.ctypes.data_as(ctypes.c_void_p), p.shape[0]) == PERQ_OK


def perq_schedule_selftest(n_units: int, n_blocks: int, workers_per_block: int, seed: int = 0, launches: int = 1) -> int:
    """Status of the host model of the run-time row schedule (PERQ_OK: consistent)."""
    return load().perq_schedule_selftest(int(n_units), int(n_blocks), int(workers_per_block), int(seed), int(launches))


# ---- device entry points ------------------------------------------------------------------
def perq_schedule_set(stream=None) -> int:
    """Counter set of the run-time row schedule for launches on `stream`; -1: fixed split."""
    return load().perq_schedule_set(_stream_ptr(stream))


def perq_reset_schedule(stream=None) -> None:
    _check(load().perq_reset_schedule(_stream_ptr(stream)), "perq_reset_schedule")


def perq_colabs_mean(x, out=None, stream=None):
    """x: CUDA bf16 [M, d] -> CUDA float32 [d]."""
    import torch
    M, d, ldx = _check_x(x)
    lib = load()
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=x.device)
    nbytes = lib.perq_colabs_mean_workspace_bytes(M, d)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    st = lib.perq_colabs_mean(_dev_ptr(x), M, d, ldx, _dev_ptr(out), _dev_ptr(ws), nbytes, _stream_ptr(stream))
    _check(st, "perq_colabs_mean")
    return out


def perq_colabs_mean_static(x, out, stream=None):
    """x: CUDA bf16 [M, d], out: CUDA float32 [d] (caller's); the call allocates nothing."""
    M, d, ldx = _check_x(x)
    st = load().perq_colabs_mean_static(_dev_ptr(x), M, d, ldx, _dev_ptr(out), _stream_ptr(stream))
    _check(st, "perq_colabs_mean_static")
    return out


def perq_colabs_absmax(x, out=None, stream=None):
    """x: CUDA bf16 [M, d] -> CUDA float32 [d], max_k |x[k, i]|."""
    import torch
    M, d, ldx = _check_x(x)
    lib = load()
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=x.device)
    nbytes = lib.perq_colabs_mean_workspace_bytes(M, d)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    st = lib.perq_colabs_absmax(_dev_ptr(x), M, d, ldx, _dev_ptr(out), _dev_ptr(ws), nbytes, _stream_ptr(stream))
    _check(st, "perq_colabs_absmax")
    return out


def perq_block_diagnostics(x, perm, b: int, out=None, stream=None):
    """x: CUDA bf16 [T, d] -> CUDA float32 [T, 4] = (|x|_inf, |x|_1, max block l1 of xP, |xP R~|_inf)."""
    import torch
    T, d, ldx = _check_x(x)
    if out is None:
        out = torch.empty((T, 4), dtype=torch.float32, device=x.device)
    st = load().perq_block_diagnostics(_dev_ptr(x), T, d, ldx, _dev_ptr(perm), int(b), _dev_ptr(out), _stream_ptr(stream))
    _check(st, "perq_block_diagnostics")
    return out


def perq_quant_error(y, codes, scales, fmt: str, out=None, stream=None):
    """y: CUDA float32 [T, d]; codes, scales: outputs of perq_permute_rotate_quant for the same input ->
    CUDA float32 [T, 3] = (|y - Q(y)|_2, |y|_2, |y|_inf)."""
    import torch
    T, d = y.shape
    if out is None:
        out = torch.empty((T, 3), dtype=torch.float32, device=y.device)
    st = load().perq_quant_error(_dev_ptr(y), T, d, _dev_ptr(codes), _dev_ptr(scales), FMT[fmt], _dev_ptr(out),
                                 _stream_ptr(stream))
    _check(st, "perq_quant_error")
    return out


def alloc_outputs(T: int, d: int, fmt: str, device):
    import torch
    codes = torch.empty((T, d // 2), dtype=torch.uint8, device=device)
    if FMT[fmt] in (PERQ_FMT_INT4_SYM_TOKEN, PERQ_FMT_FP4_TOKEN, PERQ_FMT_FP4_TOKEN_AMAX7):
        scales = torch.empty(T, dtype=torch.float32, device=device)
    elif FMT[fmt] == PERQ_FMT_INT4_ASYM_TOKEN:
        scales = torch.empty((T, 2), dtype=torch.float32, device=device)      # (step, zero point)
    else:
        scales = torch.empty((T, d // 32), dtype=torch.uint8, device=device)
    return codes, scales


def perq_permute_rotate_quant(x, perm, b: int, fmt: str, codes=None, scales=None, stream=None,
                              algo: str = "auto", placement=None):
    """x: CUDA bf16 [T, d]; perm: CUDA int32 [d] or None; placement: CUDA uint8 copy of what
    perq_perm_prepare wrote for perm, or None.  Returns (codes, scales) tensors."""
    T, d, ldx = _check_x(x)
    if codes is None or scales is None:
        codes, scales = alloc_outputs(T, d, fmt, x.device)
    lib = load()
    if placement is not None:
        if algo != "auto":
            raise ValueError("a placement goes with algo='auto'")
        import torch
        if placement.dtype != torch.uint8 or not placement.is_contiguous() or \
                placement.numel() != lib.perq_perm_prepared_bytes(d):
            raise ValueError("placement: not the bytes perq_perm_prepare writes for rows of this width")
        st = lib.perq_permute_rotate_quant_prepared(_dev_ptr(x), T, d, ldx, _dev_ptr(perm), _dev_ptr(placement), int(b),
                                                    FMT[fmt], _dev_ptr(codes), _dev_ptr(scales), _stream_ptr(stream))
    elif algo == "auto":
        st = lib.perq_permute_rotate_quant(_dev_ptr(x), T, d, ldx, _dev_ptr(perm), int(b), FMT[fmt],
                                           _dev_ptr(codes), _dev_ptr(scales), _stream_ptr(stream))
    else:
        st = lib.perq_permute_rotate_quant_algo(_dev_ptr(x), T, d, ldx, _dev_ptr(perm), int(b), FMT[fmt],
                                                ALGO[algo], _dev_ptr(codes), _dev_ptr(scales),
                                                _stream_ptr(stream))
    _check(st, "perq_permute_rotate_quant")
    return codes, scales


def perq_permute_rotate_f32(x, perm, b: int, y=None, stream=None, algo: str = "auto"):
    """Test entry: pre-quantization values, CUDA float32 [T, d]."""
    import torch
    T, d, ldx = _check_x(x)
    if y is None:
        y = torch.empty((T, d), dtype=torch.float32, device=x.device)
    st = load().perq_permute_rotate_f32(_dev_ptr(x), T, d, ldx, _dev_ptr(perm), int(b), ALGO[algo],
                                        _dev_ptr(y), _stream_ptr(stream))
    _check(st, "perq_permute_rotate_f32")
    return y


def perq_w4a4_gemm_ref(a_codes, a_scales, w_codes, w_scales, out=None, stream=None):
    """out[t, n] = a_scales[t] * w_scales[n] * <a_codes[t], w_codes[n]> for symmetric INT4 operands
    (CUDA uint8 [T, d/2] / [N, d/2], float32 [T] / [N]); returns CUDA float32 [T, N]."""
    import torch
    T, N, d = a_codes.shape[0], w_codes.shape[0], a_codes.shape[1] * 2
    if w_codes.shape[1] * 2 != d or not a_codes.is_contiguous() or not w_codes.is_contiguous():
        raise ValueError("a_codes [T, d/2] and w_codes [N, d/2] must be contiguous with the same d")
    if out is None:
        out = torch.empty((T, N), dtype=torch.float32, device=a_codes.device)
    st = load().perq_w4a4_gemm_ref(_dev_ptr(a_codes), _dev_ptr(a_scales), T, _dev_ptr(w_codes), _dev_ptr(w_scales),
                                   N, d, _dev_ptr(out), out.stride(0) if T else N, _stream_ptr(stream))
    _check(st, "perq_w4a4_gemm_ref")
    return out


def perq_w4a4_mxfp4_gemm_ref(a_codes, a_scales, w_codes, w_scales, out=None, stream=None):
    """The same product for MXFP4 operands (CUDA uint8 codes [T, d/2] / [N, d/2], uint8 scale bytes
    [T, d/32] / [N, d/32]); returns CUDA float32 [T, N]."""
    import torch
    T, N, d = a_codes.shape[0], w_codes.shape[0], a_codes.shape[1] * 2
    if w_codes.shape[1] * 2 != d or not a_codes.is_contiguous() or not w_codes.is_contiguous():
        raise ValueError("a_codes [T, d/2] and w_codes [N, d/2] must be contiguous with the same d")
    if not a_scales.is_contiguous() or not w_scales.is_contiguous():
        raise ValueError("scale bytes must be contiguous")
    if out is None:
        out = torch.empty((T, N), dtype=torch.float32, device=a_codes.device)
    st = load().perq_w4a4_mxfp4_gemm_ref(_dev_ptr(a_codes), _dev_ptr(a_scales), T, _dev_ptr(w_codes),
                                         _dev_ptr(w_scales), N, d, _dev_ptr(out), out.stride(0) if T else N,
                                         _stream_ptr(stream))
    _check(st, "perq_w4a4_mxfp4_gemm_ref")
    return out


def placement_to_device(prepared: np.ndarray, device="cuda"):
    """prepared form of a permutation (NumPy uint8) -> CUDA uint8 tensor."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(prepared, dtype=np.uint8)).to(device)


def bits_to_device(bits: np.ndarray, device="cuda"):
    """uint16 bf16 bit patterns (NumPy) -> CUDA bfloat16 tensor with the same bits."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)
