"""Thin ctypes binding of libqadc.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/qadc.h) and
takes torch tensors that live on the GPU; torch is used for device memory and
for the current HIP stream, nothing else.  There is no fallback: if the HIP
library is missing or a call fails, an exception is raised.
"""

from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libqadc.so")

QADC_OK, QADC_EINVAL, QADC_ENOMEM, QADC_EHIP = 0, -1, -2, -3
QADC_MAX_R = 1024
QADC_MAX_INIT = 8192
QADC_QMIN_PER_TABLE, QADC_QMIN_GLOBAL = 0, 1
QADC_U8_4BIT, QADC_F32_4BIT, QADC_F32_8BIT, QADC_U8_8BIT, QADC_U8_6BIT = 0, 1, 2, 3, 4
QADC_WS_SCAN_TOPK, QADC_WS_SCAN_F32_4BIT, QADC_WS_SCAN_F32_8BIT, QADC_WS_SEARCH, QADC_WS_SCAN_U8_8BIT = 0, 1, 2, 3, 4
QADC_WS_SCAN_U8_6BIT = 5
(QADC_PROF_SCAN, QADC_PROF_MERGE, QADC_PROF_SEED, QADC_PROF_IVF_INDEX, QADC_PROF_IVF_TABLES,
 QADC_PROF_TABLES, QADC_PROF_QUANTIZE, QADC_PROF_PREPARE, QADC_PROF_ROTATE, QADC_PROF_IVF_SHARED) = range(10)
QADC_LAYOUT_STANDARD, QADC_LAYOUT_TRANSPOSED = 0, 1

EXPORTS = (
    "qadc_build_luts", "qadc_quantize_luts", "qadc_quantize_luts_8bit", "qadc_quantize_luts_6bit", "qadc_scan_topk", "qadc_search", "qadc_ivf_search",
    "qadc_ivf_workspace_bytes", "qadc_pq_encode", "qadc_pq_train", "qadc_rotate",
    "qadc_profile_enable", "qadc_profile_only", "qadc_profile_read", "qadc_workspace_bytes", "qadc_workspace_init",
    "qadc_last_error", "qadc_version", "qadc_packed_bytes", "qadc_pack_codes", "qadc_unpack_codes",
    "qadc_ivf_assign", "qadc_ivf_group_workspace_bytes", "qadc_ivf_group", "qadc_ivf_encode",
    "qadc_multi_index_cells", "qadc_multi_index_assign", "qadc_multi_index_workspace_bytes",
    "qadc_multi_index_probes", "qadc_multi_index_group_workspace_bytes", "qadc_multi_index_group",
    "qadc_multi_index_encode", "qadc_multi_index_slots", "qadc_search_static", "qadc_static_scratch_bytes",
)

_lib = None


class qadc_ivf_index(ctypes.Structure):
    """Mirror of the C struct: device pointers + shapes (include/qadc.h)."""
    _fields_ = [("coarse", ctypes.c_void_p), ("list_off", ctypes.c_void_p), ("codes", ctypes.c_void_p),
                ("ids", ctypes.c_void_p), ("codebooks", ctypes.c_void_p), ("d", ctypes.c_int),
                ("m", ctypes.c_int), ("K", ctypes.c_int), ("n", ctypes.c_int64),
                ("halves", ctypes.c_void_p), ("cell_ids", ctypes.c_void_p), ("Kh", ctypes.c_int)]


class QadcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"qadc error {code}: {msg}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Loads libqadc.so (built in-tree by paper_1704_07355_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise ImportError(f"{_SO} not found: run `python -m paper_1704_07355_amd.build` first")
        L = ctypes.CDLL(_SO)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.qadc_build_luts.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, vp]
        L.qadc_build_luts.restype = i32
        L.qadc_quantize_luts.argtypes = [vp, i32, i32, i32, vp, i64, vp, i32, i32, i32,
                                         vp, vp, vp, vp, vp]
        L.qadc_quantize_luts.restype = i32
        L.qadc_quantize_luts_8bit.argtypes = L.qadc_quantize_luts.argtypes
        L.qadc_quantize_luts_8bit.restype = i32
        L.qadc_quantize_luts_6bit.argtypes = L.qadc_quantize_luts.argtypes
        L.qadc_quantize_luts_6bit.restype = i32
        L.qadc_scan_topk.argtypes = [i32, vp, i64, i32, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        L.qadc_scan_topk.restype = i32
        L.qadc_search.argtypes = [vp, i32, i32, vp, i32, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        L.qadc_search.restype = i32
        L.qadc_search_static.argtypes = [vp, i32, i32, vp, i32, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp]
        L.qadc_search_static.restype = i32
        L.qadc_static_scratch_bytes.argtypes = []
        L.qadc_static_scratch_bytes.restype = sz
        L.qadc_ivf_search.argtypes = [ctypes.POINTER(qadc_ivf_index), vp, i32, i32, i32, i32, i32, i32,
                                      vp, vp, vp, vp, vp, vp, sz, vp]
        L.qadc_ivf_search.restype = i32
        L.qadc_ivf_workspace_bytes.argtypes = [ctypes.POINTER(qadc_ivf_index), i32, i32, i32]
        L.qadc_ivf_workspace_bytes.restype = sz
        L.qadc_pq_encode.argtypes = [vp, i32, i32, i32, vp, i64, vp, vp]
        L.qadc_pq_encode.restype = i32
        L.qadc_rotate.argtypes = [vp, i32, vp, i64, vp, vp]
        L.qadc_rotate.restype = i32
        L.qadc_pq_train.argtypes = [vp, i64, i32, i32, i32, vp, i32, vp, vp, sz, vp]
        L.qadc_pq_train.restype = i32
        L.qadc_profile_only.argtypes = [i32]
        L.qadc_profile_only.restype = i32
        L.qadc_profile_enable.argtypes = [i32]
        L.qadc_profile_enable.restype = i32
        L.qadc_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.qadc_profile_read.restype = i32
        L.qadc_workspace_bytes.argtypes = [i32, i64, i32, i32, i32]
        L.qadc_workspace_bytes.restype = sz
        L.qadc_workspace_init.argtypes = [vp, sz, vp]
        L.qadc_workspace_init.restype = i32
        L.qadc_packed_bytes.argtypes = [i64, i32, i32]
        L.qadc_packed_bytes.restype = sz
        L.qadc_pack_codes.argtypes = [vp, i64, i32, i32, vp, vp]
        L.qadc_pack_codes.restype = i32
        L.qadc_unpack_codes.argtypes = [vp, i64, i32, i32, vp, vp]
        L.qadc_unpack_codes.restype = i32
        L.qadc_ivf_assign.argtypes = [vp, i32, i32, vp, i64, vp, vp]
        L.qadc_ivf_assign.restype = i32
        L.qadc_ivf_group_workspace_bytes.argtypes = [i64, i32]
        L.qadc_ivf_group_workspace_bytes.restype = sz
        L.qadc_ivf_group.argtypes = [vp, i64, i32, vp, vp, vp, sz, vp]
        L.qadc_ivf_group.restype = i32
        L.qadc_ivf_encode.argtypes = [vp, i32, vp, i32, i32, vp, i64, vp, vp, i64, vp, vp]
        L.qadc_ivf_encode.restype = i32
        L.qadc_multi_index_cells.argtypes = [vp, i32, i32, vp, vp]
        L.qadc_multi_index_cells.restype = i32
        L.qadc_multi_index_assign.argtypes = [vp, i32, i32, vp, i64, vp, vp]
        L.qadc_multi_index_assign.restype = i32
        L.qadc_multi_index_workspace_bytes.argtypes = [i32, i32, i32]
        L.qadc_multi_index_workspace_bytes.restype = sz
        L.qadc_multi_index_probes.argtypes = [vp, i32, i32, vp, i32, i32, vp, vp, sz, vp]
        L.qadc_multi_index_probes.restype = i32
        L.qadc_multi_index_group_workspace_bytes.argtypes = [i64, i32]
        L.qadc_multi_index_group_workspace_bytes.restype = sz
        L.qadc_multi_index_group.argtypes = [vp, i64, i32, i64, vp, vp, vp, vp, vp, sz, vp]
        L.qadc_multi_index_group.restype = i32
        L.qadc_multi_index_encode.argtypes = [vp, i32, vp, i32, i32, vp, i64, vp, vp, i64, vp, vp]
        L.qadc_multi_index_encode.restype = i32
        L.qadc_multi_index_slots.argtypes = [vp, i64, vp, i64, vp, vp]
        L.qadc_multi_index_slots.restype = i32
        L.qadc_last_error.restype = ctypes.c_char_p
        L.qadc_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensor must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int):
    if rc != QADC_OK:
        raise QadcError(rc, lib().qadc_last_error().decode())


def qadc_version() -> str:
    return lib().qadc_version().decode()


def qadc_last_error() -> str:
    return lib().qadc_last_error().decode()


def qadc_workspace_bytes(call: int, n: int, m: int, nq: int, R: int) -> int:
    return int(lib().qadc_workspace_bytes(call, n, m, nq, R))


def qadc_workspace_init(workspace):
    """Clears a workspace tensor before its first use; returns it."""
    _check(lib().qadc_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream()))
    return workspace


def qadc_build_luts(codebooks, queries, base=None, out=None):
    """codebooks f32 [m][ksub][dsub], queries f32 [nq][d], base f32 [nq][d] | None -> f32 [nq][m][ksub]."""
    m, ksub, dsub = codebooks.shape
    nq, d = queries.shape
    if out is None:
        out = torch.empty((nq, m, ksub), dtype=torch.float32, device=queries.device)
    _check(lib().qadc_build_luts(_ptr(codebooks, torch.float32), d, m, ksub,
                                 _ptr(queries, torch.float32), _ptr(base, torch.float32), nq,
                                 _ptr(out, torch.float32), _stream()))
    return out


def qadc_quantize_luts(luts, init_codes, R, nbins=255, qmin_mode=QADC_QMIN_PER_TABLE, qmax_in=None):
    """luts f32 [nq][m][k] or [nq][ngroup][m][k], k = 16 (init_codes u8 [n_init][m/2] | None) or
    k = 256 (8-bit components, init_codes u8 [n_init][m] | None: qadc_quantize_luts_8bit) or k = 64
    (6-bit components, init_codes u8 [n_init][3m/4] | None: qadc_quantize_luts_6bit).

    Returns (qluts u8 like luts, bias f32 [nq][m], delta f32 [nq], qmax f32 [nq]).
    """
    if luts.dim() == 3:
        nq, m, k = luts.shape
        ngroup = 1
    else:
        nq, ngroup, m, k = luts.shape
    if k not in (16, 64, 256):
        raise ValueError("tables of 16, 64 or 256 entries expected")
    fn = {16: lib().qadc_quantize_luts, 64: lib().qadc_quantize_luts_6bit, 256: lib().qadc_quantize_luts_8bit}[k]
    dev = luts.device
    qluts = torch.empty(luts.shape, dtype=torch.uint8, device=dev)
    bias = torch.empty((nq, m), dtype=torch.float32, device=dev)
    delta = torch.empty((nq,), dtype=torch.float32, device=dev)
    qmax = torch.empty((nq,), dtype=torch.float32, device=dev)
    n_init = 0 if init_codes is None else init_codes.shape[0]
    _check(fn(_ptr(luts, torch.float32), nq, ngroup, m, _ptr(init_codes, torch.uint8), n_init,
              _ptr(qmax_in, torch.float32), R, nbins, qmin_mode,
              _ptr(qluts), _ptr(bias), _ptr(delta), _ptr(qmax), _stream()))
    return qluts, bias, delta, qmax


def qadc_quantize_luts_8bit(luts, init_codes, R, nbins=255, qmin_mode=QADC_QMIN_PER_TABLE, qmax_in=None):
    """qadc_quantize_luts for 256-entry tables: luts f32 [nq][m][256] or [nq][ngroup][m][256], init_codes
    u8 [n_init][m] | None."""
    if luts.shape[-1] != 256:
        raise ValueError("tables of 256 entries expected")
    return qadc_quantize_luts(luts, init_codes, R, nbins, qmin_mode, qmax_in)


def qadc_quantize_luts_6bit(luts, init_codes, R, nbins=255, qmin_mode=QADC_QMIN_PER_TABLE, qmax_in=None):
    """qadc_quantize_luts for 64-entry tables: luts f32 [nq][m][64] or [nq][ngroup][m][64], init_codes
    u8 [n_init][3m/4] | None."""
    if luts.shape[-1] != 64:
        raise ValueError("tables of 64 entries expected")
    return qadc_quantize_luts(luts, init_codes, R, nbins, qmin_mode, qmax_in)


def qadc_scan_topk(variant, codes, luts, R, nbins=255, workspace=None, out_idx=None, out_dist=None,
                   n=None):
    """codes u8 [n][row]; luts [nq][m][ksub] (u8 or f32 by variant) -> (idx i64-viewable u32 [nq][R], dist)."""
    nq, m, ksub = luts.shape
    if n is None:
        n = codes.shape[0]
    dev = luts.device
    want = torch.uint8 if variant in (QADC_U8_4BIT, QADC_U8_8BIT, QADC_U8_6BIT) else torch.float32
    if luts.dtype != want:
        raise ValueError(f"variant {variant} needs {want} tables")
    if out_idx is None:
        out_idx = torch.empty((nq, R), dtype=torch.int32, device=dev)  # bit pattern of uint32
    if out_dist is None:
        out_dist = torch.empty((nq, R), dtype=want, device=dev)
    need = qadc_workspace_bytes({QADC_U8_4BIT: QADC_WS_SCAN_TOPK, QADC_F32_4BIT: QADC_WS_SCAN_F32_4BIT,
                                 QADC_F32_8BIT: QADC_WS_SCAN_F32_8BIT,
                                 QADC_U8_8BIT: QADC_WS_SCAN_U8_8BIT,
                                 QADC_U8_6BIT: QADC_WS_SCAN_U8_6BIT}[variant], n, m, nq, R)
    if workspace is None:
        workspace = qadc_workspace_init(torch.empty((max(need, 256),), dtype=torch.uint8, device=dev))
    _check(lib().qadc_scan_topk(variant, _ptr(codes, torch.uint8), n, m, _ptr(luts), nq, R, nbins,
                                _ptr(out_idx), _ptr(out_dist), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream()))
    return out_idx, out_dist


def qadc_pq_encode(codebooks, x, out=None):
    """codebooks f32 [m][ksub][dsub], x f32 [n][d] -> codes u8 [n][m/2] (ksub 16), [n][3m/4] (ksub 64)
    or [n][m] (ksub 256)."""
    m, ksub, dsub = codebooks.shape
    n, d = x.shape
    row = m // 2 if ksub == 16 else 3 * m // 4 if ksub == 64 else m
    if out is None:
        out = torch.empty((n, row), dtype=torch.uint8, device=x.device)
    _check(lib().qadc_pq_encode(_ptr(codebooks, torch.float32), d, m, ksub, _ptr(x, torch.float32),
                                n, _ptr(out, torch.uint8), _stream()))
    return out


def qadc_rotate(rot, x, out=None):
    """rot f32 [d][d], x f32 [n][d] -> y f32 [n][d], y[i] = rot @ x[i]."""
    n, d = x.shape
    assert rot.shape == (d, d)
    if out is None:
        out = torch.empty((n, d), dtype=torch.float32, device=x.device)
    _check(lib().qadc_rotate(_ptr(rot, torch.float32), d, _ptr(x, torch.float32), n, _ptr(out, torch.float32),
                             _stream()))
    return out


def qadc_packed_bytes(n: int, m: int, layout: int) -> int:
    return int(lib().qadc_packed_bytes(n, m, layout))


def qadc_pack_codes(std_codes, layout, out=None):
    """std_codes u8 [n][m/2] -> the list in `layout`, flat u8 [qadc_packed_bytes(n, m, layout)]."""
    n, half = std_codes.shape
    if out is None:
        out = torch.empty((qadc_packed_bytes(n, 2 * half, layout),), dtype=torch.uint8, device=std_codes.device)
    _check(lib().qadc_pack_codes(_ptr(std_codes, torch.uint8), n, 2 * half, layout, _ptr(out, torch.uint8),
                                 _stream()))
    return out


def qadc_unpack_codes(packed, n, m, layout, out=None):
    """packed flat u8 (n codes in `layout`) -> std codes u8 [n][m/2]."""
    if out is None:
        out = torch.empty((n, m // 2), dtype=torch.uint8, device=packed.device)
    _check(lib().qadc_unpack_codes(_ptr(packed, torch.uint8), n, m, layout, _ptr(out, torch.uint8), _stream()))
    return out


def qadc_ivf_assign(coarse, x, out=None):
    """coarse f32 [K][d], x f32 [n][d] -> cells i32 [n]."""
    K, d = coarse.shape
    n = x.shape[0]
    assert x.shape[1] == d
    if out is None:
        out = torch.empty((n,), dtype=torch.int32, device=x.device)
    _check(lib().qadc_ivf_assign(_ptr(coarse, torch.float32), K, d, _ptr(x, torch.float32), n,
                                 _ptr(out, torch.int32), _stream()))
    return out


def qadc_multi_index_cells(halves, out=None):
    """halves f32 [2][K][d/2] -> the K*K cell centroids f32 [K*K][d], cell id = i*K + j."""
    _, K, dh = halves.shape
    if out is None:
        out = torch.empty((K * K, 2 * dh), dtype=torch.float32, device=halves.device)
    _check(lib().qadc_multi_index_cells(_ptr(halves, torch.float32), K, 2 * dh, _ptr(out, torch.float32),
                                        _stream()))
    return out


def qadc_multi_index_assign(halves, x, out=None):
    """halves f32 [2][K][d/2], x f32 [n][d] -> cells i32 [n]."""
    _, K, dh = halves.shape
    n = x.shape[0]
    assert x.shape[1] == 2 * dh
    if out is None:
        out = torch.empty((n,), dtype=torch.int32, device=x.device)
    _check(lib().qadc_multi_index_assign(_ptr(halves, torch.float32), K, 2 * dh, _ptr(x, torch.float32), n,
                                         _ptr(out, torch.int32), _stream()))
    return out


def qadc_multi_index_workspace_bytes(K: int, nq: int, nprobe: int) -> int:
    return int(lib().qadc_multi_index_workspace_bytes(K, nq, nprobe))


def qadc_multi_index_probes(halves, queries, nprobe, workspace=None, out=None):
    """halves f32 [2][K][d/2], queries f32 [nq][d] -> probes i32 [nq][nprobe]."""
    _, K, dh = halves.shape
    nq = queries.shape[0]
    assert queries.shape[1] == 2 * dh
    if workspace is None:
        workspace = torch.empty((max(16, qadc_multi_index_workspace_bytes(K, nq, nprobe)),), dtype=torch.uint8,
                                device=queries.device)
    if out is None:
        out = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device)
    _check(lib().qadc_multi_index_probes(_ptr(halves, torch.float32), K, 2 * dh, _ptr(queries, torch.float32), nq,
                                         nprobe, _ptr(out, torch.int32), _ptr(workspace, torch.uint8),
                                         workspace.numel(), _stream()))
    return out


def qadc_multi_index_group_workspace_bytes(n: int, K: int) -> int:
    return int(lib().qadc_multi_index_group_workspace_bytes(n, K))


def qadc_multi_index_group(cells, K, workspace=None):
    """cells i32 [n] (product cells of K half-centroids per half) -> (cell_ids u32-bits [L], list_off i64 [L+1],
    ids u32-bits [n_placed]): the lists of the occupied cells, ascending.  Reads L back from the device."""
    n = cells.shape[0]
    cap = min(n, K * K)
    dev = cells.device
    if workspace is None:
        workspace = torch.empty((max(16, qadc_multi_index_group_workspace_bytes(n, K)),), dtype=torch.uint8, device=dev)
    cell_ids = torch.zeros((max(cap, 1),), dtype=torch.int32, device=dev)
    list_off = torch.zeros((cap + 1,), dtype=torch.int64, device=dev)
    ids = torch.zeros((max(n, 1),), dtype=torch.int32, device=dev)
    n_lists = torch.zeros((1,), dtype=torch.int64, device=dev)
    _check(lib().qadc_multi_index_group(_ptr(cells, torch.int32), n, K, cap, _ptr(cell_ids, torch.int32),
                                        _ptr(list_off, torch.int64), _ptr(ids, torch.int32),
                                        _ptr(n_lists, torch.int64), _ptr(workspace, torch.uint8),
                                        workspace.numel(), _stream()))
    L = int(n_lists.item())
    list_off = list_off[:L + 1].clone()
    placed = int(list_off[L].item())
    return cell_ids[:L].clone(), list_off, ids[:placed].clone()


def qadc_multi_index_encode(halves, codebooks, x, cells, ids, out=None):
    """Residual codes in list order against the half-centroids: row p = enc(x[ids[p]] - (halves[0][c // K],
    halves[1][c % K])), c = cells[ids[p]]; u8 [len(ids)][m/2]."""
    _, K, dh = halves.shape
    m = codebooks.shape[0]
    n = x.shape[0]
    n_list = ids.shape[0]
    assert x.shape[1] == 2 * dh
    if out is None:
        out = torch.empty((n_list, m // 2), dtype=torch.uint8, device=x.device)
    _check(lib().qadc_multi_index_encode(_ptr(halves, torch.float32), K, _ptr(codebooks, torch.float32), 2 * dh, m,
                                         _ptr(x, torch.float32), n, _ptr(cells, torch.int32),
                                         _ptr(ids, torch.int32), n_list, _ptr(out, torch.uint8), _stream()))
    return out


def qadc_multi_index_slots(cell_ids, cells, out=None):
    """cell_ids u32-bits [L] ascending, cells i32 [...] -> list numbers i32 [...], -1 for cells without a list."""
    if out is None:
        out = torch.empty_like(cells)
    _check(lib().qadc_multi_index_slots(_ptr(cell_ids, torch.int32), cell_ids.numel(), _ptr(cells, torch.int32),
                                        cells.numel(), _ptr(out, torch.int32), _stream()))
    return out


def qadc_ivf_group_workspace_bytes(n: int, K: int) -> int:
    return int(lib().qadc_ivf_group_workspace_bytes(n, K))


def qadc_ivf_group(cells, K, workspace=None):
    """cells i32 [n] -> (list_off i64 [K+1], ids u32 [n]) as torch int64 / int32-typed-as-uint32 tensors.

    ids is returned as an int32 tensor holding the uint32 bit patterns (torch has no uint32 arithmetic).
    """
    n = cells.shape[0]
    if workspace is None:
        workspace = torch.empty((max(16, qadc_ivf_group_workspace_bytes(n, K)),), dtype=torch.uint8,
                                device=cells.device)
    list_off = torch.empty((K + 1,), dtype=torch.int64, device=cells.device)
    ids = torch.zeros((n,), dtype=torch.int32, device=cells.device)
    _check(lib().qadc_ivf_group(_ptr(cells, torch.int32), n, K, _ptr(list_off, torch.int64),
                                _ptr(ids, torch.int32), _ptr(workspace, torch.uint8), workspace.numel(),
                                _stream()))
    return list_off, ids


def qadc_ivf_encode(coarse, codebooks, x, cells, ids, out=None):
    """Residual codes in list order: row p = enc(x[ids[p]] - coarse[cells[ids[p]]]); u8 [len(ids)][m/2]."""
    K, d = coarse.shape
    m = codebooks.shape[0]
    n = x.shape[0]
    n_list = ids.shape[0]
    if out is None:
        out = torch.empty((n_list, m // 2), dtype=torch.uint8, device=x.device)
    _check(lib().qadc_ivf_encode(_ptr(coarse, torch.float32), K, _ptr(codebooks, torch.float32), d, m,
                                 _ptr(x, torch.float32), n, _ptr(cells, torch.int32), _ptr(ids, torch.int32),
                                 n_list, _ptr(out, torch.uint8), _stream()))
    return out


def qadc_profile_enable(on: bool) -> None:
    _check(lib().qadc_profile_enable(1 if on else 0))


def qadc_profile_only(which: int) -> None:
    """Profiling on for the kernels of one slot only; qadc_profile_enable(False) ends it."""
    _check(lib().qadc_profile_only(which))


def qadc_profile_read(which: int):
    """-> (total milliseconds, launches) of the named kernel since profiling was enabled."""
    ms, cnt = ctypes.c_double(0), ctypes.c_int64(0)
    _check(lib().qadc_profile_read(which, ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value


class IvfIndex:
    """Holds the tensors of an inverted index on the GPU and the C struct that points at them.

    coarse f32 [K][d], or None for a multi-index over its occupied cells: then `halves` f32 [2][Kh][d/2]
    and `cell_ids` u32-bits [K] (ascending product cell of every list) stand in for the centroids.
    """

    def __init__(self, coarse, list_off, codes, ids, codebooks, halves=None, cell_ids=None):
        m = codebooks.shape[0]
        if coarse is not None:
            K, d = coarse.shape
            hp, cp, Kh = None, None, 0
        else:
            assert halves is not None and cell_ids is not None
            _, Kh, dh = halves.shape
            K, d = cell_ids.numel(), 2 * dh
            hp, cp = _ptr(halves, torch.float32).value, _ptr(cell_ids, torch.int32).value
        assert codebooks.shape[1] == 16 and codes.shape[1] == m // 2
        assert list_off.dtype == torch.int64 and list_off.numel() == K + 1
        assert ids.dtype == torch.int32 or ids.dtype == torch.uint32
        self.tensors = (coarse, list_off, codes, ids, codebooks)  # keep alive
        self.half_tensors = (halves, cell_ids)
        self.c = qadc_ivf_index(_ptr(coarse, torch.float32).value if coarse is not None else None,
                                _ptr(list_off).value, _ptr(codes, torch.uint8).value, _ptr(ids).value,
                                _ptr(codebooks, torch.float32).value, d, m, K, codes.shape[0], hp, cp, Kh)
        self.d, self.m, self.K, self.n = d, m, K, codes.shape[0]


def qadc_ivf_workspace_bytes(index: IvfIndex, nq: int, nprobe: int, R: int) -> int:
    return int(lib().qadc_ivf_workspace_bytes(ctypes.byref(index.c), nq, nprobe, R))


def qadc_ivf_search(index: IvfIndex, queries, nprobe, R, init, nbins=255,
                    qmin_mode=QADC_QMIN_PER_TABLE, probes_in=None, workspace=None, debug=False):
    """-> (ids i32-bits-of-u32 [nq][R], dist u8 [nq][R][, probes i32 [nq][nprobe], qluts u8 [nq][nprobe][m][16]])."""
    nq = queries.shape[0]
    dev = queries.device
    out_ids = torch.empty((nq, R), dtype=torch.int32, device=dev)
    out_dist = torch.empty((nq, R), dtype=torch.uint8, device=dev)
    dbg_p = torch.empty((nq, nprobe), dtype=torch.int32, device=dev) if debug else None
    dbg_q = torch.empty((nq, nprobe, index.m, 16), dtype=torch.uint8, device=dev) if debug else None
    need = qadc_ivf_workspace_bytes(index, nq, nprobe, R)
    if workspace is None:
        workspace = qadc_workspace_init(torch.empty((max(need, 256),), dtype=torch.uint8, device=dev))
    _check(lib().qadc_ivf_search(ctypes.byref(index.c), _ptr(queries, torch.float32), nq, nprobe, R, init,
                                 nbins, qmin_mode, _ptr(probes_in, torch.int32), _ptr(out_ids),
                                 _ptr(out_dist), _ptr(dbg_p), _ptr(dbg_q), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()))
    if debug:
        return out_ids, out_dist, dbg_p, dbg_q
    return out_ids, out_dist


def qadc_pq_train(train, m, ksub, init_rows, iters):
    """train f32 [n][d], init_rows i64 [ksub] -> codebooks f32 [m][ksub][d/m] (Lloyd k-means per sub-space)."""
    n, d = train.shape
    cb = torch.empty((m, ksub, d // m), dtype=torch.float32, device=train.device)
    ws = torch.empty((n * m,), dtype=torch.uint8, device=train.device)
    _check(lib().qadc_pq_train(_ptr(train, torch.float32), n, d, m, ksub, _ptr(init_rows, torch.int64),
                               iters, _ptr(cb), _ptr(ws), ws.numel(), _stream()))
    return cb


def qadc_search(codebooks, queries, codes, R, init, nbins=255, qmin_mode=QADC_QMIN_PER_TABLE,
                workspace=None, out_idx=None, out_dist=None, qluts_out=None, n=None):
    """Whole exhaustive Quick ADC query path in one call -> (idx u32-bits [nq][R], dist u8 [nq][R])."""
    m, ksub, dsub = codebooks.shape
    nq, d = queries.shape
    if n is None:
        n = codes.shape[0]
    dev = queries.device
    if out_idx is None:
        out_idx = torch.empty((nq, R), dtype=torch.int32, device=dev)
    if out_dist is None:
        out_dist = torch.empty((nq, R), dtype=torch.uint8, device=dev)
    if workspace is None:
        need = qadc_workspace_bytes(QADC_WS_SEARCH, n, m, nq, R)
        workspace = qadc_workspace_init(torch.empty((max(need, 256),), dtype=torch.uint8, device=dev))
    _check(lib().qadc_search(_ptr(codebooks, torch.float32), d, m, _ptr(queries, torch.float32), nq,
                             _ptr(codes, torch.uint8), n, R, init, nbins, qmin_mode, _ptr(out_idx),
                             _ptr(out_dist), _ptr(qluts_out, torch.uint8), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream()))
    return out_idx, out_dist


def qadc_static_scratch_bytes() -> int:
    return int(lib().qadc_static_scratch_bytes())


def qadc_search_static(codebooks, queries, codes, R, init, out_idx, out_dist, nbins=255,
                       qmin_mode=QADC_QMIN_PER_TABLE, qluts_out=None, n=None):
    """qadc_search without a workspace and without any allocation: the caller passes the outputs
    (idx i32 [nq][R], dist u8 [nq][R]); the scratch is the library's static device array."""
    m, ksub, dsub = codebooks.shape
    nq, d = queries.shape
    if n is None:
        n = codes.shape[0]
    _check(lib().qadc_search_static(_ptr(codebooks, torch.float32), d, m, _ptr(queries, torch.float32), nq,
                                    _ptr(codes, torch.uint8), n, R, init, nbins, qmin_mode, _ptr(out_idx),
                                    _ptr(out_dist), _ptr(qluts_out, torch.uint8), _stream()))
    return out_idx, out_dist
