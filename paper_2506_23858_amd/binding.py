"""ctypes binding of libvmoba.so: same names as the C ABI in include/vmoba.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of the path runs
in the library's HIP kernels.  There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import struct

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvmoba.so")

VMOBA_OK = 0
VMOBA_ERR_INVALID_ARG, VMOBA_ERR_UNSUPPORTED, VMOBA_ERR_WORKSPACE = -1, -2, -3
VMOBA_ERR_CAPACITY, VMOBA_ERR_HIP = -4, -5
VMOBA_F32, VMOBA_BF16 = 0, 1
OP_SELECT, OP_ATTN_FWD, OP_ATTN_BWD = 1, 2, 3

EXPORTS = ["vmoba_layer_kind", "vmoba_partition_dims", "vmoba_workspace_bytes", "vmoba_status_string",
           "vmoba_partition", "vmoba_select", "vmoba_select_static", "vmoba_attn_fwd", "vmoba_attn_bwd",
           "vmoba_profile_events", "vmoba_probe_mfma", "vmoba_probe_atomic_rows"]


class vmoba_grid(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("bt", C.c_int32), ("bh", C.c_int32), ("bw", C.c_int32), ("chunk", C.c_int64)]


class vmoba_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32),
                ("stride_b", C.c_int64), ("stride_s", C.c_int64), ("stride_h", C.c_int64)]


class VmobaError(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        super().__init__(f"{fn} failed: {code} ({status_string(code)})")


_lib = None


def lib():
    """The loaded library.  Raises if libvmoba.so has not been built (python -m
    paper_2506_23858_amd.build, or __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2506_23858_amd.build)")
    L = C.CDLL(LIB_PATH)
    P = C.c_void_p
    L.vmoba_layer_kind.argtypes = [C.c_int]
    L.vmoba_layer_kind.restype = C.c_int
    L.vmoba_partition_dims.argtypes = [C.POINTER(vmoba_grid), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
    L.vmoba_partition_dims.restype = C.c_int
    L.vmoba_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int32, C.c_int64, C.c_int]
    L.vmoba_workspace_bytes.restype = C.c_size_t
    L.vmoba_status_string.argtypes = [C.c_int]
    L.vmoba_status_string.restype = C.c_char_p
    L.vmoba_partition.argtypes = [C.POINTER(vmoba_grid), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor), P, P, P, P]
    L.vmoba_partition.restype = C.c_int
    L.vmoba_select.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int32, P,
                               C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor), C.c_float, C.c_float, C.c_int,
                               C.c_int32, P, P, P, P, P, P, P, P, C.c_int64, P, P, P, P, P, P, C.c_size_t, P]
    L.vmoba_select.restype = C.c_int
    L.vmoba_select_static.argtypes = L.vmoba_select.argtypes[:-3] + [P]      # no workspace pointer / size
    L.vmoba_select_static.restype = C.c_int
    L.vmoba_attn_fwd.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int32, P,
                                 C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor),
                                 P, P, P, P, C.c_int64, C.c_float, C.POINTER(vmoba_tensor), P, P, P, P, C.c_size_t, P]
    L.vmoba_attn_fwd.restype = C.c_int
    L.vmoba_attn_bwd.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int32, P,
                                 C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor),
                                 C.POINTER(vmoba_tensor), P, C.POINTER(vmoba_tensor),
                                 P, P, P, P, C.c_int64, C.c_float,
                                 C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor), C.POINTER(vmoba_tensor),
                                 P, P, P, P, C.c_size_t, P]
    L.vmoba_attn_bwd.restype = C.c_int
    L.vmoba_profile_events.argtypes = [C.c_int, P, P]
    L.vmoba_profile_events.restype = C.c_int
    L.vmoba_probe_mfma.argtypes = [C.c_int64, C.c_int, P, C.POINTER(C.c_double), P]
    L.vmoba_probe_mfma.restype = C.c_int
    L.vmoba_probe_atomic_rows.argtypes = [P, P, C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int, P]
    L.vmoba_probe_atomic_rows.restype = C.c_int
    _lib = L
    return L


def status_string(code: int) -> str:
    return lib().vmoba_status_string(int(code)).decode()


def _check(fn, rc):
    if rc != VMOBA_OK:
        raise VmobaError(fn, rc)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return VMOBA_F32
    if t.dtype == torch.bfloat16:
        return VMOBA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def tensor_desc(t: torch.Tensor) -> vmoba_tensor:
    """Descriptor of a 4-D tensor indexed (b, s, h, d) -- any strides with d contiguous."""
    assert t.dim() == 4 and t.stride(3) == 1, "expect a (b, s, h, d) view with contiguous d"
    return vmoba_tensor(t.data_ptr(), _dtype_code(t), t.stride(0), t.stride(1), t.stride(2))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def make_grid(T, H, W, bt=0, bh=0, bw=0, chunk=0) -> vmoba_grid:
    return vmoba_grid(T, H, W, bt, bh, bw, chunk)


# ------------------------------------------------------------------------------- host helpers
def vmoba_layer_kind(layer: int) -> int:
    return lib().vmoba_layer_kind(int(layer))


def vmoba_partition_dims(g: vmoba_grid):
    S, nb = C.c_int64(0), C.c_int32(0)
    _check("vmoba_partition_dims", lib().vmoba_partition_dims(C.byref(g), C.byref(S), C.byref(nb)))
    return S.value, nb.value


def vmoba_workspace_bytes(op, B, Hh, S, D, n_blocks, nnz_capacity, dtype) -> int:
    return lib().vmoba_workspace_bytes(op, B, Hh, S, D, n_blocks, nnz_capacity, dtype)


def nnz_capacity_for(S: int, n_blocks: int, tau: float) -> int:
    """Per-head list capacity (buffer sizing only): in exact arithmetic the selection keeps at most
    ceil(tau * S * N_b) pairs.  tau is taken as the float32 the library receives, and a margin covers
    the float32 rounding of P (rows sum to 1 within ~1e-6, so the pool can fall short of S by that
    fraction and the cut move by as much)."""
    n = S * n_blocks
    tau32 = struct.unpack("f", struct.pack("f", float(tau)))[0]
    return max(1, min(n, math.ceil(tau32 * n * (1.0 + 2.0 ** -18)) + 16))


def vmoba_profile_events(slot: int, start_event=None, stop_event=None):
    """start_event / stop_event: raw hipEvent_t handles (ints) or None."""
    _check("vmoba_profile_events", lib().vmoba_profile_events(
        int(slot), C.c_void_p(start_event) if start_event else None,
        C.c_void_p(stop_event) if stop_event else None))


def vmoba_probe_mfma(iters: int, workgroups: int, sink, stream=None) -> float:
    """Launches the matrix-rate probe; returns the FLOP count of the launch (time it with events)."""
    flop = C.c_double(0.0)
    _check("vmoba_probe_mfma", lib().vmoba_probe_mfma(int(iters), int(workgroups), _ptr(sink), C.byref(flop), _stream(stream)))
    return flop.value


def vmoba_probe_atomic_rows(dq, lists, cnt, S, runs, heads, stream=None):
    """dq: float32 [heads, S, 128] (zeroed); lists: int32 [n_lists, cnt] ascending rows."""
    _check("vmoba_probe_atomic_rows", lib().vmoba_probe_atomic_rows(_ptr(dq), _ptr(lists), int(lists.shape[0]), int(cnt),
                                                                     int(S), int(runs), int(heads), _stream(stream)))


# ------------------------------------------------------------------------------- entry points
def vmoba_partition(g, inverse, B, Hh, D, ins, outs, perm, inv_perm, blk_off, stream=None):
    """ins / outs: lists of (b, s, h, d) views."""
    n = len(ins)
    assert len(outs) == n
    arr_in = (vmoba_tensor * max(n, 1))(*[tensor_desc(t) for t in ins])
    arr_out = (vmoba_tensor * max(n, 1))(*[tensor_desc(t) for t in outs])
    rc = lib().vmoba_partition(C.byref(g), int(inverse), B, Hh, D, n, arr_in, arr_out,
                               _ptr(perm), _ptr(inv_perm), _ptr(blk_off), _stream(stream))
    _check("vmoba_partition", rc)


GLOBAL_THRESHOLD, LOCAL_TOPK, LOCAL_THRESHOLD, GLOBAL_TOPK, POOL_SOFTMAX_THRESHOLD = 0, 1, 2, 3, 4
SELECT_OWN_BLOCK = 0x100


def vmoba_select(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask,
                 blk_ptr, q_idx, row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status,
                 workspace, stream=None, query_pos=None, kv_rows=None):
    q, k = tensor_desc(Qp), tensor_desc(Kp)
    rc = lib().vmoba_select(B, Hh, S, D, n_blocks, _ptr(blk_off), C.byref(q), C.byref(k),
                            float(tau), float(score_scale), int(mode), int(topk), _ptr(Bmean), _ptr(P), _ptr(mask),
                            _ptr(blk_ptr), _ptr(q_idx), _ptr(row_ptr), _ptr(col_idx), _ptr(pair_pos),
                            int(nnz_capacity), _ptr(k_out), _ptr(theta_out), _ptr(dev_status), _ptr(query_pos),
                            _ptr(kv_rows), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check("vmoba_select", rc)


SELECT_STATIC_MAX_BYTES = 32 << 20


def vmoba_select_static(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask,
                        blk_ptr, q_idx, row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status,
                        stream=None, query_pos=None, kv_rows=None):
    """vmoba_select on the library's static scratch array (no workspace argument, nothing allocated)."""
    q, k = tensor_desc(Qp), tensor_desc(Kp)
    rc = lib().vmoba_select_static(B, Hh, S, D, n_blocks, _ptr(blk_off), C.byref(q), C.byref(k),
                                   float(tau), float(score_scale), int(mode), int(topk), _ptr(Bmean), _ptr(P),
                                   _ptr(mask), _ptr(blk_ptr), _ptr(q_idx), _ptr(row_ptr), _ptr(col_idx),
                                   _ptr(pair_pos), int(nnz_capacity), _ptr(k_out), _ptr(theta_out),
                                   _ptr(dev_status), _ptr(query_pos), _ptr(kv_rows), _stream(stream))
    _check("vmoba_select_static", rc)


def vmoba_attn_fwd(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, Vp, blk_ptr, q_idx, row_ptr, pair_pos,
                   nnz_capacity, softmax_scale, O, LSE, workspace, stream=None, out_rows=None, kv_rows=None):
    q, k, v, o = tensor_desc(Qp), tensor_desc(Kp), tensor_desc(Vp), tensor_desc(O)
    rc = lib().vmoba_attn_fwd(B, Hh, S, D, n_blocks, _ptr(blk_off), C.byref(q), C.byref(k), C.byref(v),
                              _ptr(blk_ptr), _ptr(q_idx), _ptr(row_ptr), _ptr(pair_pos), int(nnz_capacity),
                              float(softmax_scale), C.byref(o), _ptr(LSE), _ptr(out_rows), _ptr(kv_rows), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream(stream))
    _check("vmoba_attn_fwd", rc)


def vmoba_attn_bwd(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, Vp, O, LSE, dO, blk_ptr, q_idx, row_ptr,
                   pair_pos, nnz_capacity, softmax_scale, dQ, dK, dV, workspace, stream=None, rows=None, key_rows=None,
                   kv_rows=None):
    d = [tensor_desc(t) for t in (Qp, Kp, Vp, O, dO, dQ, dK, dV)]
    rc = lib().vmoba_attn_bwd(B, Hh, S, D, n_blocks, _ptr(blk_off), C.byref(d[0]), C.byref(d[1]), C.byref(d[2]),
                              C.byref(d[3]), _ptr(LSE), C.byref(d[4]), _ptr(blk_ptr), _ptr(q_idx),
                              _ptr(row_ptr), _ptr(pair_pos), int(nnz_capacity), float(softmax_scale),
                              C.byref(d[5]), C.byref(d[6]), C.byref(d[7]), _ptr(rows), _ptr(key_rows), _ptr(kv_rows),
                              _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream(stream))
    _check("vmoba_attn_bwd", rc)


# ------------------------------------------------------------------------------- buffer plan
class LayerPlan:
    """All device buffers of one layer geometry, allocated once (PyTorch is only the allocator).
    The methods call the C ABI in the order partition -> select -> attn_fwd -> attn_bwd ->
    inverse partition and allocate nothing.  With fused_io the attention calls read dO and write O,
    dQ, dK, dV in the caller's token order themselves (row map = perm): no partition of dO, no
    inverse partitions, and the block-order copies Op, dOp, dQp, dKp, dVp do not exist.
    With q_in_place (implies fused_io) only K and V are rearranged, as in the paper's Eq. 1: Q is read
    where the caller has it, a query's id is its token index everywhere (P, mask, lists, LSE), and O,
    dO, dQ need no row map at all; dK and dV go back through key_rows = perm.
    With kv_in_place (implies q_in_place) nothing is rearranged in memory at all: the partition call only
    builds the index arrays and every kernel finds key position k at row perm[k] of the caller's K and V."""

    def __init__(self, B, Hh, D, grid, block=(0, 0, 0), chunk=0, tau=0.25, dtype=torch.bfloat16,
                 device="cuda", score_scale=None, softmax_scale=None, need_bwd=True, mode=GLOBAL_THRESHOLD, topk=0,
                 fused_io=False, q_in_place=False, kv_in_place=False):
        T, H, W = grid
        self.kv_in_place = bool(kv_in_place)
        self.q_in_place = bool(q_in_place) or self.kv_in_place
        self.fused_io = bool(fused_io) or self.q_in_place
        fused_io = self.fused_io
        self.Qin = None
        self.g = make_grid(T, H, W, *block, chunk)
        self.B, self.Hh, self.D, self.tau, self.dtype, self.dev = B, Hh, D, float(tau), dtype, device
        self.S, self.nb = vmoba_partition_dims(self.g)
        self.score_scale = score_scale if score_scale is not None else 1.0 / math.sqrt(D)
        self.softmax_scale = softmax_scale if softmax_scale is not None else 1.0 / math.sqrt(D)
        self.mode, self.topk = int(mode), int(topk)
        base_mode = self.mode & ~SELECT_OWN_BLOCK
        if base_mode == GLOBAL_THRESHOLD:
            self.cap = nnz_capacity_for(self.S, self.nb, tau)
        elif base_mode in (LOCAL_THRESHOLD, POOL_SOFTMAX_THRESHOLD):   # no bound below the whole pool
            self.cap = self.S * self.nb
        else:
            self.cap = self.S * min(self.topk, self.nb)
        if self.mode & SELECT_OWN_BLOCK:
            self.cap = min(self.cap + self.S, self.S * self.nb)
        S, nb, BH, cap = self.S, self.nb, B * Hh, self.cap
        dc = VMOBA_BF16 if dtype == torch.bfloat16 else VMOBA_F32
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.perm = torch.empty(S, **i32)
        self.inv_perm = torch.empty(S, **i32)
        self.blk_off = torch.empty(nb + 1, **i32)

        def blk_tensor(dt=dtype):   # block-order storage [B, Hh, S, D], handed out as a (b, s, h, d) view
            return torch.empty(B, Hh, S, D, dtype=dt, device=device).permute(0, 2, 1, 3)

        self.Kp, self.Vp = (None, None) if self.kv_in_place else (blk_tensor() for _ in range(2))
        self.Qp = None if self.q_in_place else blk_tensor()
        self.Op = None if fused_io else blk_tensor()
        self.LSE = torch.empty(B, Hh, S, **f32)
        self.Bmean = torch.empty(B, Hh, nb, D, **f32)
        self.P = torch.empty(B, Hh, S, nb, **f32)
        self.words = (nb + 31) // 32
        self.mask = torch.empty(B, Hh, S, self.words, **i32)
        self.blk_ptr = torch.empty(BH, nb + 1, **i32)
        self.row_ptr = torch.empty(BH, S + 1, **i32)
        self.q_idx = torch.empty(BH * cap, **i32)
        self.col_idx = torch.empty(BH * cap, **i32)
        self.pair_pos = torch.empty(BH * cap, **i32)
        self.k_out = torch.empty(BH, dtype=torch.int64, device=device)
        self.theta = torch.empty(BH, **f32)
        self.dev_status = torch.zeros(1, **i32)
        n_sel = vmoba_workspace_bytes(OP_SELECT, B, Hh, S, D, nb, cap, dc)
        n_fwd = vmoba_workspace_bytes(OP_ATTN_FWD, B, Hh, S, D, nb, cap, dc)
        n_bwd = vmoba_workspace_bytes(OP_ATTN_BWD, B, Hh, S, D, nb, cap, dc) if need_bwd else 0
        self.ws_select = torch.empty(n_sel, dtype=torch.uint8, device=device)
        # forward partials are dead once O is merged, so forward and backward share one workspace
        self.ws_attn = torch.empty(max(n_fwd, n_bwd), dtype=torch.uint8, device=device)
        self.O = torch.empty(B, S, Hh, D, dtype=dtype, device=device)
        if need_bwd:
            if not fused_io:
                self.dOp, self.dQp, self.dKp, self.dVp = (blk_tensor() for _ in range(4))
            self.dQ, self.dK, self.dV = (torch.empty(B, S, Hh, D, dtype=dtype, device=device) for _ in range(3))

    # -- the hot path, one method per C-ABI call -------------------------------------------
    def partition(self, Q, K, V):
        if self.kv_in_place:         # index arrays only; the blocks of Eq. 1 are addressed where they lie
            self.Qin, self.Kp, self.Vp = Q, K, V
            vmoba_partition(self.g, 0, self.B, self.Hh, self.D, [], [], self.perm, self.inv_perm, self.blk_off)
            return
        if self.q_in_place:          # Eq. 1 as written: only the keys (and their values) are rearranged
            self.Qin = Q
            vmoba_partition(self.g, 0, self.B, self.Hh, self.D, [K, V], [self.Kp, self.Vp],
                            self.perm, self.inv_perm, self.blk_off)
            return
        vmoba_partition(self.g, 0, self.B, self.Hh, self.D, [Q, K, V], [self.Qp, self.Kp, self.Vp],
                        self.perm, self.inv_perm, self.blk_off)

    def _q(self):
        return self.Qin if self.q_in_place else self.Qp

    def select(self):
        vmoba_select(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self._q(), self.Kp, self.tau,
                     self.score_scale, self.mode, self.topk, self.Bmean, self.P, self.mask, self.blk_ptr, self.q_idx,
                     self.row_ptr, self.col_idx, self.pair_pos, self.cap, self.k_out, self.theta,
                     self.dev_status, self.ws_select, query_pos=self.inv_perm if self.q_in_place else None,
                     kv_rows=self.perm if self.kv_in_place else None)

    def attn_fwd(self):
        if self.q_in_place:
            vmoba_attn_fwd(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self.Qin, self.Kp, self.Vp,
                           self.blk_ptr, self.q_idx, self.row_ptr, self.pair_pos, self.cap, self.softmax_scale,
                           self.O, self.LSE, self.ws_attn, kv_rows=self.perm if self.kv_in_place else None)
            return
        vmoba_attn_fwd(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self.Qp, self.Kp, self.Vp,
                       self.blk_ptr, self.q_idx, self.row_ptr, self.pair_pos, self.cap, self.softmax_scale,
                       self.O if self.fused_io else self.Op, self.LSE, self.ws_attn,
                       out_rows=self.perm if self.fused_io else None)

    def unpartition_out(self):
        vmoba_partition(self.g, 1, self.B, self.Hh, self.D, [self.Op], [self.O], self.perm, None, None)

    def partition_dO(self, dO):
        vmoba_partition(self.g, 0, self.B, self.Hh, self.D, [dO], [self.dOp], self.perm, None, None)

    def attn_bwd(self, dO=None):
        """dO: the caller-layout gradient (fused_io only; otherwise partition_dO() has run)."""
        if self.q_in_place:
            vmoba_attn_bwd(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self.Qin, self.Kp, self.Vp,
                           self.O, self.LSE, dO, self.blk_ptr, self.q_idx, self.row_ptr, self.pair_pos,
                           self.cap, self.softmax_scale, self.dQ, self.dK, self.dV, self.ws_attn, key_rows=self.perm,
                           kv_rows=self.perm if self.kv_in_place else None)
            return
        if self.fused_io:
            vmoba_attn_bwd(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self.Qp, self.Kp, self.Vp,
                           self.O, self.LSE, dO, self.blk_ptr, self.q_idx, self.row_ptr, self.pair_pos,
                           self.cap, self.softmax_scale, self.dQ, self.dK, self.dV, self.ws_attn, rows=self.perm)
            return
        vmoba_attn_bwd(self.B, self.Hh, self.S, self.D, self.nb, self.blk_off, self.Qp, self.Kp, self.Vp,
                       self.Op, self.LSE, self.dOp, self.blk_ptr, self.q_idx, self.row_ptr, self.pair_pos,
                       self.cap, self.softmax_scale, self.dQp, self.dKp, self.dVp, self.ws_attn)

    def unpartition_grads(self):
        vmoba_partition(self.g, 1, self.B, self.Hh, self.D, [self.dQp, self.dKp, self.dVp],
                        [self.dQ, self.dK, self.dV], self.perm, None, None)

    def forward(self, Q, K, V):
        self.partition(Q, K, V)
        self.select()
        self.attn_fwd()
        if not self.fused_io:
            self.unpartition_out()
        return self.O

    def backward(self, dO):
        if self.fused_io:
            self.attn_bwd(dO)
            return self.dQ, self.dK, self.dV
        self.partition_dO(dO)
        self.attn_bwd()
        self.unpartition_grads()
        return self.dQ, self.dK, self.dV
