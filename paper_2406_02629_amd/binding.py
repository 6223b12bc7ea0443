"""ctypes binding of libssnet.so (the C ABI of include/ssnet.h).

Argument marshalling only: every operation on share data runs in the HIP
kernels of the library.  torch supplies device memory (int64 tensors hold the
61-bit field elements) and the stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

from . import build as _build

P61 = (1 << 61) - 1
P45 = (1 << 45) - 55          # the prime of Sec. VII-A; served by the second library

WS_HEADER_BYTES = 65536      # SSNET_WS_HEADER_BYTES
OK, EINVAL, EPRIME, ESHARES, EID, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7
STATIC_SCRATCH_BYTES = 8 << 20   # SSNET_STATIC_SCRATCH_BYTES
DOM_SHARE, DOM_RESHARE, DOM_ZERO, DOM_MASK_E, DOM_MASK_ALPHA, DOM_MASK_ALPHAT, DOM_TRUNC_GEN = range(1, 8)

_u64, _sz, _int, _ptr = C.c_uint64, C.c_size_t, C.c_int, C.c_void_p

# name -> (restype, argtypes): every symbol include/ssnet.h declares
SIGNATURES = {
    "ssnet_create": (_int, [C.POINTER(_ptr), _int, _int, _u64, _int, _u64, _ptr]),
    "ssnet_destroy": (_int, [_ptr]),
    "ssnet_workspace_bytes_stream": (_sz, [_ptr, _sz]),
    "ssnet_workspace_bytes_linear": (_sz, [_ptr, _int, _int, _int]),
    "ssnet_workspace_bytes_conv": (_sz, [_ptr] + [_int] * 9),
    "ssnet_set_workspace": (_int, [_ptr, _ptr, _sz]),
    "ssnet_share": (_int, [_ptr, _ptr, _sz, _int, _u64, _ptr]),
    "ssnet_reconstruct": (_int, [_ptr, _ptr, _sz, C.POINTER(_int), _int, _int, _ptr]),
    "ssnet_linear_mod": (_int, [_ptr, _ptr, _ptr, _int, _int, _int, _ptr]),
    "ssnet_conv_mod": (_int, [_ptr, _ptr, _ptr] + [_int] * 9 + [_ptr]),
    "ssnet_packed_weight_bytes": (_sz, [_int, _int]),
    "ssnet_pack_weights_linear": (_int, [_ptr, _ptr, _int, _int, _ptr]),
    "ssnet_pack_weights_conv": (_int, [_ptr, _ptr, _int, _int, _ptr]),
    "ssnet_linear_mod_packed": (_int, [_ptr, _ptr, _ptr, _int, _int, _int, _ptr]),
    "ssnet_conv_mod_packed": (_int, [_ptr, _ptr, _ptr] + [_int] * 9 + [_ptr]),
    "ssnet_share_packed": (_int, [_ptr, _ptr, _int, _int, _int, _u64, _ptr, _ptr]),
    "ssnet_linear_mod_prepacked": (_int, [_ptr, _ptr, _ptr, _int, _int, _int, _ptr]),
    "ssnet_conv1x1_mod_prepacked": (_int, [_ptr, _ptr, _ptr, _int, _int, _int, _int, _ptr]),
    "ssnet_conv_planes_bytes": (_sz, [_int] * 4),
    "ssnet_share_planes": (_int, [_ptr, _ptr, _int, _int, _int, _int, _u64, _ptr, _ptr]),
    "ssnet_split_planes": (_int, [_ptr, _ptr, _int, _int, _int, _int, _ptr]),
    "ssnet_pack_weights_conv_taps": (_int, [_ptr, _ptr, _int, _int, _int, _int, _ptr]),
    "ssnet_conv_mod_planes": (_int, [_ptr, _ptr, _ptr] + [_int] * 9 + [_ptr]),
    "ssnet_product_bytes_linear": (_sz, [_ptr, _int, _int, _int]),
    "ssnet_product_bytes_conv": (_sz, [_ptr] + [_int] * 9),
    "ssnet_linear_product_prepacked": (_int, [_ptr, _ptr, _ptr, _int, _int, _int]),
    "ssnet_conv1x1_product_prepacked": (_int, [_ptr, _ptr, _ptr, _int, _int, _int, _int]),
    "ssnet_conv_product_planes": (_int, [_ptr, _ptr, _ptr] + [_int] * 9),
    "ssnet_degree_reduce": (_int, [_ptr, _ptr, _sz, _u64, _ptr]),
    "ssnet_degree_reduce_static": (_int, [_ptr, _ptr, _sz, _u64, _ptr]),
    "ssnet_truncate": (_int, [_ptr, _ptr, _sz, _u64, _ptr]),
    "ssnet_degree_reduce_truncate": (_int, [_ptr, _ptr, _sz, _u64, _ptr]),
    "ssnet_degree_reduce_truncate_reconstruct": (_int, [_ptr, _ptr, _sz, _u64, _ptr, C.POINTER(_int), _int, _ptr]),
    "ssnet_reduce_truncate_direct": (_int, [_ptr, _ptr, _sz, _u64, _ptr, C.POINTER(_int), _int, _ptr]),
    "ssnet_workspace_bytes_layer_tail": (_sz, [_ptr, _int, _int, _int]),
    "ssnet_layer_tail_message_plane": (_sz, [_ptr, _int, _int, _int]),
    "ssnet_reduce_truncate_relu": (_int, [_ptr, _ptr, _int, _int, _int, _u64, _ptr, _ptr, _ptr, _ptr]),
    "ssnet_reduce_truncate_relu_direct": (_int, [_ptr, _ptr, _int, _int, _int, _ptr, _ptr, _ptr, _ptr]),
    "ssnet_nonlinear_masks": (_int, [_ptr, _sz, _u64, _ptr, _ptr]),
    "ssnet_relu": (_int, [_ptr, _ptr, _ptr, _ptr, _sz, _ptr]),
    "ssnet_truncate_div": (_int, [_ptr, _ptr, _sz, _int, _u64, _ptr]),
    "ssnet_degree_reduce_truncate_div": (_int, [_ptr, _ptr, _sz, _int, _u64, _ptr]),
    "ssnet_pool_out_size": (_int, [_int, _int, _int, _int]),
    "ssnet_pool_masks": (_int, [_ptr, _sz] + [_int] * 8 + [_u64, _ptr, _ptr]),
    "ssnet_relu_pool": (_int, [_ptr, _ptr, _ptr, _ptr, _sz] + [_int] * 9 + [_ptr]),
    "ssnet_field_prime": (_u64, []),
    "ssnet_rng_key": (_u64, [_u64] * 5),
    "ssnet_rng_draw": (_u64, [_u64, _u64]),
    "ssnet_rng_field": (_u64, [_u64, _u64]),
    "ssnet_host_lagrange": (_int, [_ptr, C.POINTER(_int), _int, C.POINTER(_u64)]),
    "ssnet_host_reduction_matrix": (_int, [_ptr, C.POINTER(_u64)]),
    "ssnet_profile_begin": (_int, [_ptr]),
    "ssnet_profile_begin_kernels": (_int, [_ptr]),
    "ssnet_profile_end": (_int, [_ptr, C.POINTER(C.c_double), C.POINTER(_u64)]),
    "ssnet_probe_planes": (_int, [_ptr, _ptr, _ptr, _sz, _int, _int, C.POINTER(C.c_double)]),
    "ssnet_probe_mfma_int8": (_int, [_ptr, _ptr, _int, _int, C.POINTER(C.c_double)]),
    "ssnet_strerror": (C.c_char_p, [_int]),
    "ssnet_last_hip_error": (_int, [_ptr]),
}

_libs = {}


def load_library(p: int = P61) -> C.CDLL:
    """Load the built library for the field F_p (any p other than P45 gets the default library, whose
    ssnet_create then rejects it); build first only if no library is there.
    There is no fallback: without the HIP library nothing here works."""
    path = _build.LIB_P45 if p == P45 else _build.LIB
    if path not in _libs:
        if not os.path.exists(path):
            _build.build(force=True)
        lib = C.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _libs[path] = lib
    return _libs[path]


class SSNetError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        msg = load_library().ssnet_strerror(code).decode()
        super().__init__(f"{where}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))
        self.code = code


def _dptr(t: torch.Tensor) -> int:
    return t.data_ptr()


def _check_i64(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.int64 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int64 tensor")
    return t


class SSNet:
    """One (k = t+1, n) scheme over F_p, p = 2^61-1 (or P45, served by the second library), fixed-point
    fraction bits f."""

    def __init__(self, n: int, t: int, f: int = 13, seed: int = 0, p: int = P61,
                 device: Optional[str] = "cuda:0", stream: Optional[int] = None):
        self.lib = load_library(p)
        self.n, self.t, self.k, self.f, self.p, self.seed = n, t, t + 1, f, p, seed
        self.device = None if device is None else torch.device(device)
        if stream is None and self.device is not None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        self._ctx = _ptr()
        rc = self.lib.ssnet_create(C.byref(self._ctx), n, t, p, f, seed, _ptr(stream or 0))
        if rc:
            self._ctx = None
            raise SSNetError(rc, "ssnet_create")
        self._ws: Optional[torch.Tensor] = None

    def close(self):
        if getattr(self, "_ctx", None):
            self.lib.ssnet_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ok(self, rc: int, where: str):
        if rc:
            raise SSNetError(rc, where, self.lib.ssnet_last_hip_error(self._ctx))

    # ---- workspace ----
    def reserve(self, nbytes: int):
        """Make the workspace at least nbytes large (allocates through torch)."""
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            self._ok(self.lib.ssnet_set_workspace(self._ctx, _dptr(self._ws), self._ws.numel()), "ssnet_set_workspace")

    def messages(self) -> torch.Tensor:
        """int64 view of the workspace behind its header: where the inter-party
        messages of the last degree_reduce / truncate call were written."""
        return self._ws[WS_HEADER_BYTES:(self._ws.numel() // 8) * 8].view(torch.int64)

    def workspace_bytes_stream(self, count: int) -> int:
        return self.lib.ssnet_workspace_bytes_stream(self._ctx, count)

    def workspace_bytes_linear(self, M: int, K: int, N: int) -> int:
        return self.lib.ssnet_workspace_bytes_linear(self._ctx, M, K, N)

    def workspace_bytes_conv(self, B, Ci, H, W, Co, kh, kw, stride, pad) -> int:
        return self.lib.ssnet_workspace_bytes_conv(self._ctx, B, Ci, H, W, Co, kh, kw, stride, pad)

    # ---- GEN / REC ----
    def share(self, secret: torch.Tensor, stream_id: int, degree: Optional[int] = None,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(secret, "secret")
        degree = self.t if degree is None else degree
        if out is None:
            out = torch.empty((self.n,) + tuple(secret.shape), dtype=torch.int64, device=secret.device)
        self._ok(self.lib.ssnet_share(self._ctx, _dptr(secret), secret.numel(), degree, stream_id, _dptr(out)),
                 "ssnet_share")
        return out

    def reconstruct(self, shares: torch.Tensor, ids: Sequence[int], degree: Optional[int] = None,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(shares, "shares")
        degree = self.t if degree is None else degree
        count = shares[0].numel()
        if out is None:
            out = torch.empty(tuple(shares.shape[1:]), dtype=torch.int64, device=shares.device)
        arr = (_int * len(ids))(*ids)
        self._ok(self.lib.ssnet_reconstruct(self._ctx, _dptr(shares), count, arr, len(ids), degree, _dptr(out)),
                 "ssnet_reconstruct")
        return out

    # ---- linear layers ----
    def linear_mod(self, x: torch.Tensor, w: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x"), _check_i64(w, "w")
        n, M, K = x.shape
        n2, K2, N = w.shape
        if n != self.n or n2 != self.n or K != K2:
            raise ValueError("shape mismatch")
        self.reserve(self.workspace_bytes_linear(M, K, N))
        if out is None:
            out = torch.empty((n, M, N), dtype=torch.int64, device=x.device)
        self._ok(self.lib.ssnet_linear_mod(self._ctx, _dptr(x), _dptr(w), M, K, N, _dptr(out)), "ssnet_linear_mod")
        return out

    def conv_mod(self, x: torch.Tensor, w: torch.Tensor, stride: int, pad: int,
                 out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x"), _check_i64(w, "w")
        n, B, Ci, H, W = x.shape
        n2, Co, Ci2, kh, kw = w.shape
        if n != self.n or n2 != self.n or Ci != Ci2:
            raise ValueError("shape mismatch")
        need = self.workspace_bytes_conv(B, Ci, H, W, Co, kh, kw, stride, pad)
        if need == 0:
            raise SSNetError(EINVAL, "ssnet_workspace_bytes_conv")
        self.reserve(need)
        Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        if out is None:
            out = torch.empty((n, B, Co, Ho, Wo), dtype=torch.int64, device=x.device)
        self._ok(self.lib.ssnet_conv_mod(self._ctx, _dptr(x), _dptr(w), B, Ci, H, W, Co, kh, kw, stride, pad,
                                         _dptr(out)), "ssnet_conv_mod")
        return out

    def pack_weights_linear(self, w: torch.Tensor) -> torch.Tensor:
        _check_i64(w, "w")
        n, K, N = w.shape
        packed = torch.empty(self.n * self.lib.ssnet_packed_weight_bytes(N, K), dtype=torch.uint8, device=w.device)
        self._ok(self.lib.ssnet_pack_weights_linear(self._ctx, _dptr(w), K, N, _dptr(packed)),
                 "ssnet_pack_weights_linear")
        return packed

    def pack_weights_conv(self, w: torch.Tensor) -> torch.Tensor:
        _check_i64(w, "w")
        n, Co, Ci, kh, kw = w.shape
        K = Ci * kh * kw
        packed = torch.empty(self.n * self.lib.ssnet_packed_weight_bytes(Co, K), dtype=torch.uint8, device=w.device)
        self._ok(self.lib.ssnet_pack_weights_conv(self._ctx, _dptr(w), Co, K, _dptr(packed)),
                 "ssnet_pack_weights_conv")
        return packed

    def linear_mod_packed(self, x: torch.Tensor, w_packed: torch.Tensor, N: int,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        n, M, K = x.shape
        self.reserve(self.workspace_bytes_linear(M, K, N))
        if out is None:
            out = torch.empty((n, M, N), dtype=torch.int64, device=x.device)
        self._ok(self.lib.ssnet_linear_mod_packed(self._ctx, _dptr(x), _dptr(w_packed), M, K, N, _dptr(out)),
                 "ssnet_linear_mod_packed")
        return out

    def share_packed(self, secret: torch.Tensor, stream_id: int, out: Optional[torch.Tensor] = None,
                     packed: Optional[torch.Tensor] = None):
        """secret [B][K][H][W] (conv input, 1x1 layer) or [M][K] (dense input)
        -> (shares [n][...], limb tiles of the shares as a GEMM operand)"""
        _check_i64(secret, "secret")
        if secret.dim() == 2:
            B, K, HW = secret.shape[0], secret.shape[1], 1
        elif secret.dim() == 4:
            B, K, HW = secret.shape[0], secret.shape[1], secret.shape[2] * secret.shape[3]
        else:
            raise SSNetError(EINVAL, "share_packed: secret must be [M][K] or [B][C][H][W]")
        if out is None:
            out = torch.empty((self.n,) + tuple(secret.shape), dtype=torch.int64, device=secret.device)
        nbytes = self.n * self.lib.ssnet_packed_weight_bytes(B * HW, K)
        if packed is None:
            packed = torch.empty(nbytes, dtype=torch.uint8, device=secret.device)
        elif packed.numel() * packed.element_size() < nbytes:
            raise SSNetError(EINVAL, "share_packed: packed buffer too small")
        self._ok(self.lib.ssnet_share_packed(self._ctx, _dptr(secret), B, K, HW, stream_id, _dptr(out), _dptr(packed)),
                 "ssnet_share_packed")
        return out, packed

    def linear_mod_prepacked(self, x_packed: torch.Tensor, w_packed: torch.Tensor, M: int, K: int, N: int,
                             out: Optional[torch.Tensor] = None) -> torch.Tensor:
        self.reserve(self.workspace_bytes_linear(M, K, N))
        if out is None:
            out = torch.empty((self.n, M, N), dtype=torch.int64, device=x_packed.device)
        self._ok(self.lib.ssnet_linear_mod_prepacked(self._ctx, _dptr(x_packed), _dptr(w_packed), M, K, N, _dptr(out)),
                 "ssnet_linear_mod_prepacked")
        return out

    def conv1x1_mod_prepacked(self, x_packed: torch.Tensor, w_packed: torch.Tensor, B: int, C: int, H: int, W: int,
                              Co: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        self.reserve(self.workspace_bytes_conv(B, C, H, W, Co, 1, 1, 1, 0))
        if out is None:
            out = torch.empty((self.n, B, Co, H, W), dtype=torch.int64, device=x_packed.device)
        self._ok(self.lib.ssnet_conv1x1_mod_prepacked(self._ctx, _dptr(x_packed), _dptr(w_packed), B, C, H * W, Co,
                                                      _dptr(out)), "ssnet_conv1x1_mod_prepacked")
        return out

    # ---- convolution on channel-innermost limb planes (no im2col matrix) ----
    def planes_supported(self, B: int, C: int, H: int, W: int) -> bool:
        return self.lib.ssnet_conv_planes_bytes(B, C, H, W) != 0

    def _planes_buffer(self, B, C, H, W, planes, device):
        nbytes = self.n * self.lib.ssnet_conv_planes_bytes(B, C, H, W)
        if nbytes == 0:
            raise SSNetError(EINVAL, "ssnet_conv_planes_bytes")
        if planes is None:
            planes = torch.empty(nbytes, dtype=torch.uint8, device=device)
        elif planes.numel() * planes.element_size() < nbytes:
            raise SSNetError(EINVAL, "planes buffer too small")
        return planes

    def share_planes(self, secret: torch.Tensor, stream_id: int, out: Optional[torch.Tensor] = None,
                     planes: Optional[torch.Tensor] = None):
        """secret [B][C][H][W] -> (shares [n][B][C][H][W], their limb planes)"""
        _check_i64(secret, "secret")
        B, C, H, W = secret.shape
        planes = self._planes_buffer(B, C, H, W, planes, secret.device)
        if out is None:
            out = torch.empty((self.n,) + tuple(secret.shape), dtype=torch.int64, device=secret.device)
        self._ok(self.lib.ssnet_share_planes(self._ctx, _dptr(secret), B, C, H, W, stream_id, _dptr(out), _dptr(planes)),
                 "ssnet_share_planes")
        return out, planes

    def split_planes(self, x: torch.Tensor, planes: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        n, B, C, H, W = x.shape
        planes = self._planes_buffer(B, C, H, W, planes, x.device)
        self._ok(self.lib.ssnet_split_planes(self._ctx, _dptr(x), B, C, H, W, _dptr(planes)), "ssnet_split_planes")
        return planes

    def pack_weights_conv_taps(self, w: torch.Tensor) -> torch.Tensor:
        _check_i64(w, "w")
        n, Co, C, kh, kw = w.shape
        packed = torch.empty(self.n * self.lib.ssnet_packed_weight_bytes(Co, C * kh * kw), dtype=torch.uint8,
                             device=w.device)
        self._ok(self.lib.ssnet_pack_weights_conv_taps(self._ctx, _dptr(w), Co, C, kh, kw, _dptr(packed)),
                 "ssnet_pack_weights_conv_taps")
        return packed

    def conv_mod_planes(self, planes: torch.Tensor, w_packed: torch.Tensor, B: int, C: int, H: int, W: int, Co: int,
                        kh: int, kw: int, stride: int, pad: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        need = self.workspace_bytes_conv(B, C, H, W, Co, kh, kw, stride, pad)
        if need == 0:
            raise SSNetError(EINVAL, "ssnet_workspace_bytes_conv")
        self.reserve(need)
        Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        if out is None:
            out = torch.empty((self.n, B, Co, Ho, Wo), dtype=torch.int64, device=planes.device)
        self._ok(self.lib.ssnet_conv_mod_planes(self._ctx, _dptr(planes), _dptr(w_packed), B, C, H, W, Co, kh, kw, stride,
                                                pad, _dptr(out)), "ssnet_conv_mod_planes")
        return out

    # ---- products left in the workspace for the reduction that follows (d_c = NULL there) ----
    def _reserve_product(self, product_bytes: int, B: int, C: int, HW: int):
        """room for the pending product plus the messages of whichever call consumes it"""
        if product_bytes == 0:
            raise SSNetError(EINVAL, "ssnet_product_bytes")
        msgs = max(self.workspace_bytes_stream(B * C * HW), self.lib.ssnet_workspace_bytes_layer_tail(self._ctx, B, C, HW))
        self.reserve(msgs + product_bytes)

    def linear_product_prepacked(self, x_packed: torch.Tensor, w_packed: torch.Tensor, M: int, K: int, N: int):
        self._reserve_product(self.lib.ssnet_product_bytes_linear(self._ctx, M, K, N), M, N, 1)
        self._ok(self.lib.ssnet_linear_product_prepacked(self._ctx, _dptr(x_packed), _dptr(w_packed), M, K, N),
                 "ssnet_linear_product_prepacked")

    def conv1x1_product_prepacked(self, x_packed: torch.Tensor, w_packed: torch.Tensor, B: int, C: int, H: int, W: int,
                                  Co: int):
        self._reserve_product(self.lib.ssnet_product_bytes_conv(self._ctx, B, C, H, W, Co, 1, 1, 1, 0), B, Co, H * W)
        self._ok(self.lib.ssnet_conv1x1_product_prepacked(self._ctx, _dptr(x_packed), _dptr(w_packed), B, C, H * W, Co),
                 "ssnet_conv1x1_product_prepacked")

    def conv_product_planes(self, planes: torch.Tensor, w_packed: torch.Tensor, B: int, C: int, H: int, W: int, Co: int,
                            kh: int, kw: int, stride: int, pad: int):
        Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        self._reserve_product(self.lib.ssnet_product_bytes_conv(self._ctx, B, C, H, W, Co, kh, kw, stride, pad), B, Co,
                              Ho * Wo)
        self._ok(self.lib.ssnet_conv_product_planes(self._ctx, _dptr(planes), _dptr(w_packed), B, C, H, W, Co, kh, kw,
                                                    stride, pad), "ssnet_conv_product_planes")

    def conv_mod_packed(self, x: torch.Tensor, w_packed: torch.Tensor, Co: int, kh: int, kw: int, stride: int,
                        pad: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        n, B, Ci, H, W = x.shape
        need = self.workspace_bytes_conv(B, Ci, H, W, Co, kh, kw, stride, pad)
        if need == 0:
            raise SSNetError(EINVAL, "ssnet_workspace_bytes_conv")
        self.reserve(need)
        Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        if out is None:
            out = torch.empty((n, B, Co, Ho, Wo), dtype=torch.int64, device=x.device)
        self._ok(self.lib.ssnet_conv_mod_packed(self._ctx, _dptr(x), _dptr(w_packed), B, Ci, H, W, Co, kh, kw, stride,
                                                pad, _dptr(out)), "ssnet_conv_mod_packed")
        return out

    # ---- RED + RERAND, truncation ----
    @staticmethod
    def _incoming(c: Optional[torch.Tensor], out: Optional[torch.Tensor]):
        """c = None stands for the pending product (d_c = NULL); `out` then gives the shape.
        -> (pointer or None, tensor of the shares' shape)"""
        if c is None:
            if out is None:
                raise TypeError("the pending product needs `out` for its shape")
            return None, _check_i64(out, "out")
        return _dptr(_check_i64(c, "c")), c

    def degree_reduce(self, c: Optional[torch.Tensor], stream_id: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        cp, c = self._incoming(c, out)
        count = c[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(c)
        self._ok(self.lib.ssnet_degree_reduce(self._ctx, cp, count, stream_id, _dptr(out)),
                 "ssnet_degree_reduce")
        return out

    def degree_reduce_static(self, c: torch.Tensor, stream_id: int, out: torch.Tensor) -> torch.Tensor:
        """ssnet_degree_reduce with the messages in the library's fixed device array: no workspace, and
        nothing is allocated here either (the caller brings `out`)."""
        _check_i64(c, "c")
        _check_i64(out, "out")
        self._ok(self.lib.ssnet_degree_reduce_static(self._ctx, _dptr(c), c[0].numel(), stream_id, _dptr(out)),
                 "ssnet_degree_reduce_static")
        return out

    def truncate(self, x: torch.Tensor, stream_id: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        count = x[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(x)
        self._ok(self.lib.ssnet_truncate(self._ctx, _dptr(x), count, stream_id, _dptr(out)), "ssnet_truncate")
        return out

    def degree_reduce_truncate(self, c: Optional[torch.Tensor], stream_id: int,
                               out: Optional[torch.Tensor] = None) -> torch.Tensor:
        cp, c = self._incoming(c, out)
        count = c[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(c)
        self._ok(self.lib.ssnet_degree_reduce_truncate(self._ctx, cp, count, stream_id, _dptr(out)),
                 "ssnet_degree_reduce_truncate")
        return out

    def truncate_div(self, x: torch.Tensor, kdiv: int, stream_id: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        count = x[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(x)
        self._ok(self.lib.ssnet_truncate_div(self._ctx, _dptr(x), count, kdiv, stream_id, _dptr(out)), "ssnet_truncate_div")
        return out

    def degree_reduce_truncate_div(self, c: Optional[torch.Tensor], kdiv: int, stream_id: int,
                                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
        cp, c = self._incoming(c, out)
        count = c[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(c)
        self._ok(self.lib.ssnet_degree_reduce_truncate_div(self._ctx, cp, count, kdiv, stream_id, _dptr(out)),
                 "ssnet_degree_reduce_truncate_div")
        return out

    def degree_reduce_truncate_reconstruct(self, c: Optional[torch.Tensor], stream_id: int, ids: Sequence[int],
                                           out: Optional[torch.Tensor] = None,
                                           secret: Optional[torch.Tensor] = None):
        """-> (truncated shares [n][...], their reconstruction from the parties `ids`)"""
        cp, c = self._incoming(c, out)
        count = c[0].numel()
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(c)
        if secret is None:
            secret = torch.empty(c.shape[1:], dtype=torch.int64, device=c.device)
        else:
            _check_i64(secret, "secret")
        arr = (_int * len(ids))(*ids)
        self._ok(self.lib.ssnet_degree_reduce_truncate_reconstruct(self._ctx, cp, count, stream_id, _dptr(out),
                                                                   arr, len(ids), _dptr(secret)),
                 "ssnet_degree_reduce_truncate_reconstruct")
        return out, secret

    # ---- live kernel timing ----
    def reduce_truncate_direct(self, c: torch.Tensor, stream_id: int, ids: Optional[Sequence[int]] = None,
                               out: Optional[torch.Tensor] = None, secret: Optional[torch.Tensor] = None):
        """-> (truncated shares, their reconstruction or None): the outputs of the protocol calls, no messages"""
        cp, c = self._incoming(c, out)
        count = c[0].numel()
        if out is None:
            out = torch.empty_like(c)
        if ids is not None and secret is None:
            secret = torch.empty(c.shape[1:], dtype=torch.int64, device=c.device)
        arr = (_int * len(ids))(*ids) if ids is not None else None
        self._ok(self.lib.ssnet_reduce_truncate_direct(self._ctx, cp, count, stream_id, _dptr(out), arr,
                                                       len(ids) if ids is not None else 0,
                                                       _dptr(secret) if secret is not None else None),
                 "ssnet_reduce_truncate_direct")
        return out, secret

    def reduce_truncate_relu(self, c: torch.Tensor, stream_id: int, beta: torch.Tensor, betainv: torch.Tensor,
                             out: Optional[torch.Tensor] = None, planes: Optional[torch.Tensor] = None,
                             want_planes: bool = False):
        """c [n][B][C][H][W] (or [n][B][C]) product shares -> (shares of ReLU(trunc(.)), limb planes or None)"""
        cp, c = self._incoming(c, out)
        n, B, C = c.shape[0], c.shape[1], c.shape[2]
        HW = c[0, 0, 0].numel()
        count = c[0].numel()
        if beta.numel() != c.numel() or betainv.numel() != c.numel():
            raise SSNetError(EINVAL, "reduce_truncate_relu: mask shares must have the shape of c")
        self.reserve(self.lib.ssnet_workspace_bytes_layer_tail(self._ctx, B, C, HW))
        if out is None:
            out = torch.empty_like(c)
        if want_planes and planes is None:
            planes = self._planes_buffer(B, C, HW, 1, None, c.device)
        self._ok(self.lib.ssnet_reduce_truncate_relu(self._ctx, cp, B, C, HW, stream_id, _dptr(beta), _dptr(betainv),
                                                     _dptr(out), _dptr(planes) if planes is not None else None),
                 "ssnet_reduce_truncate_relu")
        return out, planes

    def reduce_truncate_relu_direct(self, c: Optional[torch.Tensor], beta: torch.Tensor, betainv: torch.Tensor,
                                    out: Optional[torch.Tensor] = None, planes: Optional[torch.Tensor] = None,
                                    want_planes: bool = False):
        """the outputs of reduce_truncate_relu (shares, limb planes) in one pass without messages"""
        cp, c = self._incoming(c, out)
        B, C = c.shape[1], c.shape[2]
        HW = c[0, 0, 0].numel()
        if beta.numel() != c.numel() or betainv.numel() != c.numel():
            raise SSNetError(EINVAL, "reduce_truncate_relu_direct: mask shares must have the shape of c")
        if out is None:
            out = torch.empty_like(c)
        if want_planes and planes is None:
            planes = self._planes_buffer(B, C, HW, 1, None, c.device)
        self._ok(self.lib.ssnet_reduce_truncate_relu_direct(self._ctx, cp, B, C, HW, _dptr(beta), _dptr(betainv), _dptr(out),
                                                            _dptr(planes) if planes is not None else None),
                 "ssnet_reduce_truncate_relu_direct")
        return out, planes

    def nonlinear_masks(self, shape, stream_id: int, device=None):
        """-> (shares of beta, shares of beta^-1), each [n, *shape]; offline preprocessing"""
        shape = tuple(shape) if not isinstance(shape, int) else (shape,)
        device = device or self.device or "cuda"
        b = torch.empty((self.n,) + shape, dtype=torch.int64, device=device)
        bi = torch.empty_like(b)
        self._ok(self.lib.ssnet_nonlinear_masks(self._ctx, b[0].numel(), stream_id, _dptr(b), _dptr(bi)),
                 "ssnet_nonlinear_masks")
        return b, bi

    def relu(self, x: torch.Tensor, beta: torch.Tensor, betainv: torch.Tensor,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _check_i64(x, "x")
        _check_i64(beta, "beta")
        _check_i64(betainv, "betainv")
        count = x[0].numel()
        if beta.numel() != x.numel() or betainv.numel() != x.numel():
            raise SSNetError(EINVAL, "relu: mask shares must have the shape of x")
        self.reserve(self.workspace_bytes_stream(count))
        if out is None:
            out = torch.empty_like(x)
        self._ok(self.lib.ssnet_relu(self._ctx, _dptr(x), _dptr(beta), _dptr(betainv), count, _dptr(out)), "ssnet_relu")
        return out

    POOL_MAX, POOL_SUM = 0, 1

    def pool_out_size(self, H: int, k: int, s: int, pad: int) -> int:
        return self.lib.ssnet_pool_out_size(H, k, s, pad)

    def pool_masks(self, planes: int, H: int, W: int, kernel, stride, pad, stream_id: int, device=None):
        """-> (shares of beta [n, planes, H, W], shares of beta^-1 [n, planes, Ho, Wo]); offline preprocessing"""
        (kh, kw), (sh, sw), (ph, pw) = kernel, stride, pad
        Ho, Wo = self.pool_out_size(H, kh, sh, ph), self.pool_out_size(W, kw, sw, pw)
        if Ho < 1 or Wo < 1:
            raise SSNetError(EINVAL, "pool_masks: the pooling kernel does not fit the image")
        device = device or self.device or "cuda"
        b = torch.empty((self.n, planes, H, W), dtype=torch.int64, device=device)
        bi = torch.empty((self.n, planes, Ho, Wo), dtype=torch.int64, device=device)
        self._ok(self.lib.ssnet_pool_masks(self._ctx, planes, H, W, kh, kw, sh, sw, ph, pw, stream_id, _dptr(b), _dptr(bi)),
                 "ssnet_pool_masks")
        return b, bi

    def relu_pool(self, x: torch.Tensor, beta: torch.Tensor, betainv: torch.Tensor, kernel, stride, pad, mode: int,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """x [n, ..., H, W] -> shares of the pooled max(x, 0), [n, ..., Ho, Wo]"""
        _check_i64(x, "x")
        _check_i64(beta, "beta")
        _check_i64(betainv, "betainv")
        (kh, kw), (sh, sw), (ph, pw) = kernel, stride, pad
        H, W = x.shape[-2], x.shape[-1]
        planes = x[0].numel() // (H * W)
        Ho, Wo = self.pool_out_size(H, kh, sh, ph), self.pool_out_size(W, kw, sw, pw)
        if Ho < 1 or Wo < 1 or beta.numel() != x.numel() or betainv.numel() != self.n * planes * Ho * Wo:
            raise SSNetError(EINVAL, "relu_pool: mask shares do not fit x and the pooling kernel")
        self.reserve(self.workspace_bytes_stream(max(planes * H * W, planes * Ho * Wo)))
        if out is None:
            out = torch.empty(tuple(x.shape[:-2]) + (Ho, Wo), dtype=torch.int64, device=x.device)
        elif out.numel() != self.n * planes * Ho * Wo:
            raise SSNetError(EINVAL, "relu_pool: out has the wrong size")
        self._ok(self.lib.ssnet_relu_pool(self._ctx, _dptr(x), _dptr(beta), _dptr(betainv), planes, H, W, kh, kw, sh, sw,
                                          ph, pw, mode, _dptr(out)), "ssnet_relu_pool")
        return out

    PROF_CLASSES = ("share", "reconstruct", "pack_w", "pack_x", "gemm", "degree_reduce", "truncate", "nonlinear",
                    "gemm_kernel")   # gemm_kernel: the product kernels from their own start to their own end

    def profile_begin(self, kernels: bool = False):
        """kernels: also time every product kernel from its own start to its own end (class gemm_kernel)"""
        if kernels:
            self._ok(self.lib.ssnet_profile_begin_kernels(self._ctx), "ssnet_profile_begin_kernels")
        else:
            self._ok(self.lib.ssnet_profile_begin(self._ctx), "ssnet_profile_begin")

    def profile_end(self):
        """-> {class: (total_ms, spans)} for the calls since profile_begin"""
        ms = (C.c_double * len(self.PROF_CLASSES))()
        cnt = (_u64 * len(self.PROF_CLASSES))()
        self._ok(self.lib.ssnet_profile_end(self._ctx, ms, cnt), "ssnet_profile_end")
        return {name: (ms[i], cnt[i]) for i, name in enumerate(self.PROF_CLASSES)}

    # ---- host-side tables (no GPU needed) ----
    def host_lagrange(self, ids: Sequence[int]):
        arr = (_int * len(ids))(*ids)
        out = (_u64 * len(ids))()
        self._ok(self.lib.ssnet_host_lagrange(self._ctx, arr, len(ids), out), "ssnet_host_lagrange")
        return list(out)

    def host_reduction_matrix(self):
        nr = 2 * self.t + 1
        out = (_u64 * (nr * self.n))()
        self._ok(self.lib.ssnet_host_reduction_matrix(self._ctx, out), "ssnet_host_reduction_matrix")
        return [[out[i * self.n + m] for m in range(self.n)] for i in range(nr)]


def probe_planes(nbytes: int, planes: int, reps: int = 5, p: int = P61) -> float:
    """GB/s moved by `planes` streaming copies of nbytes (1: device copy; n: the traffic of GEN)"""
    lib = load_library(p)
    src = torch.zeros(nbytes // 8, dtype=torch.int64, device="cuda")
    dst = torch.empty(planes * (nbytes // 8), dtype=torch.int64, device="cuda")
    out = C.c_double()
    rc = lib.ssnet_probe_planes(_ptr(torch.cuda.current_stream().cuda_stream), _dptr(dst), _dptr(src), nbytes, planes, reps,
                                C.byref(out))
    if rc:
        raise SSNetError(rc, "ssnet_probe_planes")
    return out.value


def probe_mfma_int8(random_operands: bool = True, reps: int = 5, p: int = P61) -> float:
    """int8 TOP/s of a register-resident MFMA loop (two waves per SIMD)"""
    lib = load_library(p)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = C.c_double()
    rc = lib.ssnet_probe_mfma_int8(_ptr(torch.cuda.current_stream().cuda_stream), _dptr(sink), int(random_operands), reps,
                                   C.byref(out))
    if rc:
        raise SSNetError(rc, "ssnet_probe_mfma_int8")
    return out.value


def rng_key(seed, domain, stream_id, party, j) -> int:
    return load_library().ssnet_rng_key(seed, domain, stream_id, party, j)


def rng_draw(key, e) -> int:
    return load_library().ssnet_rng_draw(key, e)


def rng_field(key, e, p: int = P61) -> int:
    return load_library(p).ssnet_rng_field(key, e)
