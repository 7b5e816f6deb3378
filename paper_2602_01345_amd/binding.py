"""ctypes binding of libnova.so: argument marshalling only.

Every step of the hot path runs in the HIP kernels behind the C ABI declared in
``include/nova.h``.  PyTorch is used for device memory (tensors) and the current
stream; nothing here computes.  The method names mirror the C entry points.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import torch

NOVA_F32, NOVA_BF16 = 0, 1
NOVA_INTERP_BILINEAR, NOVA_INTERP_NEAREST, NOVA_INTERP_BICUBIC = 0, 1, 2
STAGES = ("entropy", "select", "gather_ln", "qkv", "attention", "oproj", "ln2", "ffn1", "ffn2", "merge")
_HERE = os.path.dirname(os.path.abspath(__file__))


class NovaError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what} failed: {code}")
        self.code = code


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("dtype", "B", "N", "C", "heads", "ffn_mult", "kv_len", "kv_capacity", "k")]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("w_qkv", "b_qkv", "w_o", "b_o", "w_fc1", "b_fc1", "w_fc2", "b_fc2")]


class _Variant(C.Structure):
    _fields_ = [("gelu_tanh", C.c_int32), ("qk_norm", C.c_int32), ("qk_scale", C.c_void_p), ("ada", C.c_void_p),
                ("w_cq", C.c_void_p), ("b_cq", C.c_void_p), ("w_co", C.c_void_p), ("b_co", C.c_void_p),
                ("k_text", C.c_void_p), ("v_text", C.c_void_p), ("text_len", C.c_int32), ("text_capacity", C.c_int32)]


@dataclass
class BlockVariant:
    """nova_block_variant: tanh GELU, unit-length q/k with a per-head multiplier (fp32 [heads], device),
    per-image modulation and gates ([B, 6, C] in the activations' dtype, device)."""
    gelu_tanh: bool = False
    qk_scale: Optional[torch.Tensor] = None
    ada: Optional[torch.Tensor] = None
    # cross-attention sub-layer: "w_cq", "b_cq", "w_co", "b_co" and the condition tokens' projected keys /
    # values "k_text" [B, heads, capacity, dh], "v_text" [B, heads, dh, capacity] (pack_k_cache / pack_v_cache),
    # "text_len" (int)
    cross: Optional[Dict[str, object]] = None

    def c_struct(self) -> "_Variant":
        if self.qk_scale is not None:
            assert self.qk_scale.dtype == torch.float32
        v = _Variant(int(self.gelu_tanh), int(self.qk_scale is not None), _ptr(self.qk_scale), _ptr(self.ada))
        if self.cross is not None:
            c = self.cross
            v.w_cq, v.b_cq, v.w_co, v.b_co = (_ptr(c.get(n)) for n in ("w_cq", "b_cq", "w_co", "b_co"))
            v.k_text, v.v_text = _ptr(c["k_text"]), _ptr(c["v_text"])
            v.text_len, v.text_capacity = int(c["text_len"]), int(c["k_text"].shape[2])
        return v


@dataclass
class BlockShape:
    dtype: int
    B: int
    N: int
    C: int
    heads: int
    kv_len: int
    kv_capacity: int
    k: int
    ffn_mult: int = 4

    def c_struct(self) -> _Shape:
        return _Shape(self.dtype, self.B, self.N, self.C, self.heads, self.ffn_mult, self.kv_len,
                      self.kv_capacity, self.k)


def library_path() -> str:
    return os.path.join(_HERE, "libnova.so")


_LIB = None


def load_library() -> C.CDLL:
    """Loads libnova.so from the package directory; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2602_01345_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.nova_create.argtypes = [C.POINTER(vp), i32]
    lib.nova_destroy.argtypes = [vp]
    lib.nova_strerror.argtypes = [i32]
    lib.nova_strerror.restype = C.c_char_p
    lib.nova_workspace_bytes.argtypes = [C.POINTER(_Shape)]
    lib.nova_workspace_bytes.restype = C.c_size_t
    lib.nova_entropy.argtypes = [vp, vp, vp, i32, i64, i32, i32, i64, vp, vp]
    lib.nova_select.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.nova_entropy_bits.argtypes = [vp, vp, vp, i32, i64, i32, i32, vp, vp]
    lib.nova_entropy_bits.restype = i32
    lib.nova_head_entropy_workspace_bytes.argtypes = [i64, i32, i32]
    lib.nova_head_entropy_workspace_bytes.restype = C.c_size_t
    lib.nova_head_entropy.argtypes = [vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, vp, vp, C.c_size_t]
    lib.nova_head_entropy.restype = i32
    lib.nova_head_entropy_static.argtypes = [vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, vp]
    lib.nova_head_entropy_static.restype = i32
    lib.nova_pruned_block.argtypes = [vp, vp, C.POINTER(_Shape), C.POINTER(_Weights), vp, vp, vp, vp, vp, vp,
                                      C.c_size_t]
    lib.nova_pruned_block_variant.argtypes = [vp, vp, C.POINTER(_Shape), C.POINTER(_Weights), C.POINTER(_Variant),
                                              vp, vp, vp, vp, vp, vp, C.c_size_t]
    lib.nova_pruned_block_variant.restype = i32
    lib.nova_pruned_block_rows.argtypes = [vp, vp, C.POINTER(_Shape), C.POINTER(_Weights), C.POINTER(_Variant),
                                           vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t]
    lib.nova_pruned_block_rows.restype = i32
    lib.nova_merge_cache_rows.argtypes = [vp, vp, i32, i32] + [i32] * 7 + [vp] * 8
    lib.nova_merge_cache_rows.restype = i32
    lib.nova_merge_cache.argtypes = [vp, vp, i32] + [i32] * 7 + [vp] * 7
    lib.nova_merge_cache_interp.argtypes = [vp, vp, i32, i32] + [i32] * 7 + [vp] * 7
    lib.nova_merge_cache_interp.restype = i32
    lib.nova_profile_stages.argtypes = [vp, C.c_uint32]
    lib.nova_profile_collect.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.nova_activation_scale.argtypes = [C.POINTER(C.c_double), i32, i32, C.c_double, C.POINTER(i32)]
    lib.nova_scale_ratio.argtypes = [i32, i32, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]
    lib.nova_layer_ratio.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.nova_probe.argtypes = [vp, vp, i32, vp, vp, i64, i32, vp, C.POINTER(C.c_double)]
    lib.nova_probe.restype = i32
    lib.nova_profile_stages.restype = i32
    lib.nova_profile_collect.restype = i32
    for f in (lib.nova_create, lib.nova_destroy, lib.nova_entropy, lib.nova_select, lib.nova_pruned_block,
              lib.nova_merge_cache, lib.nova_activation_scale, lib.nova_scale_ratio, lib.nova_layer_ratio):
        f.restype = i32
    _LIB = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NOVA_F32
    if t.dtype == torch.bfloat16:
        return NOVA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def activation_scale(hbar: Sequence[float], t_est: int, alpha: float) -> int:
    """nova_activation_scale: t* (1-based) for the scale mean entropies seen so far, 0 if none (host only)."""
    lib = load_library()
    arr = (C.c_double * max(len(hbar), 1))(*[float(h) for h in hbar])
    out = C.c_int(0)
    rc = lib.nova_activation_scale(arr, len(hbar), int(t_est), float(alpha), C.byref(out))
    if rc != 0:
        raise NovaError(rc, "nova_activation_scale")
    return out.value


def scale_ratio(t: int, t_star: int, g_t: float, tau: float, lam: float) -> float:
    """nova_scale_ratio: the scale-linkage reduction ratio (host only)."""
    lib = load_library()
    out = C.c_double(0.0)
    rc = lib.nova_scale_ratio(int(t), int(t_star), float(g_t), float(tau), float(lam), C.byref(out))
    if rc != 0:
        raise NovaError(rc, "nova_scale_ratio")
    return out.value


class Nova:
    """Handle on one GPU's context; methods are the four C entry points."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the NOVA hot path has no CPU fallback")
        h = C.c_void_p()
        rc = self.lib.nova_create(C.byref(h), device)
        if rc != 0:
            raise NovaError(rc, "nova_create")
        self.ctx = h
        self.device = device

    def __del__(self):
        ctx = getattr(self, "ctx", None)
        if ctx:
            self.lib.nova_destroy(ctx)
            self.ctx = None

    def strerror(self, code: int) -> str:
        return self.lib.nova_strerror(code).decode()

    def _check(self, rc: int, what: str):
        if rc != 0:
            raise NovaError(rc, f"{what} ({self.strerror(rc)})")

    # -- instrumentation ------------------------------------------------------------
    def profile_stages(self, stages):
        mask = 0
        for st in stages:
            mask |= 1 << int(st)
        self._check(self.lib.nova_profile_stages(self.ctx, mask), "nova_profile_stages")

    def profile_collect(self, stage: int):
        ms, n = C.c_double(0.0), C.c_int64(0)
        self._check(self.lib.nova_profile_collect(self.ctx, int(stage), C.byref(ms), C.byref(n)),
                    "nova_profile_collect")
        return ms.value, n.value

    def probe(self, kind: int, src: Optional[torch.Tensor], dst: Optional[torch.Tensor], iters: int,
              sink: torch.Tensor) -> float:
        """nova_probe: launches one achievable-peak kernel; returns the bytes moved / flops done."""
        work = C.c_double(0.0)
        nbytes = 0 if src is None else src.numel() * src.element_size()
        rc = self.lib.nova_probe(self.ctx, _stream(), int(kind), _ptr(src), _ptr(dst), nbytes, int(iters),
                                 _ptr(sink), C.byref(work))
        self._check(rc, "nova_probe")
        return work.value

    # -- nova_layer_ratio -----------------------------------------------------------
    def layer_ratio(self, mean_entropy: torch.Tensor, entropy_sum: torch.Tensor, ratio_t: torch.Tensor, j: int,
                    N: int, ratio_tj: torch.Tensor, k_per_row: torch.Tensor):
        """Per-row layer-linkage ratio and keep counts of layer j (1-based); entropy_sum is updated in place."""
        B = mean_entropy.shape[0]
        assert k_per_row.dtype == torch.int32 and all(t.dtype == torch.float32 for t in
                                                      (mean_entropy, entropy_sum, ratio_t, ratio_tj))
        rc = self.lib.nova_layer_ratio(self.ctx, _stream(), _ptr(mean_entropy), _ptr(entropy_sum), _ptr(ratio_t),
                                       int(j), B, int(N), _ptr(ratio_tj), _ptr(k_per_row))
        self._check(rc, "nova_layer_ratio")

    # -- nova_entropy ---------------------------------------------------------------
    def entropy(self, logits: torch.Tensor, entropy: torch.Tensor, mean: Optional[torch.Tensor] = None):
        """logits [B, N, V] (f32|bf16) -> entropy [B, N] f32 (and mean [B] f32)."""
        B, N, V = logits.shape
        rc = self.lib.nova_entropy(self.ctx, _stream(), _ptr(logits), _dtype_code(logits), N, B, V,
                                   logits.stride(1), _ptr(entropy), _ptr(mean))
        self._check(rc, "nova_entropy")

    # -- nova_entropy_bits ----------------------------------------------------------
    def entropy_bits(self, bit_logits: torch.Tensor, entropy: torch.Tensor, mean: Optional[torch.Tensor] = None):
        """bit_logits [B, N, d, 2] (f32|bf16) -> entropy [B, N] f32 (and mean [B] f32)."""
        B, N, d, two = bit_logits.shape
        assert two == 2
        rc = self.lib.nova_entropy_bits(self.ctx, _stream(), _ptr(bit_logits), _dtype_code(bit_logits), N, B, d,
                                        _ptr(entropy), _ptr(mean))
        self._check(rc, "nova_entropy_bits")

    # -- nova_head_entropy ----------------------------------------------------------
    def head_entropy_workspace_bytes(self, rows_per_batch: int, batch: int, V: int) -> int:
        return int(self.lib.nova_head_entropy_workspace_bytes(rows_per_batch, batch, V))

    def head_entropy(self, hidden: torch.Tensor, w_head: torch.Tensor, b_head: Optional[torch.Tensor],
                     entropy: torch.Tensor, workspace: torch.Tensor, mean: Optional[torch.Tensor] = None):
        """hidden [B, N, C] bf16, w_head [V, C], b_head [V] or None -> entropy [B, N] f32 (and mean [B])."""
        B, N, Cc = hidden.shape
        V = w_head.shape[0]
        rc = self.lib.nova_head_entropy(self.ctx, _stream(), _ptr(hidden), _ptr(w_head), _ptr(b_head),
                                        _dtype_code(hidden), N, B, Cc, V, _ptr(entropy), _ptr(mean),
                                        _ptr(workspace), workspace.numel() * workspace.element_size())
        self._check(rc, "nova_head_entropy")

    def head_entropy_static(self, hidden: torch.Tensor, w_head: torch.Tensor, b_head: Optional[torch.Tensor],
                            entropy: torch.Tensor, mean: Optional[torch.Tensor] = None):
        """nova_head_entropy_static: as head_entropy, the partials in the library's static device scratch."""
        B, N, Cc = hidden.shape
        V = w_head.shape[0]
        rc = self.lib.nova_head_entropy_static(self.ctx, _stream(), _ptr(hidden), _ptr(w_head), _ptr(b_head),
                                               _dtype_code(hidden), N, B, Cc, V, _ptr(entropy), _ptr(mean))
        self._check(rc, "nova_head_entropy_static")

    # -- nova_select ----------------------------------------------------------------
    def select(self, entropy: torch.Tensor, k: int, kept_idx: torch.Tensor, keep_mask: torch.Tensor,
               k_per_row: Optional[torch.Tensor] = None):
        B, N = entropy.shape
        rc = self.lib.nova_select(self.ctx, _stream(), _ptr(entropy), B, N, k, _ptr(k_per_row),
                                  _ptr(kept_idx), _ptr(keep_mask))
        self._check(rc, "nova_select")

    # -- nova_pruned_block ----------------------------------------------------------
    def workspace_bytes(self, shape: BlockShape) -> int:
        s = shape.c_struct()
        return int(self.lib.nova_workspace_bytes(C.byref(s)))

    def pruned_block(self, shape: BlockShape, weights: Dict[str, Optional[torch.Tensor]], x: torch.Tensor,
                     kept_idx: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                     y_kept: torch.Tensor, workspace: torch.Tensor):
        s = shape.c_struct()
        w = _Weights(*[_ptr(weights.get(n)) for n, _ in _Weights._fields_])
        rc = self.lib.nova_pruned_block(self.ctx, _stream(), C.byref(s), C.byref(w), _ptr(x), _ptr(kept_idx),
                                        _ptr(k_cache), _ptr(v_cache), _ptr(y_kept), _ptr(workspace),
                                        workspace.numel() * workspace.element_size())
        self._check(rc, "nova_pruned_block")

    def pruned_block_variant(self, shape: BlockShape, weights: Dict[str, Optional[torch.Tensor]],
                             variant: Optional[BlockVariant], x: torch.Tensor, kept_idx: torch.Tensor,
                             k_cache: torch.Tensor, v_cache: torch.Tensor, y_kept: torch.Tensor,
                             workspace: torch.Tensor):
        s = shape.c_struct()
        w = _Weights(*[_ptr(weights.get(n)) for n, _ in _Weights._fields_])
        v = variant.c_struct() if variant is not None else None
        rc = self.lib.nova_pruned_block_variant(self.ctx, _stream(), C.byref(s), C.byref(w),
                                                C.byref(v) if v is not None else None, _ptr(x), _ptr(kept_idx),
                                                _ptr(k_cache), _ptr(v_cache), _ptr(y_kept), _ptr(workspace),
                                                workspace.numel() * workspace.element_size())
        self._check(rc, "nova_pruned_block_variant")

    def pruned_block_rows(self, shape: BlockShape, weights: Dict[str, Optional[torch.Tensor]],
                          variant: Optional[BlockVariant], k_per_row: Optional[torch.Tensor],
                          kv_len_per_row: Optional[torch.Tensor], kv_len_next: Optional[torch.Tensor],
                          x: torch.Tensor, kept_idx: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                          y_kept: torch.Tensor, workspace: torch.Tensor):
        """nova_pruned_block_rows: per-image keep counts / cache lengths as int32 device tensors [B]."""
        for t in (k_per_row, kv_len_per_row, kv_len_next):
            assert t is None or t.dtype == torch.int32
        s = shape.c_struct()
        w = _Weights(*[_ptr(weights.get(n)) for n, _ in _Weights._fields_])
        v = variant.c_struct() if variant is not None else None
        rc = self.lib.nova_pruned_block_rows(self.ctx, _stream(), C.byref(s), C.byref(w),
                                             C.byref(v) if v is not None else None, _ptr(k_per_row),
                                             _ptr(kv_len_per_row), _ptr(kv_len_next), _ptr(x), _ptr(kept_idx),
                                             _ptr(k_cache), _ptr(v_cache), _ptr(y_kept), _ptr(workspace),
                                             workspace.numel() * workspace.element_size())
        self._check(rc, "nova_pruned_block_rows")

    def merge_cache_rows(self, interp: int, h: int, w: int, hp: int, wp: int, k: int,
                         k_per_row: Optional[torch.Tensor], x: torch.Tensor, y_kept: Optional[torch.Tensor],
                         kept_idx: Optional[torch.Tensor], keep_mask: torch.Tensor,
                         cache_prev: Optional[torch.Tensor], out: torch.Tensor,
                         cache_new: Optional[torch.Tensor] = None):
        """nova_merge_cache_rows: k is the row pitch, k_per_row the per-image counts (int32 device [B])."""
        assert k_per_row is None or k_per_row.dtype == torch.int32
        B, _, Cc = x.shape
        rc = self.lib.nova_merge_cache_rows(self.ctx, _stream(), _dtype_code(x), interp, B, Cc, h, w, hp, wp, k,
                                            _ptr(k_per_row), _ptr(x), _ptr(y_kept), _ptr(kept_idx), _ptr(keep_mask),
                                            _ptr(cache_prev), _ptr(out), _ptr(cache_new))
        self._check(rc, "nova_merge_cache_rows")

    # -- nova_merge_cache -----------------------------------------------------------
    def merge_cache(self, h: int, w: int, hp: int, wp: int, k: int, x: torch.Tensor,
                    y_kept: Optional[torch.Tensor], kept_idx: Optional[torch.Tensor], keep_mask: torch.Tensor,
                    cache_prev: Optional[torch.Tensor], out: torch.Tensor,
                    cache_new: Optional[torch.Tensor] = None):
        B, _, Cc = x.shape
        rc = self.lib.nova_merge_cache(self.ctx, _stream(), _dtype_code(x), B, Cc, h, w, hp, wp, k, _ptr(x),
                                       _ptr(y_kept), _ptr(kept_idx), _ptr(keep_mask), _ptr(cache_prev),
                                       _ptr(out), _ptr(cache_new))
        self._check(rc, "nova_merge_cache")

    def merge_cache_interp(self, interp: int, h: int, w: int, hp: int, wp: int, k: int, x: torch.Tensor,
                           y_kept: Optional[torch.Tensor], kept_idx: Optional[torch.Tensor],
                           keep_mask: torch.Tensor, cache_prev: Optional[torch.Tensor], out: torch.Tensor,
                           cache_new: Optional[torch.Tensor] = None):
        """interp: NOVA_INTERP_BILINEAR (0), NOVA_INTERP_NEAREST (1), NOVA_INTERP_BICUBIC (2)."""
        B, _, Cc = x.shape
        rc = self.lib.nova_merge_cache_interp(self.ctx, _stream(), _dtype_code(x), interp, B, Cc, h, w, hp, wp, k,
                                              _ptr(x), _ptr(y_kept), _ptr(kept_idx), _ptr(keep_mask),
                                              _ptr(cache_prev), _ptr(out), _ptr(cache_new))
        self._check(rc, "nova_merge_cache_interp")


# ------------------------------------------------------------------------------------
# KV-cache layout helpers (pure permutations, no arithmetic).  The library stores keys
# as [B, heads, capacity, dh] and values key-minor as [B, heads, dh, capacity].
# ------------------------------------------------------------------------------------
def pack_k_cache(k_rows: torch.Tensor, heads: int, capacity: int, fill: float = 0.0) -> torch.Tensor:
    """[B, P, C] logical key rows -> [B, heads, capacity, dh] with rows [0, P) filled."""
    B, P, Cc = k_rows.shape
    dh = Cc // heads
    out = torch.full((B, heads, capacity, dh), fill, dtype=k_rows.dtype, device=k_rows.device)
    out[:, :, :P] = k_rows.reshape(B, P, heads, dh).permute(0, 2, 1, 3)
    return out


def pack_v_cache(v_rows: torch.Tensor, heads: int, capacity: int, fill: float = 0.0) -> torch.Tensor:
    """[B, P, C] logical value rows -> [B, heads, dh, capacity] with columns [0, P) filled."""
    B, P, Cc = v_rows.shape
    dh = Cc // heads
    out = torch.full((B, heads, dh, capacity), fill, dtype=v_rows.dtype, device=v_rows.device)
    out[:, :, :, :P] = v_rows.reshape(B, P, heads, dh).permute(0, 2, 3, 1)
    return out


def unpack_k_rows(k_cache: torch.Tensor, start: int, stop: int) -> torch.Tensor:
    """cache rows [start, stop) back to the logical [B, stop-start, C]."""
    B, H, _, dh = k_cache.shape
    return k_cache[:, :, start:stop].permute(0, 2, 1, 3).reshape(B, stop - start, H * dh)


def unpack_v_rows(v_cache: torch.Tensor, start: int, stop: int) -> torch.Tensor:
    B, H, dh, _ = v_cache.shape
    return v_cache[:, :, :, start:stop].permute(0, 3, 1, 2).reshape(B, stop - start, H * dh)
