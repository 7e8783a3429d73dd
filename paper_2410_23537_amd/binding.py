"""Thin ctypes binding of ``libalise_kv.so`` -- argument marshalling only.

Every function here has the name and the arguments of the C entry point it calls
(``include/alise_kv.h``); tensors are torch device tensors used purely as device
memory, the stream is torch's current HIP stream.  There is no fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ALISE_KV_LIB") or os.path.join(_HERE, "libalise_kv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2410_23537_amd/build.py); there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

ALISE_OK = 0
ALISE_INVALID_ARGUMENT = 1
ALISE_UNSUPPORTED = 2
ALISE_WORKSPACE_TOO_SMALL = 3
ALISE_MISALIGNED = 4
ALISE_HIP_ERROR = 5

EXPORTS = ("alise_kv_codes_bytes", "alise_kv_meta_bytes", "alise_kv_quant_write",
           "alise_paged_decode_attn_workspace_bytes", "alise_paged_decode_attn",
           "alise_paged_decode_attn_plan", "alise_paged_decode_attn_planned", "alise_paged_decode_attn_static",
           "alise_kv_dequant_page", "alise_kv_swap_bytes", "alise_kv_swap_out", "alise_kv_swap_in",
           "alise_paged_prefill_attn_workspace_bytes", "alise_paged_prefill_attn",
           "alise_add_layernorm", "alise_bias_relu", "alise_hbm_read_probe", "alise_issue_overlap_probe",
           "alise_sched_create", "alise_sched_destroy", "alise_sched_add_job", "alise_sched_num_jobs",
           "alise_sched_step", "alise_sched_commit",
           "alise_replay_create", "alise_replay_destroy", "alise_replay_add_job", "alise_replay_num_jobs",
           "alise_replay_iterate", "alise_replay_commit", "alise_replay_synchronize", "alise_replay_get_stats",
           "alise_reload_environment", "alise_status_string")


class alise_kv_cache(ctypes.Structure):
    _fields_ = [("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
                ("k_meta", ctypes.c_void_p), ("v_meta", ctypes.c_void_p),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("codes_block_stride", ctypes.c_int64), ("meta_block_stride", ctypes.c_int64)]


_P = ctypes.POINTER(alise_kv_cache)
_lib.alise_kv_codes_bytes.restype = ctypes.c_size_t
_lib.alise_kv_codes_bytes.argtypes = [_P]
_lib.alise_kv_meta_bytes.restype = ctypes.c_size_t
_lib.alise_kv_meta_bytes.argtypes = [_P]
_lib.alise_kv_quant_write.restype = ctypes.c_int
_lib.alise_kv_quant_write.argtypes = [_P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_int32, ctypes.c_void_p]
_lib.alise_paged_decode_attn_workspace_bytes.restype = ctypes.c_size_t
_lib.alise_paged_decode_attn_workspace_bytes.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
_lib.alise_paged_decode_attn.restype = ctypes.c_int
_lib.alise_paged_decode_attn.argtypes = [_P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t,
                                         ctypes.c_void_p]
_lib.alise_paged_decode_attn_static.restype = ctypes.c_int
_lib.alise_paged_decode_attn_static.argtypes = _lib.alise_paged_decode_attn.argtypes[:10] + [ctypes.c_void_p]
_lib.alise_paged_decode_attn_planned.restype = ctypes.c_int
_lib.alise_paged_decode_attn_planned.argtypes = _lib.alise_paged_decode_attn.argtypes
_lib.alise_paged_decode_attn_plan.restype = ctypes.c_int
_lib.alise_paged_decode_attn_plan.argtypes = [_P, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.alise_kv_dequant_page.restype = ctypes.c_int
_lib.alise_kv_dequant_page.argtypes = [_P, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.alise_paged_prefill_attn_workspace_bytes.restype = ctypes.c_size_t
_lib.alise_paged_prefill_attn_workspace_bytes.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
_lib.alise_paged_prefill_attn.restype = ctypes.c_int
_lib.alise_paged_prefill_attn.argtypes = [_P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                                          ctypes.c_size_t, ctypes.c_void_p]
_lib.alise_kv_swap_bytes.restype = ctypes.c_size_t
_lib.alise_kv_swap_bytes.argtypes = [_P, ctypes.c_int32]
_lib.alise_kv_swap_out.restype = ctypes.c_int
_lib.alise_kv_swap_out.argtypes = [_P, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.alise_kv_swap_in.restype = ctypes.c_int
_lib.alise_kv_swap_in.argtypes = [_P, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.alise_add_layernorm.restype = ctypes.c_int
_lib.alise_add_layernorm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p]
_lib.alise_bias_relu.restype = ctypes.c_int
_lib.alise_bias_relu.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                 ctypes.c_void_p]
_lib.alise_hbm_read_probe.restype = ctypes.c_int
_lib.alise_hbm_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
_lib.alise_reload_environment.restype = None
_lib.alise_reload_environment.argtypes = []
_lib.alise_issue_overlap_probe.restype = ctypes.c_int
_lib.alise_issue_overlap_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
_lib.alise_status_string.restype = ctypes.c_char_p
_lib.alise_status_string.argtypes = [ctypes.c_int]


class AliseError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {alise_status_string(status)}")


def alise_status_string(status: int) -> str:
    return _lib.alise_status_string(int(status)).decode()


def alise_reload_environment() -> None:
    """Read the ALISE_* environment variables again (the library reads them once per process)."""
    _lib.alise_reload_environment()


def _check(status: int, where: str) -> None:
    if status != ALISE_OK:
        raise AliseError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dp(t) -> int:
    return 0 if t is None else t.data_ptr()


@dataclass
class KVCache:
    """Device buffers of the compressed cache plus its geometry (see alise_kv_cache in the header)."""
    k_codes: torch.Tensor   # uint8 [num_pages, Hkv, P, D*bits/8]
    v_codes: torch.Tensor
    k_meta: torch.Tensor    # fp16  [num_pages, Hkv, P, D/G, 2]
    v_meta: torch.Tensor
    num_pages: int
    page_size: int
    num_kv_heads: int
    head_dim: int
    bits: int
    group_size: int
    codes_block_stride: int = 0     # bytes between (page, head) blocks; 0 = dense
    meta_block_stride: int = 0
    storage: torch.Tensor | None = None   # the single allocation of an interleaved cache

    @staticmethod
    def allocate(num_pages, page_size, num_kv_heads, head_dim, bits, group_size, device="cuda", fill=None,
                 layout="interleaved"):
        """``layout="dense"``: four separate arrays in the canonical shapes.
        ``layout="interleaved"``: one allocation whose (page, head) blocks hold
        [K codes | V codes | K meta | V meta]; the four tensors are strided views of it with
        the same logical shapes."""
        rowb = head_dim * bits // 8
        ng = head_dim // group_size
        cshape = (num_pages, num_kv_heads, page_size, rowb)
        mshape = (num_pages, num_kv_heads, page_size, ng, 2)
        if layout == "dense":
            mk = (lambda s, dt: torch.empty(s, dtype=dt, device=device)) if fill is None else \
                 (lambda s, dt: torch.full(s, fill, dtype=dt, device=device))
            return KVCache(mk(cshape, torch.uint8), mk(cshape, torch.uint8), mk(mshape, torch.float16),
                           mk(mshape, torch.float16), num_pages, page_size, num_kv_heads, head_dim, bits,
                           group_size)
        assert layout == "interleaved"
        cb, mb = page_size * rowb, page_size * ng * 4
        blk = 2 * cb + 2 * mb
        store = torch.empty((num_pages, num_kv_heads, blk), dtype=torch.uint8, device=device)
        if fill is not None:
            store.fill_(fill)
        kc = store[:, :, 0:cb].unflatten(-1, (page_size, rowb))
        vc = store[:, :, cb:2 * cb].unflatten(-1, (page_size, rowb))
        km = store[:, :, 2 * cb:2 * cb + mb].view(torch.float16).unflatten(-1, (page_size, ng, 2))
        vm = store[:, :, 2 * cb + mb:blk].view(torch.float16).unflatten(-1, (page_size, ng, 2))
        if fill is not None:
            km.fill_(fill)
            vm.fill_(fill)
        return KVCache(kc, vc, km, vm, num_pages, page_size, num_kv_heads, head_dim, bits, group_size,
                       blk, blk, store)

    def c_struct(self) -> alise_kv_cache:
        return alise_kv_cache(_dp(self.k_codes), _dp(self.v_codes), _dp(self.k_meta), _dp(self.v_meta),
                              self.num_pages, self.page_size, self.num_kv_heads, self.head_dim,
                              self.bits, self.group_size, self.codes_block_stride, self.meta_block_stride)


def alise_kv_codes_bytes(cache: KVCache) -> int:
    return _lib.alise_kv_codes_bytes(ctypes.byref(cache.c_struct()))


def alise_kv_meta_bytes(cache: KVCache) -> int:
    return _lib.alise_kv_meta_bytes(ctypes.byref(cache.c_struct()))


def alise_kv_quant_write(cache: KVCache, k: torch.Tensor, v: torch.Tensor, slot_mapping: torch.Tensor) -> None:
    """k, v: fp16 [T, Hkv, D] device; slot_mapping: int64 [T] device."""
    T = int(slot_mapping.numel())
    assert k.dtype == torch.float16 and v.dtype == torch.float16 and slot_mapping.dtype == torch.int64
    assert k.is_contiguous() and v.is_contiguous() and slot_mapping.is_contiguous()
    assert tuple(k.shape) == (T, cache.num_kv_heads, cache.head_dim) == tuple(v.shape)
    st = _lib.alise_kv_quant_write(ctypes.byref(cache.c_struct()), _dp(k), _dp(v), _dp(slot_mapping), T, _stream())
    _check(st, "alise_kv_quant_write")


def alise_paged_decode_attn_workspace_bytes(cache: KVCache, B: int, num_q_heads: int, max_context_len: int) -> int:
    return _lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(cache.c_struct()), B, num_q_heads,
                                                        max_context_len)


def alise_paged_decode_attn(cache: KVCache, q: torch.Tensor, out: torch.Tensor, block_tables: torch.Tensor,
                            context_lens: torch.Tensor, max_context_len: int, softmax_scale: float,
                            workspace: torch.Tensor) -> None:
    """q, out: fp16 [B, H, D]; block_tables: int32 [B, max_blocks]; context_lens: int32 [B];
    workspace: uint8 device tensor of at least alise_paged_decode_attn_workspace_bytes(...) bytes."""
    B, H, D = q.shape
    assert q.dtype == torch.float16 and out.dtype == torch.float16 and tuple(out.shape) == (B, H, D)
    assert block_tables.dtype == torch.int32 and context_lens.dtype == torch.int32
    assert q.is_contiguous() and out.is_contiguous() and block_tables.is_contiguous() and context_lens.is_contiguous()
    assert block_tables.shape[0] == B and context_lens.numel() == B
    st = _lib.alise_paged_decode_attn(ctypes.byref(cache.c_struct()), _dp(q), _dp(out), _dp(block_tables),
                                      int(block_tables.shape[1]), _dp(context_lens), B, H, int(max_context_len),
                                      float(softmax_scale), _dp(workspace),
                                      int(workspace.numel() * workspace.element_size()), _stream())
    _check(st, "alise_paged_decode_attn")


ALISE_STATIC_SCRATCH_BYTES = 32 << 20


def alise_paged_decode_attn_static(cache: KVCache, q: torch.Tensor, out: torch.Tensor, block_tables: torch.Tensor,
                                   context_lens: torch.Tensor, max_context_len: int, softmax_scale: float) -> None:
    """alise_paged_decode_attn on the library's own static workspace (nothing is allocated)."""
    B, H, D = q.shape
    assert q.dtype == torch.float16 and out.dtype == torch.float16 and tuple(out.shape) == (B, H, D)
    assert block_tables.dtype == torch.int32 and context_lens.dtype == torch.int32
    assert q.is_contiguous() and out.is_contiguous() and block_tables.is_contiguous() and context_lens.is_contiguous()
    assert block_tables.shape[0] == B and context_lens.numel() == B
    st = _lib.alise_paged_decode_attn_static(ctypes.byref(cache.c_struct()), _dp(q), _dp(out), _dp(block_tables),
                                             int(block_tables.shape[1]), _dp(context_lens), B, H, int(max_context_len),
                                             float(softmax_scale), _stream())
    _check(st, "alise_paged_decode_attn_static")


def alise_paged_decode_attn_plan(cache: KVCache, context_lens: torch.Tensor, num_q_heads: int, max_context_len: int,
                                 workspace: torch.Tensor) -> None:
    """The part of alise_paged_decode_attn that depends on the lengths alone: once per decode iteration."""
    assert context_lens.dtype == torch.int32 and context_lens.is_contiguous() and context_lens.is_cuda
    st = _lib.alise_paged_decode_attn_plan(ctypes.byref(cache.c_struct()), _dp(context_lens), int(context_lens.numel()),
                                           int(num_q_heads), int(max_context_len), _dp(workspace),
                                           int(workspace.numel() * workspace.element_size()), _stream())
    _check(st, "alise_paged_decode_attn_plan")


def alise_paged_decode_attn_planned(cache: KVCache, q: torch.Tensor, out: torch.Tensor, block_tables: torch.Tensor,
                                    context_lens: torch.Tensor, max_context_len: int, softmax_scale: float,
                                    workspace: torch.Tensor) -> None:
    """alise_paged_decode_attn on the plan that alise_paged_decode_attn_plan left in the workspace: once per layer."""
    B, H, D = q.shape
    assert q.dtype == torch.float16 and out.dtype == torch.float16 and tuple(out.shape) == (B, H, D)
    assert block_tables.dtype == torch.int32 and context_lens.dtype == torch.int32
    assert q.is_contiguous() and out.is_contiguous() and block_tables.is_contiguous() and context_lens.is_contiguous()
    assert block_tables.shape[0] == B and context_lens.numel() == B
    st = _lib.alise_paged_decode_attn_planned(ctypes.byref(cache.c_struct()), _dp(q), _dp(out), _dp(block_tables),
                                              int(block_tables.shape[1]), _dp(context_lens), B, H, int(max_context_len),
                                              float(softmax_scale), _dp(workspace),
                                              int(workspace.numel() * workspace.element_size()), _stream())
    _check(st, "alise_paged_decode_attn_planned")


def alise_kv_dequant_page(cache: KVCache, page: int, k_out: torch.Tensor, v_out: torch.Tensor) -> None:
    """k_out, v_out: fp16 [P, Hkv, D] device."""
    shape = (cache.page_size, cache.num_kv_heads, cache.head_dim)
    assert tuple(k_out.shape) == shape == tuple(v_out.shape)
    assert k_out.dtype == torch.float16 and v_out.dtype == torch.float16
    assert k_out.is_contiguous() and v_out.is_contiguous()
    st = _lib.alise_kv_dequant_page(ctypes.byref(cache.c_struct()), int(page), _dp(k_out), _dp(v_out), _stream())
    _check(st, "alise_kv_dequant_page")


def alise_paged_prefill_attn_workspace_bytes(cache: KVCache, B: int, total_q_tokens: int, num_q_heads: int,
                                             max_context_len: int) -> int:
    return int(_lib.alise_paged_prefill_attn_workspace_bytes(ctypes.byref(cache.c_struct()), int(B), int(total_q_tokens),
                                                             int(num_q_heads), int(max_context_len)))


def alise_paged_prefill_attn(cache: KVCache, q: torch.Tensor, out: torch.Tensor, q_start: torch.Tensor,
                             block_tables: torch.Tensor, context_lens: torch.Tensor, max_context_len: int,
                             softmax_scale: float, workspace: torch.Tensor) -> None:
    """q, out: fp16 [total_q, H, D]; q_start: int32 [B+1]; block_tables: int32 [B, max_blocks]; context_lens: int32 [B]."""
    assert q.dtype == torch.float16 and out.dtype == torch.float16 and q.shape == out.shape and q.dim() == 3
    assert q.is_contiguous() and out.is_contiguous() and block_tables.is_contiguous()
    assert q_start.dtype == torch.int32 and block_tables.dtype == torch.int32 and context_lens.dtype == torch.int32
    B = context_lens.shape[0]
    assert q_start.shape[0] == B + 1 and block_tables.shape[0] == B
    st = _lib.alise_paged_prefill_attn(ctypes.byref(cache.c_struct()), _dp(q), _dp(out), _dp(q_start), _dp(block_tables),
                                       block_tables.shape[1], _dp(context_lens), B, q.shape[0], q.shape[1],
                                       int(max_context_len), float(softmax_scale), _dp(workspace), workspace.numel(),
                                       _stream())
    _check(st, "alise_paged_prefill_attn")


def alise_kv_swap_bytes(cache: KVCache, num_tokens: int) -> int:
    return int(_lib.alise_kv_swap_bytes(ctypes.byref(cache.c_struct()), int(num_tokens)))


def alise_kv_swap_out(cache: KVCache, block_table: torch.Tensor, num_tokens: int, packed: torch.Tensor) -> None:
    """block_table: int32 device [>= ceil(num_tokens / P)]; packed: uint8, device or pinned host memory."""
    assert block_table.dtype == torch.int32 and block_table.is_cuda and block_table.is_contiguous()
    assert packed.dtype == torch.uint8 and packed.is_contiguous() and (packed.is_cuda or packed.is_pinned())
    st = _lib.alise_kv_swap_out(ctypes.byref(cache.c_struct()), _dp(block_table), int(num_tokens), _dp(packed),
                                packed.numel(), _stream())
    _check(st, "alise_kv_swap_out")


def alise_kv_swap_in(cache: KVCache, block_table: torch.Tensor, num_tokens: int, packed: torch.Tensor) -> None:
    assert block_table.dtype == torch.int32 and block_table.is_cuda and block_table.is_contiguous()
    assert packed.dtype == torch.uint8 and packed.is_contiguous() and (packed.is_cuda or packed.is_pinned())
    st = _lib.alise_kv_swap_in(ctypes.byref(cache.c_struct()), _dp(block_table), int(num_tokens), _dp(packed),
                               packed.numel(), _stream())
    _check(st, "alise_kv_swap_in")


def _is_matrix(t) -> bool:
    return t.dtype == torch.float16 and t.is_cuda and t.is_contiguous() and t.dim() == 2


def alise_add_layernorm(x: torch.Tensor, residual, gamma: torch.Tensor, beta: torch.Tensor, eps: float,
                        h_out, y_out: torch.Tensor) -> None:
    """x, residual (or None), h_out (or None), y_out: fp16 [rows, hidden]; gamma, beta: fp16 [hidden]."""
    assert _is_matrix(x) and _is_matrix(y_out) and y_out.shape == x.shape
    assert residual is None or (_is_matrix(residual) and residual.shape == x.shape)
    assert h_out is None or (_is_matrix(h_out) and h_out.shape == x.shape)
    rows, hidden = x.shape
    for v in (gamma, beta):
        assert v.dtype == torch.float16 and v.is_cuda and v.is_contiguous() and v.shape == (hidden,)
    st = _lib.alise_add_layernorm(_dp(x), _dp(residual), _dp(gamma), _dp(beta), float(eps), _dp(h_out), _dp(y_out),
                                  rows, hidden, _stream())
    _check(st, "alise_add_layernorm")


def alise_bias_relu(x: torch.Tensor, bias, y_out: torch.Tensor) -> None:
    """x, y_out: fp16 [rows, cols] (y_out may be x); bias: fp16 [cols] or None."""
    assert _is_matrix(x) and _is_matrix(y_out) and y_out.shape == x.shape
    rows, cols = x.shape
    assert bias is None or (bias.dtype == torch.float16 and bias.is_cuda and bias.is_contiguous() and bias.shape == (cols,))
    st = _lib.alise_bias_relu(_dp(x), _dp(bias), _dp(y_out), rows, cols, _stream())
    _check(st, "alise_bias_relu")


def alise_hbm_read_probe(src: torch.Tensor, xor_out: torch.Tensor) -> None:
    """src: any contiguous device tensor whose size in bytes is a multiple of 16; xor_out: int32 or uint32 [1], device."""
    assert src.is_cuda and src.is_contiguous() and xor_out.is_cuda and xor_out.numel() == 1 and xor_out.element_size() == 4
    st = _lib.alise_hbm_read_probe(_dp(src), src.numel() * src.element_size(), _dp(xor_out), _stream())
    _check(st, "alise_hbm_read_probe")


def alise_issue_overlap_probe(mode: int, iters: int, sink: torch.Tensor) -> None:
    """mode 1: matrix instructions, 2: vector instructions, 3: both; sink: float32 [1], device."""
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() == 1
    st = _lib.alise_issue_overlap_probe(int(mode), int(iters), _dp(sink), _stream())
    _check(st, "alise_issue_overlap_probe")


class alise_sched_config(ctypes.Structure):
    _fields_ = [("num_queues", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("gpu_job_limit", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("limit0", ctypes.c_int64), ("age_threshold", ctypes.c_int64),
                ("t0", ctypes.c_int64), ("alpha", ctypes.c_int64), ("beta", ctypes.c_int64)]


_I64P, _I32P = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)


class alise_sched_decision(ctypes.Structure):
    _fields_ = [("batch_ids", _I64P), ("batch_phase", _I32P), ("batch_cap", ctypes.c_int32), ("n_batch", ctypes.c_int32),
                ("upload_ids", _I64P), ("upload_cap", ctypes.c_int32), ("n_upload", ctypes.c_int32),
                ("offload_ids", _I64P), ("offload_cap", ctypes.c_int32), ("n_offload", ctypes.c_int32),
                ("order_ids", _I64P), ("order_queue", _I32P), ("order_ewt", _I64P), ("order_cap", ctypes.c_int32),
                ("n_order", ctypes.c_int32), ("model_time", ctypes.c_int64)]


_lib.alise_sched_create.restype = ctypes.c_int
_lib.alise_sched_create.argtypes = [ctypes.POINTER(alise_sched_config), ctypes.POINTER(ctypes.c_void_p)]
_lib.alise_sched_destroy.restype = None
_lib.alise_sched_destroy.argtypes = [ctypes.c_void_p]
_lib.alise_sched_add_job.restype = ctypes.c_int
_lib.alise_sched_add_job.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
_lib.alise_sched_num_jobs.restype = ctypes.c_int32
_lib.alise_sched_num_jobs.argtypes = [ctypes.c_void_p]
_lib.alise_sched_step.restype = ctypes.c_int
_lib.alise_sched_step.argtypes = [ctypes.c_void_p, ctypes.POINTER(alise_sched_decision)]
_lib.alise_sched_commit.restype = ctypes.c_int
_lib.alise_sched_commit.argtypes = [ctypes.c_void_p, ctypes.c_int64, _I64P, ctypes.c_int32]


class Scheduler:
    """The scheduler object of alise_sched.h; argument marshalling only.  ``step()`` returns a dict of lists."""

    def __init__(self, num_queues, limit0, age_threshold, max_batch, gpu_job_limit, t0, alpha, beta, want_order=True):
        self.cfg = alise_sched_config(num_queues, max_batch, gpu_job_limit, 0, limit0, age_threshold, t0, alpha, beta)
        self._h = ctypes.c_void_p()
        _check(_lib.alise_sched_create(ctypes.byref(self.cfg), ctypes.byref(self._h)), "alise_sched_create")
        self.want_order = want_order
        self._cap = 0

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.alise_sched_destroy(self._h)
            self._h = None

    def add_job(self, id, arrival, prompt_len, predicted_len):
        _check(_lib.alise_sched_add_job(self._h, int(id), int(arrival), int(prompt_len), int(predicted_len)), "alise_sched_add_job")

    def num_jobs(self):
        return int(_lib.alise_sched_num_jobs(self._h))

    def _buffers(self, n):
        if n > self._cap:
            self._cap = max(16, 2 * n)
            c = self._cap
            self._b = ((ctypes.c_int64 * c)(), (ctypes.c_int32 * c)(), (ctypes.c_int64 * c)(), (ctypes.c_int64 * c)(),
                       (ctypes.c_int64 * c)(), (ctypes.c_int32 * c)(), (ctypes.c_int64 * c)())
        return self._b

    def step(self):
        n = self.num_jobs()
        bi, bp, up, off, oi, oq, oe = self._buffers(n)
        c = self._cap
        d = alise_sched_decision(bi, bp, c, 0, up, c, 0, off, c, 0,
                                 oi if self.want_order else None, oq if self.want_order else None,
                                 oe if self.want_order else None, c if self.want_order else 0, 0, 0)
        _check(_lib.alise_sched_step(self._h, ctypes.byref(d)), "alise_sched_step")
        return {"batch": bi[:d.n_batch], "phase": bp[:d.n_batch], "upload": up[:d.n_upload], "offload": off[:d.n_offload],
                "order": oi[:d.n_order], "queue": oq[:d.n_order], "ewt": oe[:d.n_order], "model_time": int(d.model_time)}

    def commit(self, elapsed, finished):
        f = (ctypes.c_int64 * max(1, len(finished)))(*finished)
        _check(_lib.alise_sched_commit(self._h, int(elapsed), f, len(finished)), "alise_sched_commit")


class alise_replay_config(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("max_context", ctypes.c_int32), ("max_iter_tokens", ctypes.c_int32),
                ("overlap_swaps", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("reserved", ctypes.c_int32)]


class alise_replay_iteration(ctypes.Structure):
    _fields_ = [("batch_ids", _I64P), ("batch_phase", _I32P), ("batch_out_row", _I64P), ("batch_cap", ctypes.c_int32),
                ("n_batch", ctypes.c_int32),
                ("upload_ids", _I64P), ("upload_cap", ctypes.c_int32), ("n_upload", ctypes.c_int32),
                ("offload_ids", _I64P), ("offload_host", ctypes.POINTER(ctypes.c_void_p)),
                ("offload_bytes", ctypes.POINTER(ctypes.c_size_t)), ("offload_cap", ctypes.c_int32), ("n_offload", ctypes.c_int32),
                ("model_time", ctypes.c_int64), ("n_prefill_tokens", ctypes.c_int32), ("n_decode_tokens", ctypes.c_int32)]


class alise_replay_stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("iterations", "prefill_tokens", "decode_tokens", "offloads", "uploads",
                                              "offload_bytes", "upload_bytes")] + \
               [("free_pages", ctypes.c_int32), ("live_jobs", ctypes.c_int32)]


_lib.alise_replay_create.restype = ctypes.c_int
_lib.alise_replay_create.argtypes = [_P, ctypes.POINTER(alise_sched_config), ctypes.POINTER(alise_replay_config),
                                     ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
_lib.alise_replay_destroy.restype = None
_lib.alise_replay_destroy.argtypes = [ctypes.c_void_p]
_lib.alise_replay_add_job.restype = ctypes.c_int
_lib.alise_replay_add_job.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.c_int64]
_lib.alise_replay_num_jobs.restype = ctypes.c_int32
_lib.alise_replay_num_jobs.argtypes = [ctypes.c_void_p]
_lib.alise_replay_iterate.restype = ctypes.c_int
_lib.alise_replay_iterate.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.POINTER(alise_replay_iteration)]
_lib.alise_replay_commit.restype = ctypes.c_int
_lib.alise_replay_commit.argtypes = [ctypes.c_void_p, ctypes.c_int64, _I64P, ctypes.c_int32]
_lib.alise_replay_synchronize.restype = ctypes.c_int
_lib.alise_replay_synchronize.argtypes = [ctypes.c_void_p]
_lib.alise_replay_get_stats.restype = ctypes.c_int
_lib.alise_replay_get_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(alise_replay_stats)]


class NativeReplay:
    """The serving loop object of alise_replay.h; argument marshalling only.  Every page of the cache belongs to the object
    until close(); k_tokens, v_tokens ([rows, Hkv, D]) and q_tokens ([rows, H, D]) are device fp16 tensors in which a job finds its
    token t at row token_row + t.  ``iterate()`` returns a dict: the decision's lists, 'out' (fp16 [max_iter_tokens, H, D],
    reused by the next iteration), 'out_row' (first row of each batch job), 'n_prefill_tokens', 'n_decode_tokens', and
    'offloaded' (id -> (address of the pinned host buffer, bytes))."""

    def __init__(self, cache: "KVCache", num_q_heads: int, sched_cfg: dict, max_context: int, max_iter_tokens: int,
                 k_tokens: torch.Tensor, v_tokens: torch.Tensor, q_tokens: torch.Tensor, softmax_scale: float,
                 overlap_swaps: bool = True):
        for t, h in ((k_tokens, cache.num_kv_heads), (v_tokens, cache.num_kv_heads), (q_tokens, num_q_heads)):
            assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous() and t.shape[1:] == (h, cache.head_dim)
        assert k_tokens.shape[0] == v_tokens.shape[0] == q_tokens.shape[0]
        self.cache, self.tokens = cache, (k_tokens, v_tokens, q_tokens)
        self.scfg = alise_sched_config(sched_cfg["num_queues"], sched_cfg["max_batch"], sched_cfg["gpu_job_limit"], 0,
                                       sched_cfg["limit0"], sched_cfg["age_threshold"], sched_cfg["t0"], sched_cfg["alpha"],
                                       sched_cfg["beta"])
        self.rcfg = alise_replay_config(num_q_heads, max_context, max_iter_tokens, int(overlap_swaps), float(softmax_scale), 0)
        self.out = torch.empty((max_iter_tokens, num_q_heads, cache.head_dim), dtype=torch.float16, device=k_tokens.device)
        self._rows = k_tokens.shape[0]
        self._h = ctypes.c_void_p()
        _check(_lib.alise_replay_create(ctypes.byref(cache.c_struct()), ctypes.byref(self.scfg), ctypes.byref(self.rcfg),
                                        _stream(), ctypes.byref(self._h)), "alise_replay_create")
        nb, nm = sched_cfg["max_batch"], sched_cfg["gpu_job_limit"]
        self._b = ((ctypes.c_int64 * nb)(), (ctypes.c_int32 * nb)(), (ctypes.c_int64 * nb)(), (ctypes.c_int64 * nm)(),
                   (ctypes.c_int64 * nm)(), (ctypes.c_void_p * nm)(), (ctypes.c_size_t * nm)())
        bi, bp, br, up, off, oh, ob = self._b
        self._it = alise_replay_iteration(bi, bp, br, nb, 0, up, nm, 0, off, oh, ob, nm, 0, 0, 0, 0)

    def close(self):
        if getattr(self, "_h", None):
            _lib.alise_replay_destroy(self._h)
            self._h = None

    __del__ = close

    def add_job(self, id, arrival, prompt_len, predicted_len, token_row):
        assert 0 <= token_row and token_row + self.rcfg.max_context <= self._rows, "the job's tokens must lie inside the token arrays"
        _check(_lib.alise_replay_add_job(self._h, int(id), int(arrival), int(prompt_len), int(predicted_len), int(token_row)),
               "alise_replay_add_job")

    def num_jobs(self):
        return int(_lib.alise_replay_num_jobs(self._h))

    def iterate(self):
        k, v, q = self.tokens
        it = self._it
        _check(_lib.alise_replay_iterate(self._h, _dp(k), _dp(v), _dp(q), _dp(self.out), ctypes.byref(it)), "alise_replay_iterate")
        bi, bp, br, up, off, oh, ob = self._b
        return {"batch": bi[:it.n_batch], "phase": bp[:it.n_batch], "out_row": br[:it.n_batch], "upload": up[:it.n_upload],
                "offload": off[:it.n_offload], "offloaded": {off[i]: (oh[i], ob[i]) for i in range(it.n_offload)},
                "model_time": int(it.model_time), "n_prefill_tokens": it.n_prefill_tokens,
                "n_decode_tokens": it.n_decode_tokens, "out": self.out}

    def commit(self, elapsed, finished):
        f = (ctypes.c_int64 * max(1, len(finished)))(*finished)
        _check(_lib.alise_replay_commit(self._h, int(elapsed), f, len(finished)), "alise_replay_commit")

    def synchronize(self):
        _check(_lib.alise_replay_synchronize(self._h), "alise_replay_synchronize")

    def stats(self) -> dict:
        s = alise_replay_stats()
        _check(_lib.alise_replay_get_stats(self._h, ctypes.byref(s)), "alise_replay_get_stats")
        return {n: int(getattr(s, n)) for n, _ in s._fields_}


def raw():
    """The ctypes library handle, for tests of the error paths."""
    return _lib
