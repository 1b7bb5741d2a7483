"""ctypes binding of libfocus.so: same names as include/focus.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the decode path runs in the library's HIP
kernels.  Importing this module fails loudly when the library has not been built
(python -m paper_2601_23278_amd.build, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfocus.so")

FOCUS_OK, FOCUS_EINVAL, FOCUS_ENOMEM, FOCUS_EHIP = 0, -1, -2, -3
FOCUS_F32, FOCUS_BF16 = 0, 1
FOCUS_MAX_BLOCK = 64
KC_GEMM, KC_ATTENTION, KC_IMPORTANCE, KC_POINTWISE, KC_DECODE, KC_ROUTE, KC_EXPERTS, KC_SELECT, KC_GATHER, KC_KV_WRITE, KC_COUNT = range(11)
KC_NAMES = ["gemm", "attention", "importance", "pointwise", "decode", "route", "experts", "select", "gather", "kv_write"]


class focus_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                         "dtype")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("block_size", "mask_token_id", "max_batch", "max_prefix_len", "page_size",
                                         "n_pages", "evict_layer", "importance_mode", "maxpool_k", "budget_mode",
                                         "topk")] + \
               [("keep_ratio", C.c_float), ("alpha", C.c_float), ("constraints", C.c_int32),
                ("conf_threshold", C.c_float), ("intra_block_cache", C.c_int32), ("selection", C.c_int32),
                ("selection_seed", C.c_uint32)] + \
               [(n, C.c_int32) for n in ("n_experts", "experts_per_token", "expert_ffn", "shared_ffn", "first_moe_layer")] + \
               [("route_scale", C.c_float)]


class focus_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down",
                                                     "w_router", "w_expert_gate_up", "w_expert_down", "w_shared_gate_up",
                                                     "w_shared_down")]


_OUT_FIELDS = ("tokens", "mask_bits", "n_decoded", "importance_prev", "importance", "delta_I", "K", "keep_bits",
               "cu_seqlens", "row_map", "conf", "argmax", "hidden_full", "hidden_packed", "logits", "route_experts",
               "route_weights")


class focus_step_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _OUT_FIELDS]


class focus_seq_state(C.Structure):
    _fields_ = [("prefix_len", C.c_int32), ("total_steps", C.c_int32), ("token_sum", C.c_int64),
                ("mask_bits", C.c_uint64), ("processed_bits", C.c_uint64), ("cached_bits", C.c_uint64),
                ("tokens", C.c_int32 * FOCUS_MAX_BLOCK)]


class FocusError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("libfocus error %d: %s" % (code, text))
        self.code = code


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfocus.so is not built (%s): run `python -m paper_2601_23278_amd.build`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    P, I, SZ = C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)
    sig = {
        "focus_workspace_bytes": [C.POINTER(focus_config), SZ],
        "focus_kv_pool_bytes": [C.POINTER(focus_config), SZ],
        "focus_init": [C.POINTER(focus_config), C.POINTER(focus_weights), P, C.c_size_t, P, C.c_size_t, C.POINTER(P)],
        "focus_prefill_kv": [P, P, I, C.POINTER(I), C.POINTER(I), C.POINTER(I), I, C.POINTER(I), I],
        "focus_step": [P, P, I, P, P, P, C.POINTER(focus_step_out)],
        "focus_select_compact": [P, P, I, P, P, P, C.POINTER(focus_step_out)],
        "focus_select_compact_noalloc": [C.POINTER(focus_config), P, I, P, P, P, P, P, P, C.POINTER(focus_step_out)],
        "focus_commit": [P, P, I, P, P, P, P, P, C.POINTER(focus_step_out)],
        "focus_run_layers": [P, P, I, P, P, P, I, I, P],
        "focus_finalize_blocks": [P, P, I, P, P],
        "focus_set_route_override": [P, P],
        "focus_set_row_hint": [P, I, I],
        "focus_run_steps": [P, P, I, P, I, I, P, C.POINTER(focus_step_out)],
        "focus_get_state": [P, I, C.POINTER(focus_seq_state)],
        "focus_set_state": [P, I, C.POINTER(focus_seq_state)],
        "focus_set_timing": [P, I],
        "focus_get_kernel_time": [P, I, C.POINTER(C.c_float), C.POINTER(I)],
        "focus_free": [P],
    }
    for name, args in sig.items():
        f = getattr(lib, name)
        f.argtypes, f.restype = args, C.c_int
    lib.focus_last_error.argtypes, lib.focus_last_error.restype = [P], C.c_char_p
    return lib


_lib = load_library()
EXPORTS = ["focus_workspace_bytes", "focus_kv_pool_bytes", "focus_init", "focus_prefill_kv", "focus_step",
           "focus_select_compact", "focus_select_compact_noalloc", "focus_commit", "focus_run_layers", "focus_finalize_blocks", "focus_set_route_override", "focus_set_row_hint", "focus_run_steps", "focus_get_state", "focus_set_state", "focus_set_timing",
           "focus_get_kernel_time", "focus_free", "focus_last_error"]


def _check(rc: int, ctx=None):
    if rc != FOCUS_OK:
        raise FocusError(rc, (_lib.focus_last_error(ctx) or b"").decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _i32(xs: Optional[Sequence[int]]):
    return None if xs is None else (C.c_int32 * len(xs))(*xs)


def focus_workspace_bytes(cfg: focus_config) -> int:
    n = C.c_size_t()
    _check(_lib.focus_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def focus_kv_pool_bytes(cfg: focus_config) -> int:
    n = C.c_size_t()
    _check(_lib.focus_kv_pool_bytes(C.byref(cfg), C.byref(n)))
    return n.value


FOCUS_NOALLOC_MAX_SEQ = 16384


def focus_select_compact_noalloc(cfg: focus_config, n_seq: int, delta_I: torch.Tensor, mask_bits: torch.Tensor,
                                 out: "focus_step_out", cached_bits: Optional[torch.Tensor] = None,
                                 token_sum: Optional[torch.Tensor] = None, total_steps: Optional[torch.Tensor] = None,
                                 k_override: Optional[torch.Tensor] = None, stream=None):
    _check(_lib.focus_select_compact_noalloc(C.byref(cfg), Focus._stream(stream), n_seq, _ptr(delta_I), _ptr(mask_bits),
                                             _ptr(cached_bits), _ptr(token_sum), _ptr(total_steps), _ptr(k_override),
                                             C.byref(out)))


def make_step_out(**tensors) -> focus_step_out:
    o = focus_step_out()
    for k, t in tensors.items():
        if k not in _OUT_FIELDS:
            raise KeyError(k)
        setattr(o, k, None if t is None else t.data_ptr())
    return o


class Focus:
    """A context: marshals tensors to the C ABI and keeps the borrowed buffers alive."""

    def __init__(self, cfg: focus_config, embed: torch.Tensor, lm_head: torch.Tensor, final_norm: torch.Tensor,
                 layers: List[Dict[str, torch.Tensor]], kv_pool: torch.Tensor, workspace: Optional[torch.Tensor] = None):
        self.cfg = cfg
        self.keep = [embed, lm_head, final_norm, layers, kv_pool]
        need = focus_workspace_bytes(cfg)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=kv_pool.device)
        self.workspace = workspace
        w = focus_weights()
        w.embed, w.lm_head, w.final_norm = embed.data_ptr(), lm_head.data_ptr(), final_norm.data_ptr()
        self._arrays = {}
        names = ["attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down"]
        if cfg.n_experts > 0:
            names += ["w_router", "w_expert_gate_up", "w_expert_down"] + (["w_shared_gate_up", "w_shared_down"] if cfg.shared_ffn else [])
        for name in names:
            arr = (C.c_void_p * cfg.n_layers)(*[l[name].data_ptr() if name in l else None for l in layers])
            self._arrays[name] = arr
            setattr(w, name, arr)
        self._ctx = C.c_void_p()
        _check(_lib.focus_init(C.byref(cfg), C.byref(w), _ptr(kv_pool), kv_pool.numel() * kv_pool.element_size(),
                               _ptr(workspace), workspace.numel(), C.byref(self._ctx)))

    # -- entry points, same names as the header -------------------------------------------------
    def focus_prefill_kv(self, prefix_len: Sequence[int], page_table: Sequence[Sequence[int]],
                         prompt_tokens: Optional[Sequence[Sequence[int]]] = None,
                         seq_slot: Optional[Sequence[int]] = None, keep_stats: bool = False, stream=None):
        n = len(prefix_len)
        stride = max([len(t) for t in page_table] + [1])
        flat = [-1] * (n * stride)
        for b, t in enumerate(page_table):
            flat[b * stride:b * stride + len(t)] = list(t)
        prompts = None if prompt_tokens is None else [t for row in prompt_tokens for t in row]
        _check(_lib.focus_prefill_kv(self._ctx, self._stream(stream), n, _i32(seq_slot), _i32(list(prefix_len)),
                                     _i32(flat), stride, _i32(prompts), int(keep_stats)), self._ctx)

    def focus_step(self, n_seq: int, seq_slot: Optional[torch.Tensor] = None, k_override: Optional[torch.Tensor] = None,
                   keep_override: Optional[torch.Tensor] = None, out: Optional[focus_step_out] = None, stream=None):
        _check(_lib.focus_step(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), _ptr(k_override),
                               _ptr(keep_override), None if out is None else C.byref(out)), self._ctx)

    def focus_select_compact(self, n_seq: int, delta_I: torch.Tensor, out: focus_step_out,
                             seq_slot: Optional[torch.Tensor] = None, k_override: Optional[torch.Tensor] = None, stream=None):
        _check(_lib.focus_select_compact(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), _ptr(delta_I),
                                         _ptr(k_override), C.byref(out)), self._ctx)

    def focus_commit(self, n_seq: int, keep_bits: torch.Tensor, cu_seqlens: torch.Tensor, conf: torch.Tensor,
                     argmax: torch.Tensor, out: Optional[focus_step_out] = None, seq_slot: Optional[torch.Tensor] = None,
                     stream=None):
        _check(_lib.focus_commit(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), _ptr(keep_bits), _ptr(cu_seqlens),
                                 _ptr(conf), _ptr(argmax), None if out is None else C.byref(out)), self._ctx)

    def focus_run_layers(self, n_seq: int, keep_bits: torch.Tensor, vis_bits: torch.Tensor, layer_begin: int,
                         layer_end: int, hidden: torch.Tensor, seq_slot: Optional[torch.Tensor] = None, stream=None):
        _check(_lib.focus_run_layers(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), _ptr(keep_bits), _ptr(vis_bits),
                                     layer_begin, layer_end, _ptr(hidden)), self._ctx)

    def focus_finalize_blocks(self, n_seq: int, finalized: Optional[torch.Tensor] = None, seq_slot: Optional[torch.Tensor] = None,
                              stream=None):
        _check(_lib.focus_finalize_blocks(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), _ptr(finalized)), self._ctx)

    def focus_run_steps(self, n_seq: int, n_steps: int, finalize: bool = True, decoded: Optional[torch.Tensor] = None,
                        out: Optional[focus_step_out] = None, seq_slot: Optional[torch.Tensor] = None, stream=None):
        _check(_lib.focus_run_steps(self._ctx, self._stream(stream), n_seq, _ptr(seq_slot), n_steps, int(finalize), _ptr(decoded),
                                    None if out is None else C.byref(out)), self._ctx)

    def focus_set_route_override(self, experts: Optional[torch.Tensor]):
        self._route_override = experts       # borrowed by the library
        _check(_lib.focus_set_route_override(self._ctx, _ptr(experts)), self._ctx)

    def focus_set_row_hint(self, packed_rows: int, rows_per_seq: int = 0):
        _check(_lib.focus_set_row_hint(self._ctx, packed_rows, rows_per_seq), self._ctx)

    def focus_get_state(self, slot: int) -> focus_seq_state:
        st = focus_seq_state()
        _check(_lib.focus_get_state(self._ctx, slot, C.byref(st)), self._ctx)
        return st

    def focus_set_state(self, slot: int, st: focus_seq_state):
        _check(_lib.focus_set_state(self._ctx, slot, C.byref(st)), self._ctx)

    def focus_set_timing(self, enable: bool):
        _check(_lib.focus_set_timing(self._ctx, int(enable)), self._ctx)

    def focus_get_kernel_time(self, kernel_class: int):
        ms, n = C.c_float(), C.c_int32()
        _check(_lib.focus_get_kernel_time(self._ctx, kernel_class, C.byref(ms), C.byref(n)), self._ctx)
        return ms.value, n.value

    def focus_free(self):
        if self._ctx:
            _lib.focus_free(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.focus_free()
        except Exception:
            pass

    @staticmethod
    def _stream(stream):
        if stream is None:
            stream = torch.cuda.current_stream()
        return C.c_void_p(stream.cuda_stream)
