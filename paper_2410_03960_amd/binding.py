"""ctypes binding of libswiftkv.so: argument marshalling only.

Function names mirror include/swiftkv.h.  Tensors are PyTorch CUDA tensors used
purely as device-memory handles (`.data_ptr()`); every step of the computation
runs inside the HIP library.  Loading fails loudly when the library has not
been built (`python -m paper_2410_03960_amd.build`); there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswiftkv.so")

SWIFTKV_OK, SWIFTKV_EINVAL, SWIFTKV_ENOSPC, SWIFTKV_EHIP, SWIFTKV_EDATA = 0, -1, -2, -3, -4
SWIFTKV_KV_BF16, SWIFTKV_KV_FP8_E4M3 = 0, 1
SWIFTKV_SCALE_COMPUTE_ABSMAX, SWIFTKV_SCALE_USE_GIVEN, SWIFTKV_SCALE_PER_TOKEN = 0, 1, 2
N_TIME_CLASSES = 10
TIME_CLASS_NAMES = ("qkv_gemm", "o_gemm", "gateup_gemm", "down_gemm", "fused_kv_gemm",
                    "attn_prefill", "other", "tail", "norm", "kv_commit")

EXPORTS = (
    "swiftkv_pack_bytes", "swiftkv_pack_bytes_min",
    "swiftkv_create", "swiftkv_destroy", "swiftkv_workspace_bytes", "swiftkv_workspace_bytes_prefix", "swiftkv_prefill",
    "swiftkv_kv_from_hidden", "swiftkv_set_early_exit", "swiftkv_export_exit_flags", "swiftkv_export_plan", "swiftkv_export_hidden", "swiftkv_op_gemm",
    "swiftkv_op_gemm_packed", "swiftkv_op_gemm_rows", "swiftkv_op_gemm_rows_workspace", "swiftkv_op_gemm_rows_static",
    "swiftkv_op_attention_prefill", "swiftkv_op_attention_workspace", "swiftkv_op_attention_decode", "swiftkv_op_attention_decode_workspace", "swiftkv_op_fp8_quantize", "swiftkv_op_mfma_rate",
    "swiftkv_flops", "swiftkv_set_timing", "swiftkv_get_timing", "swiftkv_last_error",
    "swiftkv_version",
)


class SwiftKVError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libswiftkv error {code}: {msg}")
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
        [(n, C.POINTER(C.c_void_p)) for n in ("norm1", "wq", "wk", "wv", "wo", "norm2", "wgate", "wup", "wdown")] + \
        [("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class KVCacheDesc(C.Structure):
    _fields_ = [("data", C.c_void_p), ("scales", C.c_void_p), ("block_tables", C.c_void_p),
                ("context_lens", C.POINTER(C.c_int32)),
                ("n_cache_layers", C.c_int32), ("n_blocks", C.c_int32), ("block_size", C.c_int32),
                ("max_blocks_per_seq", C.c_int32), ("dtype", C.c_int32), ("scale_mode", C.c_int32)]


_lib = None


def load() -> C.CDLL:
    """dlopen libswiftkv.so (built in-tree); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2410_03960_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.swiftkv_pack_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.swiftkv_pack_bytes.restype = C.c_size_t
    lib.swiftkv_pack_bytes_min.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.swiftkv_pack_bytes_min.restype = C.c_size_t
    lib.swiftkv_create.argtypes = [C.POINTER(vp), C.POINTER(ModelCfg), C.POINTER(Weights), i32, i32, vp, C.c_size_t, vp]
    lib.swiftkv_destroy.argtypes = [vp]
    lib.swiftkv_destroy.restype = None
    lib.swiftkv_workspace_bytes.argtypes = [vp, i64, i32, i32]
    lib.swiftkv_workspace_bytes.restype = C.c_size_t
    lib.swiftkv_workspace_bytes_prefix.argtypes = [vp, i64, i32, i32, i64]
    lib.swiftkv_workspace_bytes_prefix.restype = C.c_size_t
    lib.swiftkv_prefill.argtypes = [vp, vp, C.POINTER(i32), i32, C.POINTER(KVCacheDesc), vp, vp, C.c_size_t, vp]
    lib.swiftkv_kv_from_hidden.argtypes = [vp, vp, C.POINTER(i32), i32, C.POINTER(KVCacheDesc), vp, C.c_size_t, vp]
    lib.swiftkv_export_plan.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.swiftkv_set_early_exit.argtypes = [vp, vp, vp, C.c_float]
    lib.swiftkv_export_exit_flags.argtypes = [vp, vp, vp, vp]
    lib.swiftkv_export_hidden.argtypes = [vp, vp, vp, vp]
    lib.swiftkv_op_gemm.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp]
    lib.swiftkv_op_gemm_packed.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    lib.swiftkv_op_gemm_rows.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, C.c_size_t, vp]
    lib.swiftkv_op_gemm_rows_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    lib.swiftkv_op_gemm_rows_workspace.argtypes = [i32, i32]
    lib.swiftkv_op_gemm_rows_workspace.restype = C.c_size_t
    lib.swiftkv_op_attention_prefill.argtypes = [vp, vp, vp, vp, C.POINTER(i32), i32, i32, i32, i32, vp, C.c_size_t, vp]
    lib.swiftkv_op_attention_workspace.argtypes = [i64, i32, i32, i32]
    lib.swiftkv_op_attention_workspace.restype = C.c_size_t
    lib.swiftkv_op_attention_decode.argtypes = [vp, vp, C.POINTER(i32), i32, i32, i32, i32, vp, vp, i32, i32, vp, vp, vp, i32, i32,
                                                vp, C.c_size_t, vp]
    lib.swiftkv_op_attention_decode_workspace.argtypes = [i32, i32, i32]
    lib.swiftkv_op_attention_decode_workspace.restype = C.c_size_t
    lib.swiftkv_op_fp8_quantize.argtypes = [vp, C.c_float, vp, i64, vp]
    lib.swiftkv_op_mfma_rate.argtypes = [vp, i32, vp, C.c_size_t, C.POINTER(C.c_double), vp]
    lib.swiftkv_flops.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.swiftkv_set_timing.argtypes = [vp, i32]
    lib.swiftkv_get_timing.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.swiftkv_last_error.restype = C.c_char_p
    lib.swiftkv_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise SwiftKVError(rc, load().swiftkv_last_error().decode())


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _i32_array(vals: Sequence[int]):
    return (C.c_int32 * len(vals))(*[int(v) for v in vals])


def _dev(t: torch.Tensor, dtype=None) -> int:
    assert t.is_cuda and t.is_contiguous(), "expected a contiguous CUDA tensor"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


_PER_LAYER = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wgate", "wup", "wdown")


def pack_bytes(shape, l: int, g: int, minimum: bool = False) -> int:
    """swiftkv_pack_bytes / swiftkv_pack_bytes_min."""
    cfg = ModelCfg(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
    fn = load().swiftkv_pack_bytes_min if minimum else load().swiftkv_pack_bytes
    return int(fn(C.byref(cfg), l, g))


class Context:
    """swiftkv_create / swiftkv_destroy.  `weights` maps "embed", "final_norm",
    "lm_head" and "<name>.<layer>" to bf16 CUDA tensors; they must outlive the
    context (a reference is kept here).  The pack buffer is a torch allocation
    of swiftkv_pack_bytes() bytes (swiftkv_pack_bytes_min() with
    packed_weights=False), kept alive here as well."""

    def __init__(self, shape, weights: Dict[str, torch.Tensor], l: int, g: int, packed_weights: bool = True,
                 stream=None):
        lib = load()
        self.shape, self.l, self.g = shape, l, g
        self._weights = weights
        cfg = ModelCfg(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                       shape.ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
        n_pack = pack_bytes(shape, l, g, minimum=not packed_weights)
        if n_pack == 0:
            _check(lib.swiftkv_create(C.byref(C.c_void_p()), C.byref(cfg), C.byref(Weights()), l, g, None, 0, None))
        self.pack_buf = torch.empty(n_pack, dtype=torch.uint8, device=weights["embed"].device)
        w = Weights()
        self._arrays = {}
        for n in _PER_LAYER:
            arr = (C.c_void_p * shape.n_layers)()
            for j in range(shape.n_layers):
                t = weights.get(f"{n}.{j}")
                arr[j] = _dev(t, torch.bfloat16) if t is not None else None
            self._arrays[n] = arr
            setattr(w, n, C.cast(arr, C.POINTER(C.c_void_p)))
        w.embed = _dev(weights["embed"], torch.bfloat16)
        w.final_norm = _dev(weights["final_norm"], torch.bfloat16)
        w.lm_head = _dev(weights["lm_head"], torch.bfloat16)
        self._h = C.c_void_p()
        _check(lib.swiftkv_create(C.byref(self._h), C.byref(cfg), C.byref(w), l, g, _dev(self.pack_buf),
                                  self.pack_buf.numel(), _stream_ptr(stream)))
        self.n_cache_layers = l + (shape.n_layers - l) // g

    def close(self):
        if getattr(self, "_h", None):
            load().swiftkv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- thin wrappers, one per C entry point ----
    def workspace_bytes(self, max_tokens: int, max_seqs: int, kv_dtype: int = SWIFTKV_KV_BF16,
                        max_prefix_tokens: int = 0) -> int:
        if max_prefix_tokens:
            return int(load().swiftkv_workspace_bytes_prefix(self._h, max_tokens, max_seqs, kv_dtype, max_prefix_tokens))
        return int(load().swiftkv_workspace_bytes(self._h, max_tokens, max_seqs, kv_dtype))

    def prefill(self, token_ids: torch.Tensor, seq_lens: Sequence[int], kv: "KVCache", logits_out: torch.Tensor,
                workspace: torch.Tensor, stream=None):
        desc = kv.desc()
        _check(load().swiftkv_prefill(self._h, _dev(token_ids, torch.int32), _i32_array(seq_lens), len(seq_lens),
                                      C.byref(desc), _dev(logits_out, torch.float32), _dev(workspace),
                                      workspace.numel() * workspace.element_size(), _stream_ptr(stream)))

    def kv_from_hidden(self, hidden_l: torch.Tensor, seq_lens: Sequence[int], kv: "KVCache",
                       workspace: torch.Tensor, stream=None):
        desc = kv.desc()
        _check(load().swiftkv_kv_from_hidden(self._h, _dev(hidden_l, torch.bfloat16), _i32_array(seq_lens),
                                             len(seq_lens), C.byref(desc), _dev(workspace),
                                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)))

    def export_plan(self, workspace: torch.Tensor, n_tokens: int, n_seqs: int, stream=None):
        dev = workspace.device
        slots = torch.empty(n_tokens, dtype=torch.int64, device=dev)
        pos = torch.empty(n_tokens, dtype=torch.int32, device=dev)
        cu = torch.empty(n_seqs + 1, dtype=torch.int32, device=dev)
        last = torch.empty(n_seqs, dtype=torch.int32, device=dev)
        _check(load().swiftkv_export_plan(self._h, _dev(workspace), _dev(slots), _dev(pos), _dev(cu), _dev(last),
                                          _stream_ptr(stream)))
        return slots, pos, cu, last

    def set_early_exit(self, gain: Optional[torch.Tensor], head: Optional[torch.Tensor], threshold: float = 0.95) -> None:
        """Extra head on the layer-l output (both None switches it off); the tensors are kept alive here."""
        self._ee = (gain, head)
        _check(load().swiftkv_set_early_exit(self._h, _dev(gain) if gain is not None else None,
                                             _dev(head) if head is not None else None, float(threshold)))

    def export_exit_flags(self, workspace: torch.Tensor, n_seqs: int, stream=None) -> torch.Tensor:
        out = torch.empty(n_seqs, dtype=torch.int32, device=workspace.device)
        _check(load().swiftkv_export_exit_flags(self._h, _dev(workspace), _dev(out), _stream_ptr(stream)))
        return out

    def export_hidden(self, workspace: torch.Tensor, n_tokens: int, stream=None) -> torch.Tensor:
        out = torch.empty((n_tokens, self.shape.hidden), dtype=torch.bfloat16, device=workspace.device)
        _check(load().swiftkv_export_hidden(self._h, _dev(workspace), _dev(out), _stream_ptr(stream)))
        return out

    def flops(self, seq_lens: Sequence[int], context_lens: Sequence[int]):
        g, a = C.c_double(), C.c_double()
        _check(load().swiftkv_flops(self._h, _i32_array(seq_lens), _i32_array(context_lens), len(seq_lens),
                                    C.byref(g), C.byref(a)))
        return g.value, a.value

    def set_timing(self, enable: bool, classes: Optional[Sequence[str]] = None):
        """Bracket launches with HIP events: every class, or only the named ones (TIME_CLASS_NAMES)."""
        mask = 0
        if enable:
            mask = (1 << N_TIME_CLASSES) - 1 if classes is None else sum(1 << TIME_CLASS_NAMES.index(c) for c in classes)
        _check(load().swiftkv_set_timing(self._h, mask))

    def get_timing(self):
        ms = (C.c_double * N_TIME_CLASSES)()
        n = (C.c_int32 * N_TIME_CLASSES)()
        _check(load().swiftkv_get_timing(self._h, ms, n))
        return {TIME_CLASS_NAMES[i]: (ms[i], n[i]) for i in range(N_TIME_CLASSES)}


class KVCache:
    """Device memory for a paged cache + its descriptor (swiftkv_kv_cache)."""

    def __init__(self, n_cache_layers: int, n_blocks: int, n_kv_heads: int, head_dim: int,
                 block_tables: torch.Tensor, context_lens: Sequence[int], fp8: bool = False,
                 scale_mode: int = SWIFTKV_SCALE_COMPUTE_ABSMAX, device="cuda"):
        self.fp8 = fp8
        shape = (n_cache_layers, 2, n_blocks * 16, n_kv_heads, head_dim)
        self.data = torch.zeros(shape, dtype=torch.uint8 if fp8 else torch.bfloat16, device=device)
        per_token = fp8 and scale_mode == SWIFTKV_SCALE_PER_TOKEN
        self.scales = torch.zeros((n_cache_layers, 2, n_blocks * 16 if per_token else n_kv_heads), dtype=torch.float32,
                                  device=device) if fp8 else None
        self.block_tables = block_tables.to(device=device, dtype=torch.int32).contiguous()
        self.context_lens = _i32_array(context_lens)
        self.n_cache_layers, self.n_blocks = n_cache_layers, n_blocks
        self.scale_mode = scale_mode

    def set_context_lens(self, context_lens: Sequence[int]) -> None:
        """Tokens already cached per sequence, for the next call (host array)."""
        self.context_lens = _i32_array(context_lens)

    def desc(self) -> KVCacheDesc:
        return KVCacheDesc(self.data.data_ptr(), self.scales.data_ptr() if self.scales is not None else None,
                           self.block_tables.data_ptr(), C.cast(self.context_lens, C.POINTER(C.c_int32)),
                           self.n_cache_layers, self.n_blocks, 16, self.block_tables.shape[1],
                           SWIFTKV_KV_FP8_E4M3 if self.fp8 else SWIFTKV_KV_BF16, self.scale_mode)


def op_mfma_rate(operands: torch.Tensor, iters: int = 20000, stream=None) -> float:
    """TFLOP/s of MFMA instructions alone on `operands` (bf16 CUDA tensor, >= 16384 elements)."""
    assert operands.dtype == torch.bfloat16 and operands.numel() >= 16384 and operands.is_contiguous()
    out = C.c_double(0.0)
    sink = torch.empty(1 << 20, dtype=torch.uint8, device=operands.device)
    _check(load().swiftkv_op_mfma_rate(_dev(operands), iters, _dev(sink), sink.numel(), C.byref(out), _stream_ptr(stream)))
    return float(out.value)


def op_gemm(A: torch.Tensor, W: torch.Tensor, out_f32: bool = False, variant: int = 0, stream=None,
            out: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device=A.device)
    _check(load().swiftkv_op_gemm(_dev(A, torch.bfloat16), _dev(W, torch.bfloat16), _dev(out), M, N, K,
                                  int(out_f32), variant, _stream_ptr(stream)))
    return out


def op_gemm_packed(A: torch.Tensor, W: torch.Tensor, stream=None) -> torch.Tensor:
    """bf16 product through the packed-weight loop (W is re-arranged into a scratch tensor first)."""
    M, K = A.shape
    N = W.shape[0]
    out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    scratch = torch.empty_like(W)
    _check(load().swiftkv_op_gemm_packed(_dev(A, torch.bfloat16), _dev(W, torch.bfloat16), _dev(scratch), _dev(out),
                                         M, N, K, _stream_ptr(stream)))
    return out


def op_gemm_rows(A: torch.Tensor, W: torch.Tensor, out_f32: bool = False, stream=None) -> torch.Tensor:
    """Weight-streaming GEMM for M <= 80 rows with its K-split scratch in a caller workspace."""
    M, K = A.shape
    N = W.shape[0]
    lib = load()
    ws = torch.empty(int(lib.swiftkv_op_gemm_rows_workspace(M, N)), dtype=torch.uint8, device=A.device)
    out = torch.empty((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device=A.device)
    _check(lib.swiftkv_op_gemm_rows(_dev(A, torch.bfloat16), _dev(W, torch.bfloat16), _dev(out), M, N, K, int(out_f32),
                                    _dev(ws), ws.numel(), _stream_ptr(stream)))
    return out


def op_gemm_rows_static(A: torch.Tensor, W: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
    """swiftkv_op_gemm_rows_static: the caller passes inputs and the output; nothing is allocated here or there."""
    M, K = A.shape
    N = W.shape[0]
    _check(load().swiftkv_op_gemm_rows_static(_dev(A, torch.bfloat16), _dev(W, torch.bfloat16), _dev(out), M, N, K,
                                              int(out.dtype == torch.float32), _stream_ptr(stream)))
    return out


def op_attention_prefill(q, k, v, seq_lens, n_q_heads, n_kv_heads, head_dim, stream=None) -> torch.Tensor:
    T = q.shape[0]
    lib = load()
    nbytes = int(lib.swiftkv_op_attention_workspace(T, len(seq_lens), n_kv_heads, head_dim))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    out = torch.empty_like(q)
    _check(lib.swiftkv_op_attention_prefill(_dev(q, torch.bfloat16), _dev(k, torch.bfloat16), _dev(v, torch.bfloat16),
                                            _dev(out), _i32_array(seq_lens), len(seq_lens), n_q_heads, n_kv_heads,
                                            head_dim, _dev(ws), nbytes, _stream_ptr(stream)))
    return out


def op_attention_decode(q: torch.Tensor, n_keys: Sequence[int], cache_k: torch.Tensor, cache_v: torch.Tensor,
                        block_tables: torch.Tensor, n_q_heads: int, n_kv_heads: int, head_dim: int,
                        scale_k: Optional[torch.Tensor] = None, scale_v: Optional[torch.Tensor] = None,
                        per_token: bool = False, stream=None) -> torch.Tensor:
    """Single-query attention of each row of q over its block-table row of one cache layer's K / V planes
    ([n_blocks*16, Hkv, hd], bf16 or uint8 e4m3 codes with scales)."""
    lib = load()
    n_rows = q.shape[0]
    fp8 = cache_k.dtype == torch.uint8
    ws = torch.empty(int(lib.swiftkv_op_attention_decode_workspace(n_rows, n_q_heads, head_dim)), dtype=torch.uint8, device=q.device)
    out = torch.empty_like(q)
    bt = block_tables.to(device=q.device, dtype=torch.int32).contiguous()
    _check(lib.swiftkv_op_attention_decode(
        _dev(q, torch.bfloat16), _dev(out), _i32_array(n_keys), n_rows, n_q_heads, n_kv_heads, head_dim,
        _dev(cache_k), _dev(cache_v), SWIFTKV_KV_FP8_E4M3 if fp8 else SWIFTKV_KV_BF16,
        SWIFTKV_SCALE_PER_TOKEN if per_token else SWIFTKV_SCALE_USE_GIVEN,
        _dev(scale_k, torch.float32) if fp8 else None, _dev(scale_v, torch.float32) if fp8 else None,
        _dev(bt), bt.shape[1], cache_k.shape[0] // 16, _dev(ws), ws.numel(), _stream_ptr(stream)))
    return out


def op_fp8_quantize(x: torch.Tensor, scale: float, stream=None) -> torch.Tensor:
    codes = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(load().swiftkv_op_fp8_quantize(_dev(x, torch.float32), float(scale), _dev(codes), x.numel(),
                                          _stream_ptr(stream)))
    return codes
