"""ctypes binding of libsssd_verify.so: same names as the C ABI, argument
marshalling only.  PyTorch supplies device memory and streams; every step of
the verification path runs in the library's HIP kernels.  There is no CPU or
PyTorch fallback: a missing library is an ImportError."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsssd_verify.so")

SSSD_OK, SSSD_EINVAL, SSSD_ECAPACITY, SSSD_ENOSPACE, SSSD_EHIP = 0, -1, -2, -3, -4
SSSD_PACK_IN_PLACE = 1
SSSD_PROF_CLASSES = 8
PROF_NAMES = ("gemm", "attention", "elementwise", "accept")


class SssdError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_batch", "max_k", "max_seq")]


class SamplingParams(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_int32), ("top_p", C.c_float)]


_PER_LAYER = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "mlp_norm")


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "lm_head", "final_norm")] + \
               [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises ImportError if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2411_05894_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        l = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        l.sssd_strerror.restype = C.c_char_p
        l.sssd_strerror.argtypes = [C.c_int]
        l.sssd_verify_sizes.argtypes = [C.POINTER(ModelConfig), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        l.sssd_verify_plan_check.argtypes = [C.POINTER(ModelConfig), i32, i32]
        l.sssd_verify_init.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), vp, sz, vp, sz, vp, sz,
                                       C.c_uint32, C.POINTER(vp)]
        l.sssd_verify_step.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
        l.sssd_kv_rollback.argtypes = [vp, i32, vp, vp, vp, vp]
        l.sssd_verify_step_tree.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        l.sssd_kv_commit_tree.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        l.sssd_verify_step_tree_sampled.argtypes = [vp, i32, i32, vp, vp, vp, C.POINTER(SamplingParams), vp, vp, vp, vp, vp, vp]
        l.sssd_op_gemm_static.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        l.sssd_op_gemm_static_scratch_limit.argtypes = []
        l.sssd_op_gemm_static_scratch_limit.restype = sz
        l.sssd_op_gemm_small_step_rows.argtypes = []
        l.sssd_op_gemm_small_step_rows.restype = i32
        l.sssd_op_gemm_kernel_name.argtypes = [i32]
        l.sssd_op_gemm_kernel_name.restype = C.c_char_p
        l.sssd_op_stream_read.argtypes = [vp, sz, vp, vp]
        l.sssd_op_sample_scratch_bytes.argtypes = [i32]
        l.sssd_op_sample_scratch_bytes.restype = sz
        l.sssd_op_sample_wide.argtypes = [vp, i32, i32, C.POINTER(SamplingParams), vp, vp, vp, sz, vp]
        l.sssd_op_sample.argtypes = [vp, i32, i32, C.POINTER(SamplingParams), vp, vp, vp]
        l.sssd_verify_sync.argtypes = [vp, vp]
        l.sssd_kv_geometry.argtypes = [C.POINTER(ModelConfig), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        l.sssd_kv_set_block_table.argtypes = [vp, vp]
        l.sssd_debug_outputs.argtypes = [vp, vp, vp]
        l.sssd_debug_logits.argtypes = [vp, vp]
        l.sssd_debug_argmax.argtypes = [vp, vp]
        l.sssd_kv_import.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        l.sssd_kv_export.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        l.sssd_profile_enable.argtypes = [vp, i32]
        l.sssd_profile_read.argtypes = [vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        l.sssd_verify_destroy.argtypes = [vp]
        l.sssd_op_packed_weight_bytes.restype = sz
        l.sssd_op_packed_weight_bytes.argtypes = [i32, i32]
        l.sssd_op_packed_act_bytes.restype = sz
        l.sssd_op_packed_act_bytes.argtypes = [i32, i32]
        l.sssd_op_pack_weight.argtypes = [vp, vp, i32, i32, vp]
        l.sssd_op_pack_activation.argtypes = [vp, i32, i32, vp, vp, vp]
        l.sssd_op_gemm_scratch_bytes.argtypes = [i32, i32, i32]
        l.sssd_op_gemm_scratch_bytes.restype = C.c_size_t
        l.sssd_op_gemm.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, C.c_size_t, vp]
        l.sssd_op_attention.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().sssd_strerror(code).decode()


def _check(code: int, what: str) -> None:
    if code != SSSD_OK:
        raise SssdError(code, what)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device pointers must come from contiguous CUDA tensors"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_config(shape, max_batch: int, max_k: int, max_seq: int) -> ModelConfig:
    return ModelConfig(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                       shape.vocab, shape.rms_eps, shape.rope_base, max_batch, max_k, max_seq)


def sssd_verify_sizes(cfg: ModelConfig):
    kv, ws, pk = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().sssd_verify_sizes(C.byref(cfg), C.byref(kv), C.byref(ws), C.byref(pk)), "sssd_verify_sizes")
    return kv.value, ws.value, pk.value


def sssd_kv_geometry(cfg: ModelConfig):
    rows, bps, pages = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().sssd_kv_geometry(C.byref(cfg), C.byref(rows), C.byref(bps), C.byref(pages)), "sssd_kv_geometry")
    return rows.value, bps.value, pages.value


class VerifyContext:
    """Owns the device buffers (as torch tensors) and the sssd_ctx handle."""

    def __init__(self, cfg: ModelConfig, layers: Sequence[Dict[str, torch.Tensor]], globals_: Dict[str, torch.Tensor],
                 in_place: bool = False, device: str = "cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        kv_b, ws_b, pk_b = sssd_verify_sizes(cfg)
        self.kv_cache = torch.empty(kv_b, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(ws_b, dtype=torch.uint8, device=self.device)
        self.packed = None if in_place else torch.empty(pk_b, dtype=torch.uint8, device=self.device)
        # embed and the norm vectors are used where they are; with in_place every matrix is.
        self._keep = [globals_["embed"], globals_["final_norm"]] + \
                     [l[n] for l in layers for n in ("attn_norm", "mlp_norm")]
        if in_place:
            self._keep += [l[n] for l in layers for n in _PER_LAYER] + [globals_["lm_head"]]
        w = Weights()
        w.embed, w.lm_head, w.final_norm = (_ptr(globals_[n]) for n in ("embed", "lm_head", "final_norm"))
        self._arrays = []
        for n in _PER_LAYER:
            arr = (C.c_void_p * cfg.n_layers)(*[_ptr(l[n]) for l in layers])
            self._arrays.append(arr)
            setattr(w, n, arr)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().sssd_verify_init(C.byref(cfg), C.byref(w), _ptr(self.kv_cache), kv_b, _ptr(self.workspace),
                                          ws_b, _ptr(self.packed), pk_b if self.packed is not None else 0,
                                          SSSD_PACK_IN_PLACE if in_place else 0, C.byref(h)), "sssd_verify_init")
        self.handle = h

    # -- the C ABI, one method per entry point --
    def sssd_verify_step(self, tokens: torch.Tensor, lens: torch.Tensor, accepted_len: torch.Tensor,
                         next_token: torch.Tensor) -> None:
        B, sq = tokens.shape
        for t in (tokens, lens, accepted_len, next_token):
            assert t.dtype == torch.int32
        _check(lib().sssd_verify_step(self.handle, B, sq - 1, _ptr(tokens), _ptr(lens), _ptr(accepted_len),
                                      _ptr(next_token), _stream()), "sssd_verify_step")

    def sssd_verify_step_tree(self, tokens: torch.Tensor, parents: torch.Tensor, lens: torch.Tensor,
                              accepted_len: torch.Tensor, next_token: torch.Tensor, accepted_path: torch.Tensor) -> None:
        B, sq = tokens.shape
        assert parents.shape == tokens.shape and accepted_path.shape == tokens.shape
        for t in (tokens, parents, lens, accepted_len, next_token, accepted_path):
            assert t.dtype == torch.int32
        _check(lib().sssd_verify_step_tree(self.handle, B, sq - 1, _ptr(tokens), _ptr(parents), _ptr(lens),
                                           _ptr(accepted_len), _ptr(next_token), _ptr(accepted_path), _stream()),
               "sssd_verify_step_tree")

    def sssd_verify_step_tree_sampled(self, tokens: torch.Tensor, parents: torch.Tensor, lens: torch.Tensor,
                                      sampling: SamplingParams, uniforms: torch.Tensor, logits_scratch: torch.Tensor,
                                      accepted_len: torch.Tensor, next_token: torch.Tensor,
                                      accepted_path: torch.Tensor) -> None:
        B, sq = tokens.shape
        assert parents.shape == tokens.shape and accepted_path.shape == tokens.shape and uniforms.shape == tokens.shape
        assert uniforms.dtype == torch.float32 and logits_scratch.dtype == torch.float32
        assert logits_scratch.numel() >= B * sq * self.cfg.vocab
        for t in (tokens, parents, lens, accepted_len, next_token, accepted_path):
            assert t.dtype == torch.int32
        _check(lib().sssd_verify_step_tree_sampled(self.handle, B, sq - 1, _ptr(tokens), _ptr(parents), _ptr(lens),
                                                   C.byref(sampling), _ptr(uniforms), _ptr(logits_scratch),
                                                   _ptr(accepted_len), _ptr(next_token), _ptr(accepted_path), _stream()),
               "sssd_verify_step_tree_sampled")

    def sssd_kv_commit_tree(self, lens: torch.Tensor, accepted_len: torch.Tensor, accepted_path: torch.Tensor) -> None:
        B, sq = accepted_path.shape
        for t in (lens, accepted_len, accepted_path):
            assert t.dtype == torch.int32
        _check(lib().sssd_kv_commit_tree(self.handle, B, sq - 1, _ptr(lens), _ptr(accepted_len), _ptr(accepted_path),
                                         _stream()), "sssd_kv_commit_tree")

    def sssd_kv_rollback(self, lens: torch.Tensor, accepted_len: Optional[torch.Tensor] = None,
                         new_lens: Optional[torch.Tensor] = None) -> None:
        _check(lib().sssd_kv_rollback(self.handle, lens.numel(), _ptr(lens), _ptr(accepted_len), _ptr(new_lens),
                                      _stream()), "sssd_kv_rollback")

    def sssd_kv_set_block_table(self, block_table: Optional[torch.Tensor]) -> None:
        if block_table is not None:
            assert block_table.dtype == torch.int32
        self._block_table = block_table          # keep the tensor alive while the library reads it
        _check(lib().sssd_kv_set_block_table(self.handle, _ptr(block_table)), "sssd_kv_set_block_table")

    def sssd_verify_sync(self) -> int:
        return lib().sssd_verify_sync(self.handle, _stream())

    def sssd_debug_outputs(self, logits: Optional[torch.Tensor], hidden: Optional[torch.Tensor]) -> None:
        _check(lib().sssd_debug_outputs(self.handle, _ptr(logits), _ptr(hidden)), "sssd_debug_outputs")

    def sssd_debug_logits(self, logits: Optional[torch.Tensor]) -> None:
        _check(lib().sssd_debug_logits(self.handle, _ptr(logits)), "sssd_debug_logits")

    def sssd_debug_argmax(self, that: Optional[torch.Tensor]) -> None:
        _check(lib().sssd_debug_argmax(self.handle, _ptr(that)), "sssd_debug_argmax")

    def sssd_kv_import(self, layer: int, b: int, t0: int, k_src: torch.Tensor, v_src: torch.Tensor) -> None:
        assert k_src.dtype == torch.bfloat16 and k_src.shape == v_src.shape
        _check(lib().sssd_kv_import(self.handle, layer, b, t0, k_src.shape[1], _ptr(k_src), _ptr(v_src), _stream()),
               "sssd_kv_import")

    def sssd_kv_export(self, layer: int, b: int, t0: int, k_dst: torch.Tensor, v_dst: torch.Tensor) -> None:
        _check(lib().sssd_kv_export(self.handle, layer, b, t0, k_dst.shape[1], _ptr(k_dst), _ptr(v_dst), _stream()),
               "sssd_kv_export")

    def sssd_profile_enable(self, on: bool) -> None:
        _check(lib().sssd_profile_enable(self.handle, int(on)), "sssd_profile_enable")

    def sssd_profile_read(self) -> Dict[str, Dict[str, float]]:
        ms = (C.c_double * SSSD_PROF_CLASSES)()
        n = (C.c_int64 * SSSD_PROF_CLASSES)()
        _check(lib().sssd_profile_read(self.handle, _stream(), ms, n), "sssd_profile_read")
        return {name: {"ms": ms[i], "launches": n[i]} for i, name in enumerate(PROF_NAMES)}

    def sssd_op_attention(self, layer: int, q: torch.Tensor, lens: torch.Tensor, out: torch.Tensor) -> None:
        B, sq = q.shape[0], q.shape[1]
        assert q.dtype == torch.float32 and out.dtype == torch.float32 and lens.dtype == torch.int32
        _check(lib().sssd_op_attention(self.handle, layer, B, sq - 1, _ptr(q), _ptr(lens), _ptr(out), _stream()),
               "sssd_op_attention")

    def sssd_verify_destroy(self) -> None:
        if self.handle:
            _check(lib().sssd_verify_destroy(self.handle), "sssd_verify_destroy")
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.sssd_verify_destroy()
        except Exception:
            pass


# -- kernel-level entry points --
def sssd_op_pack_weight(w: torch.Tensor) -> torch.Tensor:
    N, K = w.shape
    assert w.dtype == torch.bfloat16
    out = torch.empty(lib().sssd_op_packed_weight_bytes(N, K), dtype=torch.uint8, device=w.device)
    _check(lib().sssd_op_pack_weight(_ptr(w), _ptr(out), N, K, _stream()), "sssd_op_pack_weight")
    return out


def sssd_op_pack_activation(x: torch.Tensor):
    M, K = x.shape
    assert x.dtype == torch.float32
    nbytes = lib().sssd_op_packed_act_bytes(M, K)
    hi = torch.zeros(nbytes, dtype=torch.uint8, device=x.device)
    lo = torch.zeros(nbytes, dtype=torch.uint8, device=x.device)
    _check(lib().sssd_op_pack_activation(_ptr(x), M, K, _ptr(hi), _ptr(lo), _stream()), "sssd_op_pack_activation")
    return hi, lo


def sssd_op_gemm(a_hi: torch.Tensor, a_lo: torch.Tensor, w_packed: torch.Tensor, M: int, N: int,
                 K: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(M, N, dtype=torch.float32, device=a_hi.device)
    nbytes = lib().sssd_op_gemm_scratch_bytes(M, N, K)
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=a_hi.device)
    _check(lib().sssd_op_gemm(_ptr(a_hi), _ptr(a_lo), _ptr(w_packed), M, N, K, _ptr(out), _ptr(scratch), nbytes,
                              _stream()), "sssd_op_gemm")
    return out


def sssd_op_gemm_static(a_hi: torch.Tensor, a_lo: torch.Tensor, w_packed: torch.Tensor, M: int, N: int, K: int,
                        out: torch.Tensor) -> None:
    """The entry point that allocates nothing: `out` (fp32 [M][N]) is the caller's, nothing is created here."""
    _check(lib().sssd_op_gemm_static(_ptr(a_hi), _ptr(a_lo), _ptr(w_packed), M, N, K, _ptr(out), _stream()),
           "sssd_op_gemm_static")


def sssd_op_gemm_static_scratch_limit() -> int:
    return int(lib().sssd_op_gemm_static_scratch_limit())


def sssd_op_sample(logits: torch.Tensor, sampling: SamplingParams, uniforms: torch.Tensor) -> torch.Tensor:
    rows, vocab = logits.shape
    assert logits.dtype == torch.float32 and uniforms.dtype == torch.float32 and uniforms.numel() == rows
    out = torch.empty(rows, dtype=torch.int32, device=logits.device)
    _check(lib().sssd_op_sample(_ptr(logits), rows, vocab, C.byref(sampling), _ptr(uniforms), _ptr(out), _stream()),
           "sssd_op_sample")
    return out


def sssd_op_sample_wide(logits: torch.Tensor, sampling: SamplingParams, uniforms: torch.Tensor) -> torch.Tensor:
    """sssd_op_sample with several workgroups per row when there are few rows; the scratch is allocated here."""
    rows, vocab = logits.shape
    assert logits.dtype == torch.float32 and uniforms.dtype == torch.float32 and uniforms.numel() == rows
    out = torch.empty(rows, dtype=torch.int32, device=logits.device)
    nbytes = lib().sssd_op_sample_scratch_bytes(rows)
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=logits.device)
    _check(lib().sssd_op_sample_wide(_ptr(logits), rows, vocab, C.byref(sampling), _ptr(uniforms), _ptr(out), _ptr(scratch),
                                     nbytes, _stream()), "sssd_op_sample_wide")
    return out


def sssd_op_gemm_small_step_rows() -> int:
    return int(lib().sssd_op_gemm_small_step_rows())


def sssd_op_gemm_kernel_name(M: int) -> str:
    return lib().sssd_op_gemm_kernel_name(int(M)).decode()


def sssd_op_stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """One read-only pass over `src` (any dtype, contiguous); sink: int32/uint32 tensor of >= 4096 words."""
    assert src.is_contiguous() and sink.numel() >= 4096 and sink.element_size() == 4
    _check(lib().sssd_op_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()),
           "sssd_op_stream_read")
