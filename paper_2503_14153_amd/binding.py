"""ctypes binding of libspecdec.so: same names as the C ABI, marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = [
    "sd_model_create", "sd_model_destroy", "sd_kv_bytes", "sd_kv_create", "sd_kv_destroy", "sd_kv_len",
    "sd_kv_set_len", "sd_kv_write_rows", "sd_kv_read_rows", "sd_kv_set_draft", "sd_kv_get_draft",
    "sd_tree_create", "sd_tree_destroy", "sd_prefill", "sd_spec_step", "sd_greedy_step", "sd_verify_tree",
    "sd_kv_commit_rows", "sd_spec_step_typical", "sd_verify_tree_typical", "sd_verify_tree_typical_static", "sd_sample_tokens", "sd_build_labels",
    "sd_set_graph_mode", "sd_set_draft_schedule", "sd_set_greedy_drafts", "sd_set_fused", "sd_set_sync_timeout", "sd_set_layer_timeline", "sd_profile_begin", "sd_profile_end", "sd_last_error", "sd_version",
]

SD_ERR = {-1: "SD_ERR_NULL", -2: "SD_ERR_SHAPE", -3: "SD_ERR_BAD_TREE", -4: "SD_ERR_KV_FULL", -5: "SD_ERR_HIP",
          -6: "SD_ERR_STATE"}


class SpecDecError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{SD_ERR.get(code, code)}: {message}")
        self.code = code
        self.name = SD_ERR.get(code, str(code))


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "n_medusa",
                                         "topk", "dtype", "trunc_fallback")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate", "w_up", "w_down",
                                                     "medusa_w", "medusa_b")]


class _StepIO(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("n_accept", "tokens", "src_slots", "n_accept_raw", "logits", "argmax",
                                          "head_logits", "forced_cand")]


class _Typical(C.Structure):
    _fields_ = [("temperature", C.c_float), ("epsilon", C.c_float), ("delta", C.c_float), ("u", C.c_void_p),
                ("row_stats", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(_HERE, "libspecdec.so")


def lib() -> C.CDLL:
    """Load libspecdec.so (once). There is no fallback: without the library nothing runs."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2503_14153_amd.build`")
        L = C.CDLL(path)
        L.sd_last_error.restype = C.c_char_p
        L.sd_version.restype = C.c_char_p
        L.sd_kv_bytes.restype = C.c_size_t
        L.sd_kv_bytes.argtypes = [C.POINTER(_Config), C.c_int32, C.c_int32]
        L.sd_model_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.c_int32, C.c_void_p,
                                      C.POINTER(C.c_void_p)]
        L.sd_model_destroy.argtypes = [C.c_void_p]
        L.sd_kv_create.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
        L.sd_kv_destroy.argtypes = [C.c_void_p]
        L.sd_kv_len.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
        L.sd_kv_set_len.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
        rows = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sd_kv_write_rows.argtypes = rows
        L.sd_kv_read_rows.argtypes = rows
        L.sd_kv_set_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sd_kv_get_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        i32p = C.POINTER(C.c_int32)
        L.sd_tree_create.argtypes = [C.c_int32, i32p, i32p, i32p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        L.sd_tree_destroy.argtypes = [C.c_void_p]
        L.sd_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, i32p, C.c_void_p]
        L.sd_spec_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_StepIO), C.c_void_p]
        L.sd_greedy_step.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(_StepIO), C.c_void_p]
        L.sd_verify_tree.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 8
        L.sd_kv_commit_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.sd_spec_step_typical.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_StepIO),
                                           C.POINTER(_Typical), C.c_void_p]
        L.sd_verify_tree_typical.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                             C.c_void_p, C.c_float, C.c_float, C.c_float] + [C.c_void_p] * 7
        L.sd_verify_tree_typical_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                                    C.c_void_p, C.c_float, C.c_float, C.c_float] + [C.c_void_p] * 6
        L.sd_sample_tokens.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                       C.c_float, C.c_void_p, C.c_void_p]
        L.sd_build_labels.argtypes = [C.c_void_p] + [C.c_int32] * 7 + [C.c_void_p, C.c_void_p]
        L.sd_profile_begin.argtypes = [C.c_void_p, C.c_int32]
        L.sd_set_graph_mode.argtypes = [C.c_void_p, C.c_int32]
        L.sd_set_draft_schedule.argtypes = [C.c_void_p, C.c_int32]
        L.sd_set_greedy_drafts.argtypes = [C.c_void_p, C.c_int32]
        L.sd_set_fused.argtypes = [C.c_void_p, C.c_int32]
        L.sd_set_sync_timeout.argtypes = [C.c_void_p, C.c_int64]
        L.sd_set_layer_timeline.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.sd_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                     C.POINTER(C.c_double)]
        _LIB = L
    return _LIB


def _check(rc: int):
    if rc != 0:
        raise SpecDecError(rc, lib().sd_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _i32_array(values):
    values = [int(v) for v in values]
    return (C.c_int32 * len(values))(*values)


def _config(shape, trunc_fallback: str) -> _Config:
    return _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                   shape.n_medusa, shape.topk, 1 if shape.dtype == "bf16" else 0,
                   {"keep_all": 0, "keep_one": 1}[trunc_fallback], shape.rope_theta, shape.rms_eps)


class Model:
    """sd_model_create / sd_model_destroy. `weights`: name -> CUDA tensor [out, in] of the shape's dtype
    (bfloat16 for "bf16", float32 for "f32": the float32 path keeps weights, activations and the cache in float32)."""

    def __init__(self, shape, weights: dict, max_rows: int, trunc_fallback: str = "keep_all"):
        self.shape = shape
        self.cfg = _config(shape, trunc_fallback)
        L, H = shape.n_layers, shape.n_medusa

        def arr(names):
            return (C.c_void_p * len(names))(*[weights[n].data_ptr() for n in names])

        self.torch_dtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        for name, t in weights.items():
            if not (t.is_cuda and t.dtype == self.torch_dtype and t.is_contiguous()):
                raise ValueError(f"weight {name} must be a contiguous {shape.dtype} CUDA tensor")
        keep = [arr([f"l{l}.{k}" for l in range(L)]) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate",
                                                             "w_up", "w_down")]
        mw = arr([f"medusa{i}.w" for i in range(H)])
        mb = arr([f"medusa{i}.b" for i in range(H)])
        w = _Weights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(), weights["final_norm"].data_ptr(),
                     *[C.cast(a, C.POINTER(C.c_void_p)) for a in keep],
                     C.cast(mw, C.POINTER(C.c_void_p)), C.cast(mb, C.POINTER(C.c_void_p)))
        self.handle = C.c_void_p()
        _check(lib().sd_model_create(C.byref(self.cfg), C.byref(w), max_rows, _stream(), C.byref(self.handle)))

    def set_graph_mode(self, on: bool):
        _check(lib().sd_set_graph_mode(self.handle, 1 if on else 0))

    def set_draft_schedule(self, schedule: str):
        """"after_accept" (default) or "all_nodes": where in a step the draft heads run."""
        _check(lib().sd_set_draft_schedule(self.handle, {"after_accept": 0, "all_nodes": 1}[schedule]))

    def set_greedy_drafts(self, on: bool):
        """Whether sd_greedy_step also runs the draft heads (default) or leaves the carried candidates alone."""
        _check(lib().sd_set_greedy_drafts(self.handle, 1 if on else 0))

    def set_fused(self, on: bool):
        """The optional persistent layer kernel (True) or one launch per stage (False, the default and the faster
        of the two); the two agree within the parity tolerance, not bit for bit."""
        _check(lib().sd_set_fused(self.handle, 1 if on else 0))

    def set_layer_timeline(self, buf: torch.Tensor | None):
        """Diagnostic time stamps of the layer kernel into an int64 CUDA tensor [launches, 24, 256] (None: off)."""
        if buf is None:
            _check(lib().sd_set_layer_timeline(self.handle, None, 0))
        else:
            assert buf.is_cuda and buf.dtype == torch.int64 and buf.is_contiguous()
            _check(lib().sd_set_layer_timeline(self.handle, buf.data_ptr(), buf.numel() * 8))
        self._timeline = buf

    def set_sync_timeout(self, microseconds: int):
        _check(lib().sd_set_sync_timeout(self.handle, int(microseconds)))

    def profile_begin(self, max_launches: int = 65536):
        _check(lib().sd_profile_begin(self.handle, max_launches))

    def profile_end(self) -> dict:
        ms, n, by = (C.c_double * 2)(), (C.c_int64 * 2)(), (C.c_double * 2)()
        _check(lib().sd_profile_end(self.handle, _stream(), ms, n, by))
        return {name: {"ms": ms[i], "launches": n[i], "bytes": by[i]} for i, name in enumerate(("gemm", "attn"))}

    def close(self):
        if getattr(self, "handle", None):
            lib().sd_model_destroy(self.handle)
            self.handle = None

    __del__ = close


class KVCache:
    """sd_kv_*: the cache buffer is a torch allocation; its tiling is private to the library."""

    def __init__(self, model: Model, batch: int, cap: int, buf: torch.Tensor | None = None):
        """`buf`: a uint8 CUDA tensor of at least sd_kv_bytes bytes to hold the cache (its old contents do
        not matter: sd_kv_create clears it); allocated here when None."""
        self.model, self.batch, self.cap = model, batch, cap
        nbytes = lib().sd_kv_bytes(C.byref(model.cfg), batch, cap)
        if buf is None:
            buf = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        assert buf.is_cuda and buf.dtype == torch.uint8 and buf.is_contiguous() and buf.numel() >= nbytes
        self.buf = buf
        self.handle = C.c_void_p()
        _check(lib().sd_kv_create(model.handle, batch, cap, self.buf.data_ptr(), nbytes, C.byref(self.handle)))

    def len(self) -> list[int]:
        out = (C.c_int32 * self.batch)()
        _check(lib().sd_kv_len(self.handle, out, _stream()))
        return list(out)

    def set_len(self, lens):
        _check(lib().sd_kv_set_len(self.handle, _i32_array(lens), _stream()))

    def write_rows(self, layer, seq, row0, k_rows, v_rows):
        assert k_rows.dtype == v_rows.dtype == self.model.torch_dtype and k_rows.is_cuda and v_rows.is_cuda
        assert k_rows.is_contiguous() and v_rows.is_contiguous() and k_rows.shape == v_rows.shape
        _check(lib().sd_kv_write_rows(self.handle, layer, seq, row0, k_rows.shape[0], k_rows.data_ptr(),
                                      v_rows.data_ptr(), _stream()))

    def read_rows(self, layer, seq, row0, nrows):
        s = self.model.shape
        k = torch.empty((nrows, s.n_heads, s.head_dim), dtype=self.model.torch_dtype, device="cuda")
        v = torch.empty_like(k)
        _check(lib().sd_kv_read_rows(self.handle, layer, seq, row0, nrows, k.data_ptr(), v.data_ptr(), _stream()))
        return k, v

    def set_draft(self, root_tok, cand):
        root_tok = torch.as_tensor(root_tok, dtype=torch.int32).reshape(self.batch).cuda().contiguous()
        s = self.model.shape
        cand = torch.as_tensor(cand, dtype=torch.int32).reshape(self.batch, s.n_medusa, s.topk).cuda().contiguous()
        _check(lib().sd_kv_set_draft(self.handle, root_tok.data_ptr(), cand.data_ptr(), _stream()))
        torch.cuda.current_stream().synchronize()      # the temporaries above die with this frame

    def get_draft(self):
        s = self.model.shape
        root = torch.empty(self.batch, dtype=torch.int32, device="cuda")
        cand = torch.empty((self.batch, s.n_medusa, s.topk), dtype=torch.int32, device="cuda")
        _check(lib().sd_kv_get_draft(self.handle, root.data_ptr(), cand.data_ptr(), _stream()))
        return root, cand

    def close(self):
        if getattr(self, "handle", None):
            lib().sd_kv_destroy(self.handle)
            self.handle = None

    __del__ = close


class Tree:
    """sd_tree_create / sd_tree_destroy."""

    def __init__(self, parent, depth, rank, n_medusa: int, topk: int):
        self.T = len(parent)
        self.n_medusa, self.topk = n_medusa, topk
        self.handle = C.c_void_p()
        _check(lib().sd_tree_create(self.T, _i32_array(parent), _i32_array(depth), _i32_array(rank), n_medusa, topk,
                                    C.byref(self.handle)))

    def close(self):
        if getattr(self, "handle", None):
            lib().sd_tree_destroy(self.handle)
            self.handle = None

    __del__ = close


@dataclass
class StepOutput:
    n_accept: torch.Tensor
    tokens: torch.Tensor
    src_slots: torch.Tensor
    n_accept_raw: torch.Tensor
    logits: torch.Tensor | None = None
    argmax: torch.Tensor | None = None
    head_logits: torch.Tensor | None = None
    row_stats: torch.Tensor | None = None


def prefill(model: Model, kv: KVCache, tokens: torch.Tensor, lens) -> None:
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
    assert int(sum(lens)) == tokens.numel()
    _check(lib().sd_prefill(model.handle, kv.handle, tokens.data_ptr(), _i32_array(lens), _stream()))


def _alloc_io(model, batch, T, want_logits, want_argmax, want_head_logits, forced_cand, out):
    s = model.shape
    W = s.n_medusa + 1
    if out is None:
        i32 = dict(dtype=torch.int32, device="cuda")
        out = StepOutput(torch.empty(batch, **i32), torch.empty((batch, W), **i32), torch.empty((batch, W), **i32),
                         torch.empty(batch, **i32))
        if want_logits:
            out.logits = torch.empty((batch, T, s.vocab), dtype=torch.float32, device="cuda")
        if want_argmax:
            out.argmax = torch.empty((batch, T), **i32)
        if want_head_logits:
            out.head_logits = torch.empty((batch, s.n_medusa, s.vocab), dtype=torch.float32, device="cuda")
    io = _StepIO(_ptr(out.n_accept), _ptr(out.tokens), _ptr(out.src_slots), _ptr(out.n_accept_raw), _ptr(out.logits),
                 _ptr(out.argmax), _ptr(out.head_logits), _ptr(forced_cand))
    return out, io


def spec_step(model: Model, kv: KVCache, tree: Tree, stop_mask: torch.Tensor, *, want_logits=False,
              want_argmax=False, want_head_logits=False, forced_cand: torch.Tensor | None = None,
              out: StepOutput | None = None) -> StepOutput:
    """sd_spec_step. `stop_mask`: int32/uint32 CUDA words (bit id%32 of word id//32). Asynchronous."""
    assert stop_mask.is_cuda and stop_mask.element_size() == 4 and stop_mask.numel() >= (model.shape.vocab + 31) // 32
    if forced_cand is not None:
        assert forced_cand.dtype == torch.int32 and forced_cand.is_cuda and forced_cand.is_contiguous()
        assert forced_cand.numel() == kv.batch * model.shape.n_medusa * model.shape.topk
    out, io = _alloc_io(model, kv.batch, tree.T, want_logits, want_argmax, want_head_logits, forced_cand, out)
    _check(lib().sd_spec_step(model.handle, kv.handle, tree.handle, stop_mask.data_ptr(), C.byref(io), _stream()))
    return out


def spec_step_typical(model: Model, kv: KVCache, tree: Tree, stop_mask: torch.Tensor, u: torch.Tensor, *,
                      temperature: float, epsilon: float, delta: float, want_logits=False, want_argmax=False,
                      want_head_logits=False, want_row_stats=False, forced_cand: torch.Tensor | None = None,
                      out: StepOutput | None = None) -> StepOutput:
    """sd_spec_step_typical: sampling decoding. `u`: fp32 CUDA [batch], uniform numbers in [0, 1)."""
    assert stop_mask.is_cuda and stop_mask.element_size() == 4 and stop_mask.numel() >= (model.shape.vocab + 31) // 32
    assert u.is_cuda and u.dtype == torch.float32 and u.is_contiguous() and u.numel() == kv.batch
    if forced_cand is not None:
        assert forced_cand.dtype == torch.int32 and forced_cand.is_cuda and forced_cand.is_contiguous()
        assert forced_cand.numel() == kv.batch * model.shape.n_medusa * model.shape.topk
    out, io = _alloc_io(model, kv.batch, tree.T, want_logits, want_argmax, want_head_logits, forced_cand, out)
    if want_row_stats and out.row_stats is None:
        out.row_stats = torch.empty((kv.batch, tree.T, 4), dtype=torch.float32, device="cuda")
    ty = _Typical(temperature, epsilon, delta, u.data_ptr(), _ptr(out.row_stats))
    _check(lib().sd_spec_step_typical(model.handle, kv.handle, tree.handle, stop_mask.data_ptr(), C.byref(io),
                                      C.byref(ty), _stream()))
    return out


def greedy_step(model: Model, kv: KVCache, *, want_logits=False, want_head_logits=False,
                out: StepOutput | None = None) -> StepOutput:
    """sd_greedy_step: plain next-token decoding (tree = root only)."""
    out, io = _alloc_io(model, kv.batch, 1, want_logits, False, want_head_logits, None, out)
    _check(lib().sd_greedy_step(model.handle, kv.handle, C.byref(io), _stream()))
    return out


def kv_commit_rows(model: Model, kv: KVCache, src_slots: torch.Tensor, n_rows: torch.Tensor) -> None:
    """sd_kv_commit_rows: append tree rows of the last pass. src_slots int32 CUDA [batch, width], n_rows int32 CUDA [batch]."""
    assert src_slots.dtype == n_rows.dtype == torch.int32 and src_slots.is_cuda and n_rows.is_cuda
    assert src_slots.is_contiguous() and n_rows.is_contiguous()
    assert src_slots.shape[0] == kv.batch and n_rows.numel() == kv.batch
    _check(lib().sd_kv_commit_rows(model.handle, kv.handle, src_slots.data_ptr(), n_rows.data_ptr(), src_slots.shape[1],
                                   _stream()))


def verify_tree(tree: Tree, tok: torch.Tensor, am: torch.Tensor, stop_mask: torch.Tensor, vocab: int,
                trunc_fallback: str = "keep_all"):
    """sd_verify_tree: acceptance + fragment cut alone. tok, am: int32 CUDA [batch, T]."""
    batch = tok.shape[0]
    assert tok.shape == am.shape == (batch, tree.T) and tok.dtype == am.dtype == torch.int32
    assert tok.is_contiguous() and am.is_contiguous() and tok.is_cuda and am.is_cuda
    W = tree.n_medusa + 1
    i32 = dict(dtype=torch.int32, device="cuda")
    n_acc, n_raw = torch.empty(batch, **i32), torch.empty(batch, **i32)
    tokens, slots = torch.empty((batch, W), **i32), torch.empty((batch, W), **i32)
    _check(lib().sd_verify_tree(tree.handle, batch, tree.n_medusa, {"keep_all": 0, "keep_one": 1}[trunc_fallback],
                                vocab, tok.data_ptr(), am.data_ptr(), stop_mask.data_ptr(), n_acc.data_ptr(),
                                n_raw.data_ptr(), tokens.data_ptr(), slots.data_ptr(), _stream()))
    return n_acc, n_raw, tokens, slots


def verify_tree_typical(tree: Tree, tok: torch.Tensor, logits: torch.Tensor, stop_mask: torch.Tensor, *,
                        temperature: float, epsilon: float, delta: float, trunc_fallback: str = "keep_all"):
    """sd_verify_tree_typical: typical acceptance + fragment cut alone. tok int32 CUDA [batch, T], logits fp32
    CUDA [batch, T, vocab]. Returns (n_accept, n_accept_raw, tokens, src_slots, row_stats)."""
    batch, T, vocab = logits.shape
    assert T == tree.T and tok.shape == (batch, T) and tok.dtype == torch.int32 and logits.dtype == torch.float32
    assert tok.is_contiguous() and logits.is_contiguous() and tok.is_cuda and logits.is_cuda
    W = tree.n_medusa + 1
    i32 = dict(dtype=torch.int32, device="cuda")
    n_acc, n_raw = torch.empty(batch, **i32), torch.empty(batch, **i32)
    tokens, slots = torch.empty((batch, W), **i32), torch.empty((batch, W), **i32)
    stats = torch.empty((batch, T, 4), dtype=torch.float32, device="cuda")
    _check(lib().sd_verify_tree_typical(tree.handle, batch, tree.n_medusa,
                                        {"keep_all": 0, "keep_one": 1}[trunc_fallback], vocab, tok.data_ptr(),
                                        logits.data_ptr(), temperature, epsilon, delta, stop_mask.data_ptr(),
                                        stats.data_ptr(), n_acc.data_ptr(), n_raw.data_ptr(), tokens.data_ptr(),
                                        slots.data_ptr(), _stream()))
    return n_acc, n_raw, tokens, slots, stats


def verify_tree_typical_static(tree: Tree, tok: torch.Tensor, logits: torch.Tensor, stop_mask: torch.Tensor, out, *,
                               temperature: float, epsilon: float, delta: float, trunc_fallback: str = "keep_all"):
    """sd_verify_tree_typical_static: as verify_tree_typical, statistics in the library's static buffer.
    `out` = (n_accept, n_accept_raw, tokens, src_slots), int32 CUDA tensors the caller made beforehand:
    nothing is allocated here or in the library."""
    batch, T, vocab = logits.shape
    assert T == tree.T and tok.shape == (batch, T) and tok.dtype == torch.int32 and logits.dtype == torch.float32
    assert tok.is_contiguous() and logits.is_contiguous() and tok.is_cuda and logits.is_cuda
    n_acc, n_raw, tokens, slots = out
    W = tree.n_medusa + 1
    assert n_acc.numel() >= batch and n_raw.numel() >= batch and tokens.numel() >= batch * W and slots.numel() >= batch * W
    _check(lib().sd_verify_tree_typical_static(tree.handle, batch, tree.n_medusa,
                                               {"keep_all": 0, "keep_one": 1}[trunc_fallback], vocab, tok.data_ptr(),
                                               logits.data_ptr(), temperature, epsilon, delta, stop_mask.data_ptr(),
                                               n_acc.data_ptr(), n_raw.data_ptr(), tokens.data_ptr(), slots.data_ptr(),
                                               _stream()))


def sample_tokens(logits: torch.Tensor, rows: torch.Tensor, u: torch.Tensor, temperature: float) -> torch.Tensor:
    """sd_sample_tokens: inverse-CDF draws. logits fp32 CUDA [n_rows, vocab]; rows int32, u fp32 CUDA [n]."""
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
    assert rows.dtype == torch.int32 and u.dtype == torch.float32 and rows.numel() == u.numel()
    assert rows.is_cuda and u.is_cuda and rows.is_contiguous() and u.is_contiguous()
    out = torch.empty(rows.numel(), dtype=torch.int32, device="cuda")
    _check(lib().sd_sample_tokens(logits.data_ptr(), logits.shape[0], logits.stride(0), logits.shape[1],
                                  rows.data_ptr(), u.data_ptr(), rows.numel(), temperature, out.data_ptr(), _stream()))
    return out


def build_labels(l0: torch.Tensor, n_heads: int, frag_id: int, pad_id: int, ignore_id: int = -100,
                 no_frag: str = "keep_base", out: torch.Tensor | None = None) -> torch.Tensor:
    """sd_build_labels: int32 CUDA [batch, seq] -> int32 CUDA [batch, n_heads + 1, seq]."""
    assert l0.is_cuda and l0.dtype == torch.int32 and l0.dim() == 2 and l0.is_contiguous()
    batch, seq = l0.shape
    if out is None:
        out = torch.empty((batch, n_heads + 1, seq), dtype=torch.int32, device="cuda")
    assert out.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and out.shape == (batch, n_heads + 1, seq)
    _check(lib().sd_build_labels(l0.data_ptr(), batch, seq, n_heads, frag_id, pad_id, ignore_id,
                                 {"keep_base": 0, "keep_all": 1}[no_frag], out.data_ptr(), _stream()))
    return out
