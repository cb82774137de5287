"""ctypes binding of include/stairs.h.  Function names mirror the C ABI one to one."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstairs.so")
_SOURCES = [os.path.join(_HERE, "csrc", f) for f in ("stairs_kernels.hip", "stairs_api.hip")]

STAIRS_MAX_ROWS = 32
DTYPE_FP32, DTYPE_BF16 = 0, 1

EXPORTED_SYMBOLS = [
    "stairs_strerror", "stairs_last_error", "stairs_init", "stairs_free", "stairs_prefill",
    "draft_propose", "stairs_verify", "stairs_verify_tokens", "stairs_generate", "stairs_decode", "stairs_decode_adaptive", "stairs_reserve_batch", "stairs_generate_batch",
    "stairs_get_tokens", "stairs_set_eos", "stairs_gemm_host", "stairs_gemm_device", "stairs_time_kernel", "stairs_copy_probe",
    "stairs_encdec_init", "stairs_encode", "stairs_encdec_generate",
    "stairs_decode_sampled", "stairs_generate_sampled", "draft_propose_sampled", "stairs_verify_sampled",
    "stairs_rel_bucket",
]


class StairsError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: error {code} ({stairs_strerror(code)}) {detail}".strip())


def build_library(verbose: bool = False) -> str:
    """Compile the HIP sources for gfx950 into libstairs.so next to this file."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *_SOURCES, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return LIB_PATH


class _ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_seq", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wq", C.POINTER(C.c_void_p)),
                ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate", C.POINTER(C.c_void_p)), ("w_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p))]


_ED_LAYER_FIELDS = ["enc_attn_norm", "enc_ffn_norm", "enc_wq", "enc_wk", "enc_wv", "enc_wo", "enc_w_in", "enc_w_out",
                    "dec_attn_norm", "dec_cross_norm", "dec_ffn_norm", "dec_wq", "dec_wk", "dec_wv", "dec_wo",
                    "dec_cq", "dec_ck", "dec_cv", "dec_co", "dec_w_in", "dec_w_out"]


class _EncDecCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_enc_layers", "n_dec_layers", "d_model", "n_heads", "head_dim", "d_ffn",
                                         "vocab", "max_src", "max_seq", "rel_buckets", "rel_max_distance")] + \
               [("rms_eps", C.c_float)]


class _EncDecWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("tok_emb", "lm_head", "enc_rel_bias", "dec_rel_bias", "enc_final_norm",
                                          "dec_final_norm")] + \
               [(n, C.POINTER(C.c_void_p)) for n in _ED_LAYER_FIELDS]


class StairsStats(C.Structure):
    _fields_ = [("iterations", C.c_int32), ("tokens", C.c_int32), ("accepted", C.c_int64),
                ("ms_prefill", C.c_float), ("ms_decode", C.c_float), ("ms_draft", C.c_float),
                ("ms_verify", C.c_float), ("accept_hist", C.c_int32 * (STAIRS_MAX_ROWS + 1))]

    def as_dict(self) -> dict:
        return dict(iterations=self.iterations, tokens=self.tokens, accepted=self.accepted,
                    ms_prefill=self.ms_prefill, ms_decode=self.ms_decode, ms_draft=self.ms_draft,
                    ms_verify=self.ms_verify, accept_hist=list(self.accept_hist))


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first "
                          "(python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(LIB_PATH)
    vp, i32, i32p, f32p = C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    L.stairs_strerror.restype = C.c_char_p
    L.stairs_strerror.argtypes = [C.c_int]
    L.stairs_last_error.restype = C.c_char_p
    L.stairs_last_error.argtypes = [vp]
    L.stairs_init.argtypes = [C.POINTER(vp), C.POINTER(_ModelCfg), C.POINTER(_Weights),
                              C.POINTER(_ModelCfg), C.POINTER(_Weights), i32, vp]
    L.stairs_free.argtypes = [vp]
    L.stairs_free.restype = None
    L.stairs_prefill.argtypes = [vp, i32p, i32]
    L.draft_propose.argtypes = [vp, i32, i32p]
    L.stairs_verify.argtypes = [vp, i32, i32p, i32p, vp]
    L.stairs_verify_tokens.argtypes = [vp, i32p, i32, i32p, i32p, vp]
    L.stairs_generate.argtypes = [vp, i32p, i32, i32, i32, i32p, C.POINTER(StairsStats)]
    L.stairs_decode.argtypes = [vp, i32, i32, i32p, C.POINTER(StairsStats)]
    L.stairs_decode_adaptive.argtypes = [vp, i32, i32, i32p, C.POINTER(StairsStats)]
    L.stairs_set_eos.argtypes = [vp, i32]
    L.stairs_reserve_batch.argtypes = [vp, i32]
    L.stairs_generate_batch.argtypes = [vp, C.POINTER(i32p), i32p, i32, i32, i32, i32p, C.POINTER(StairsStats)]
    L.stairs_get_tokens.argtypes = [vp, i32p, i32, i32p]
    L.stairs_gemm_host.argtypes = [i32, vp, f32p, f32p, i32, i32, i32, vp]
    L.stairs_gemm_device.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp]
    L.stairs_time_kernel.argtypes = [vp, i32, i32, i32, i32, f32p, C.POINTER(C.c_double)]
    L.stairs_copy_probe.argtypes = [C.c_int64, i32, f32p, vp]
    L.stairs_encdec_init.argtypes = [C.POINTER(vp), C.POINTER(_EncDecCfg), C.POINTER(_EncDecWeights),
                                     C.POINTER(_EncDecCfg), C.POINTER(_EncDecWeights), i32, i32, vp]
    L.stairs_encode.argtypes = [vp, i32p, i32]
    L.stairs_rel_bucket.argtypes = [i32, i32, i32, i32]
    L.stairs_decode_sampled.argtypes = [vp, i32, i32, C.c_float, C.c_uint64, i32p, C.POINTER(StairsStats)]
    L.stairs_generate_sampled.argtypes = [vp, i32p, i32, i32, i32, C.c_float, C.c_uint64, i32p, C.POINTER(StairsStats)]
    L.draft_propose_sampled.argtypes = [vp, i32, C.c_float, C.c_uint64, i32p, f32p]
    L.stairs_verify_sampled.argtypes = [vp, i32, C.c_float, C.c_uint64, i32p, i32p, f32p]
    L.stairs_encdec_generate.argtypes = [vp, i32p, i32, i32, i32, i32p, C.POINTER(StairsStats)]
    for name in EXPORTED_SYMBOLS:
        if name not in ("stairs_strerror", "stairs_last_error", "stairs_free"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def stairs_strerror(code: int) -> str:
    return lib().stairs_strerror(code).decode()


def stairs_last_error(ctx) -> str:
    return lib().stairs_last_error(ctx).decode()


def _check(rc: int, where: str, ctx=None):
    if rc != 0:
        raise StairsError(rc, where, stairs_last_error(ctx) if ctx else "")


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _marshal(model, max_seq: int, keep: list):
    """model: object with n_layers, d_model, n_heads, d_ffn, vocab, dtype ('fp32'|'bf16'),
    rope_theta, rms_eps, tok_emb, lm_head, final_norm, layers[list of dict] (numpy arrays)."""
    want = np.uint16 if model.dtype == "bf16" else np.float32

    def mat(a):
        if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
            raise TypeError(f"matrix must be C-contiguous {want.__name__}")
        keep.append(a)
        return a.ctypes.data

    def vec(a):
        if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"]:
            raise TypeError("norm gain must be C-contiguous float32")
        keep.append(a)
        return a.ctypes.data

    cfg = _ModelCfg(model.n_layers, model.d_model, model.n_heads, model.d_ffn, model.vocab, max_seq,
                    float(model.rope_theta), float(model.rms_eps),
                    DTYPE_BF16 if model.dtype == "bf16" else DTYPE_FP32)
    w = _Weights()
    w.tok_emb, w.lm_head, w.final_norm = mat(model.tok_emb), mat(model.lm_head), vec(model.final_norm)
    n = model.n_layers
    for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
        arr = (C.c_void_p * n)()
        for l in range(n):
            t = model.layers[l][name]
            arr[l] = vec(t) if name.endswith("norm") else mat(t)
        keep.append(arr)
        setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
    return cfg, w


def stairs_init(target, draft, k_max: int, max_seq: int, stream: Optional[int] = None):
    keep: list = []
    tcfg, tw = _marshal(target, max_seq, keep)
    ctx = C.c_void_p()
    if draft is not None:
        dcfg, dw = _marshal(draft, max_seq, keep)
        rc = lib().stairs_init(C.byref(ctx), C.byref(tcfg), C.byref(tw), C.byref(dcfg), C.byref(dw), k_max, stream)
    else:
        rc = lib().stairs_init(C.byref(ctx), C.byref(tcfg), C.byref(tw), None, None, k_max, stream)
    _check(rc, "stairs_init")
    return ctx


def stairs_free(ctx):
    lib().stairs_free(ctx)


def stairs_prefill(ctx, prompt: Sequence[int]):
    p = _i32(prompt)
    _check(lib().stairs_prefill(ctx, _ptr(p, C.c_int32), len(p)), "stairs_prefill", ctx)


def draft_propose(ctx, k: int) -> np.ndarray:
    out = np.zeros(max(k, 1), np.int32)
    _check(lib().draft_propose(ctx, k, _ptr(out, C.c_int32)), "draft_propose", ctx)
    return out[:k]


def _logits_arg(logits, k, vocab):
    """None | True (allocate a host array) | int device pointer."""
    if logits is None or logits is False:
        return None, None
    if logits is True:
        buf = np.empty((k + 1, vocab), np.float32)
        return buf, C.c_void_p(buf.ctypes.data)
    return None, C.c_void_p(int(logits))


def stairs_verify(ctx, k: int, vocab: int = 0, logits=None):
    tgt = np.zeros(k + 1, np.int32)
    n = C.c_int32(0)
    buf, lp = _logits_arg(logits, k, vocab)
    _check(lib().stairs_verify(ctx, k, _ptr(tgt, C.c_int32), C.byref(n), lp), "stairs_verify", ctx)
    return tgt, n.value, buf


def stairs_verify_tokens(ctx, draft: Sequence[int], vocab: int = 0, logits=None):
    d = _i32(draft)
    k = len(d)
    tgt = np.zeros(k + 1, np.int32)
    n = C.c_int32(0)
    buf, lp = _logits_arg(logits, k, vocab)
    dp = _ptr(d, C.c_int32) if k else None
    _check(lib().stairs_verify_tokens(ctx, dp, k, _ptr(tgt, C.c_int32), C.byref(n), lp),
           "stairs_verify_tokens", ctx)
    return tgt, n.value, buf


def stairs_generate(ctx, prompt: Sequence[int], G: int, k: int):
    p = _i32(prompt)
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_generate(ctx, _ptr(p, C.c_int32), len(p), G, k, _ptr(out, C.c_int32), C.byref(st)),
           "stairs_generate", ctx)
    return out[:G], st


def stairs_decode_adaptive(ctx, G: int, k_first: int):
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_decode_adaptive(ctx, G, k_first, _ptr(out, C.c_int32), C.byref(st)), "stairs_decode_adaptive", ctx)
    return out[:G], st


def stairs_set_eos(ctx, eos_id: int):
    _check(lib().stairs_set_eos(ctx, eos_id), "stairs_set_eos", ctx)


def stairs_reserve_batch(ctx, max_batch: int):
    _check(lib().stairs_reserve_batch(ctx, max_batch), "stairs_reserve_batch", ctx)


def stairs_generate_batch(ctx, prompts: Sequence[Sequence[int]], G: int, k: int):
    ps = [_i32(p) for p in prompts]
    B = len(ps)
    i32p = C.POINTER(C.c_int32)
    ptrs = (i32p * max(B, 1))(*[_ptr(p, C.c_int32) for p in ps])
    lens = np.array([len(p) for p in ps], np.int32)
    out = np.zeros((max(B, 1), max(G, 1)), np.int32)
    st = StairsStats()
    _check(lib().stairs_generate_batch(ctx, ptrs, _ptr(lens, C.c_int32), B, G, k, _ptr(out, C.c_int32), C.byref(st)),
           "stairs_generate_batch", ctx)
    return out[:B, :G].copy() if G > 0 else np.zeros((B, 0), np.int32), st


def stairs_decode(ctx, G: int, k: int):
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_decode(ctx, G, k, _ptr(out, C.c_int32), C.byref(st)), "stairs_decode", ctx)
    return out[:G], st


def stairs_get_tokens(ctx, cap: int = 1 << 20) -> np.ndarray:
    n = C.c_int32(0)
    _check(lib().stairs_get_tokens(ctx, None, 0, C.byref(n)), "stairs_get_tokens", ctx)
    out = np.zeros(max(1, min(cap, n.value)), np.int32)
    _check(lib().stairs_get_tokens(ctx, _ptr(out, C.c_int32), len(out), C.byref(n)), "stairs_get_tokens", ctx)
    return out[:min(cap, n.value)]


def stairs_gemm_host(W: np.ndarray, X: np.ndarray, stream: Optional[int] = None) -> np.ndarray:
    """Y = X . W^T through the library's GEMM path.  W: uint16 (bf16 bits) or float32 [N, K]."""
    W = np.ascontiguousarray(W)
    X = np.ascontiguousarray(X, dtype=np.float32)
    dt = DTYPE_BF16 if W.dtype == np.uint16 else DTYPE_FP32
    (N, K), M = W.shape, X.shape[0]
    Y = np.empty((M, N), np.float32)
    _check(lib().stairs_gemm_host(dt, C.c_void_p(W.ctypes.data), _ptr(X, C.c_float), _ptr(Y, C.c_float), M, N, K,
                                  stream), "stairs_gemm_host")
    return Y


def stairs_gemm_device(dtype: int, W_dev: int, X_dev: int, Y_dev: int, M: int, N: int, K: int,
                       stream: Optional[int] = None) -> None:
    """stairs_gemm_host on DEVICE addresses (ints) the caller owns, without any allocation inside the library; the
    work is enqueued on `stream` and not waited for."""
    _check(lib().stairs_gemm_device(dtype, C.c_void_p(W_dev), C.c_void_p(X_dev), C.c_void_p(Y_dev), M, N, K, stream),
           "stairs_gemm_device")


def stairs_time_kernel(ctx, which: int, M: int, ctx_len: int, reps: int):
    ms, by = C.c_float(0), C.c_double(0)
    _check(lib().stairs_time_kernel(ctx, which, M, ctx_len, reps, C.byref(ms), C.byref(by)), "stairs_time_kernel", ctx)
    return ms.value, by.value


def stairs_copy_probe(nbytes: int, reps: int = 4, stream: Optional[int] = None) -> float:
    ms = C.c_float(0)
    _check(lib().stairs_copy_probe(nbytes, reps, C.byref(ms), stream), "stairs_copy_probe")
    return ms.value


def _marshal_encdec(model, max_src: int, max_seq: int, keep: list):
    """model: object with the members of synth_inputs.EncDecInputs (numpy arrays; matrices uint16 bf16 bit patterns)."""
    def mat(a):
        if a.dtype != np.uint16 or not a.flags["C_CONTIGUOUS"]:
            raise TypeError("matrix must be C-contiguous uint16 (bfloat16 bit patterns)")
        keep.append(a)
        return a.ctypes.data

    def vec(a):
        if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"]:
            raise TypeError("gains and bias tables must be C-contiguous float32")
        keep.append(a)
        return a.ctypes.data

    cfg = _EncDecCfg(model.n_enc_layers, model.n_dec_layers, model.d_model, model.n_heads, model.head_dim, model.d_ffn,
                     model.vocab, max_src, max_seq, model.rel_buckets, model.rel_max_distance, float(model.rms_eps))
    w = _EncDecWeights()
    w.tok_emb, w.lm_head = mat(model.tok_emb), mat(model.lm_head)
    w.enc_rel_bias, w.dec_rel_bias = vec(model.enc_rel_bias), vec(model.dec_rel_bias)
    w.enc_final_norm, w.dec_final_norm = vec(model.enc_final_norm), vec(model.dec_final_norm)
    for field in _ED_LAYER_FIELDS:
        stack, name = field[:3], field[4:]
        layers = model.enc_layers if stack == "enc" else model.dec_layers
        arr = (C.c_void_p * len(layers))()
        for l, ly in enumerate(layers):
            arr[l] = vec(ly[name]) if name.endswith("norm") else mat(ly[name])
        keep.append(arr)
        setattr(w, field, C.cast(arr, C.POINTER(C.c_void_p)))
    return cfg, w


def stairs_encdec_init(target, draft, k_max: int, max_src: int, max_seq: int, start_token: int = 0,
                       stream: Optional[int] = None):
    keep: list = []
    tcfg, tw = _marshal_encdec(target, max_src, max_seq, keep)
    ctx = C.c_void_p()
    if draft is not None:
        dcfg, dw = _marshal_encdec(draft, max_src, max_seq, keep)
        rc = lib().stairs_encdec_init(C.byref(ctx), C.byref(tcfg), C.byref(tw), C.byref(dcfg), C.byref(dw), k_max,
                                      start_token, stream)
    else:
        rc = lib().stairs_encdec_init(C.byref(ctx), C.byref(tcfg), C.byref(tw), None, None, k_max, start_token, stream)
    _check(rc, "stairs_encdec_init")
    return ctx


def stairs_rel_bucket(rel: int, two_sided: bool, buckets: int, max_distance: int) -> int:
    return lib().stairs_rel_bucket(rel, 1 if two_sided else 0, buckets, max_distance)


def stairs_encode(ctx, src: Sequence[int]):
    p = _i32(src)
    _check(lib().stairs_encode(ctx, _ptr(p, C.c_int32), len(p)), "stairs_encode", ctx)


def stairs_encdec_generate(ctx, src: Sequence[int], G: int, k: int):
    p = _i32(src)
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_encdec_generate(ctx, _ptr(p, C.c_int32), len(p), G, k, _ptr(out, C.c_int32), C.byref(st)),
           "stairs_encdec_generate", ctx)
    return out[:G], st


def stairs_decode_sampled(ctx, G: int, k: int, temperature: float, seed: int):
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_decode_sampled(ctx, G, k, temperature, seed, _ptr(out, C.c_int32), C.byref(st)),
           "stairs_decode_sampled", ctx)
    return out[:G], st


def stairs_generate_sampled(ctx, prompt: Sequence[int], G: int, k: int, temperature: float, seed: int):
    p = _i32(prompt)
    out = np.zeros(max(G, 1), np.int32)
    st = StairsStats()
    _check(lib().stairs_generate_sampled(ctx, _ptr(p, C.c_int32), len(p), G, k, temperature, seed, _ptr(out, C.c_int32),
                                         C.byref(st)), "stairs_generate_sampled", ctx)
    return out[:G], st


def draft_propose_sampled(ctx, k: int, temperature: float, seed: int, vocab: int = 0):
    """-> (k tokens, their logits rows [k, vocab] or None when vocab == 0)."""
    out = np.zeros(max(k, 1), np.int32)
    lg = np.empty((k, vocab), np.float32) if vocab else None
    _check(lib().draft_propose_sampled(ctx, k, temperature, seed, _ptr(out, C.c_int32),
                                       _ptr(lg, C.c_float) if vocab else None), "draft_propose_sampled", ctx)
    return out[:k], lg


def stairs_verify_sampled(ctx, k: int, temperature: float, seed: int, vocab: int = 0):
    """-> (emitted tokens (n + 1), n, main-model logits [k+1, vocab] or None when vocab == 0)."""
    out = np.zeros(k + 1, np.int32)
    n = C.c_int32(0)
    lg = np.empty((k + 1, vocab), np.float32) if vocab else None
    _check(lib().stairs_verify_sampled(ctx, k, temperature, seed, _ptr(out, C.c_int32), C.byref(n),
                                       _ptr(lg, C.c_float) if vocab else None), "stairs_verify_sampled", ctx)
    return out[:n.value + 1], n.value, lg


class Stairs:
    """Convenience wrapper owning one context."""

    def __init__(self, target, draft=None, k_max: int = 0, max_seq: int = 1024, stream: Optional[int] = None):
        self.vocab = target.vocab
        self.ctx = stairs_init(target, draft, k_max, max_seq, stream)

    def close(self):
        if self.ctx is not None:
            stairs_free(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, prompt):
        stairs_prefill(self.ctx, prompt)

    def propose(self, k):
        return draft_propose(self.ctx, k)

    def verify(self, k, logits=None):
        return stairs_verify(self.ctx, k, self.vocab, logits)

    def verify_tokens(self, draft, logits=None):
        return stairs_verify_tokens(self.ctx, draft, self.vocab, logits)

    def generate(self, prompt, G, k):
        return stairs_generate(self.ctx, prompt, G, k)

    def decode(self, G, k):
        return stairs_decode(self.ctx, G, k)

    def decode_adaptive(self, G, k_first):
        return stairs_decode_adaptive(self.ctx, G, k_first)

    def set_eos(self, eos_id):
        stairs_set_eos(self.ctx, eos_id)

    def reserve_batch(self, max_batch):
        stairs_reserve_batch(self.ctx, max_batch)

    def generate_batch(self, prompts, G, k):
        return stairs_generate_batch(self.ctx, prompts, G, k)

    def tokens(self):
        return stairs_get_tokens(self.ctx)

    def decode_sampled(self, G, k, temperature, seed):
        return stairs_decode_sampled(self.ctx, G, k, temperature, seed)

    def generate_sampled(self, prompt, G, k, temperature, seed):
        return stairs_generate_sampled(self.ctx, prompt, G, k, temperature, seed)

    def propose_sampled(self, k, temperature, seed, logits=True):
        return draft_propose_sampled(self.ctx, k, temperature, seed, self.vocab if logits else 0)

    def verify_sampled(self, k, temperature, seed, logits=True):
        return stairs_verify_sampled(self.ctx, k, temperature, seed, self.vocab if logits else 0)

    def time_kernel(self, which, M, ctx_len=0, reps=64):
        return stairs_time_kernel(self.ctx, which, M, ctx_len, reps)


class StairsEncDec(Stairs):
    """Wrapper owning one encoder-decoder context: encode() starts a sequence, the decoding calls are Stairs'."""

    def __init__(self, target, draft=None, k_max: int = 0, max_src: int = 512, max_seq: int = 1024, start_token: int = 0,
                 stream: Optional[int] = None):
        self.vocab = target.vocab
        self.ctx = stairs_encdec_init(target, draft, k_max, max_src, max_seq, start_token, stream)

    def encode(self, src):
        stairs_encode(self.ctx, src)

    def generate(self, src, G, k):
        return stairs_encdec_generate(self.ctx, src, G, k)
