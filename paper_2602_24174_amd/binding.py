"""ctypes binding of libtasc.so: the same entry points as include/tasc.h, argument marshalling only.

PyTorch supplies device memory (`torch.empty(..., device="cuda")`) and the current stream; every step of
the path runs in the library's HIP kernels.  There is no CPU fallback: if the library is missing or a
call fails, TascError is raised.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtasc.so")

TASC_OK, TASC_EINVAL, TASC_ENOMEM, TASC_EHIP, TASC_ESTATE = 0, -1, -2, -3, -4
TASC_MEM_HOST, TASC_MEM_DEVICE = 0, 1
TASC_F32, TASC_BF16 = 0, 1
TASC_MAX_ORDER, TASC_MAX_K = 8, 15

EXPORTS = [
    "tasc_last_error", "tasc_ngram_build", "tasc_ngram_destroy", "tasc_ngram_export", "tasc_ngram_export_contexts",
    "tasc_ngram_unigram", "tasc_ngram_get_stats", "tasc_ngram_entropy", "tasc_ngram_entropy_noalloc", "tasc_model_bigram", "tasc_ngram_from_bigram", "tasc_tok_enrich", "tasc_model_create", "tasc_model_destroy", "tasc_session_kv_bytes",
    "tasc_session_workspace_bytes", "tasc_session_create", "tasc_session_destroy", "tasc_session_prefill", "tasc_draft",
    "tasc_verify_step", "tasc_generate", "tasc_session_get_tokens", "tasc_session_status", "tasc_profile_enable", "tasc_profile_read", "tasc_profile_durations", "tasc_config_set", "tasc_profile_phases", "tasc_calibration_copy", "tasc_calibration_mfma", "tasc_calibration_read", "tasc_calibration_handover", "tasc_calibration_gemm",
]
KERNEL_CLASSES = ["draft", "prepare", "norm", "gemm_qkv", "rope_kv", "attn", "gemm_o", "gemm_gu", "gemm_d", "lmhead", "accept",
                  "verify", "layers"]


class TascError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"tasc status {status}: {message}")
        self.status = status


class NgramStats(C.Structure):
    _fields_ = [("n_tokens", C.c_int64), ("windows", C.c_int64 * (TASC_MAX_ORDER + 1)),
                ("distinct", C.c_int64 * (TASC_MAX_ORDER + 1)), ("kept", C.c_int64 * (TASC_MAX_ORDER + 1)),
                ("contexts", C.c_int64 * (TASC_MAX_ORDER + 1)), ("build_ms", C.c_double), ("count_ms", C.c_double)]


class TableEntropy(C.Structure):
    _fields_ = [("n_entries", C.c_int64), ("total", C.c_int64), ("n_cover", C.c_int64), ("shannon", C.c_double),
                ("renyi2", C.c_double)]


class ModelDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("max_pos", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class WeightPtrs(C.Structure):
    _fields_ = [("where", C.c_int32), ("embed", C.c_void_p), ("lm_head", C.c_void_p), ("gf", C.c_void_p),
                ("wq", C.POINTER(C.c_void_p)), ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("wg", C.POINTER(C.c_void_p)), ("wu", C.POINTER(C.c_void_p)),
                ("wd", C.POINTER(C.c_void_p)), ("g1", C.POINTER(C.c_void_p)), ("g2", C.POINTER(C.c_void_p)),
                ("bias_rowptr", C.c_void_p), ("bias_col", C.c_void_p), ("bias_val", C.c_void_p), ("bias_base", C.c_void_p)]


class SpecParams(C.Structure):
    _fields_ = [("k", C.c_int32), ("lambda_q16", C.c_int32), ("p_min_ctx", C.c_int32), ("ctx_includes_generated", C.c_int32)]


class GenStats(C.Structure):
    _fields_ = [("steps", C.c_int64), ("emitted", C.c_int64), ("accepted", C.c_int64), ("proposed", C.c_int64),
                ("accept_hist", C.c_int64 * (TASC_MAX_K + 1)), ("prefill_ms", C.c_double), ("decode_ms", C.c_double),
                ("xcd_local_steps", C.c_int64)]


_lib = None


def lib():
    """Loads libtasc.so (built by paper_2602_24174_amd/build.py or __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise TascError(TASC_EHIP, f"{LIB_PATH} is not built; run `python -m paper_2602_24174_amd.build`")
        # PyTorch first: it supplies the device memory and streams, and the process must end up with ONE HIP
        # runtime.  If libtasc.so pulled in the system's libamdhip64 before torch loaded its own, the runtime
        # that initialises second finds no device.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.tasc_last_error.restype = C.c_char_p
        L.tasc_session_kv_bytes.restype = C.c_size_t
        L.tasc_session_workspace_bytes.restype = C.c_size_t
        L.tasc_session_kv_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.tasc_session_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        L.tasc_ngram_build.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_void_p, C.POINTER(C.c_void_p)]
        L.tasc_ngram_export.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
        L.tasc_ngram_export_contexts.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.POINTER(C.c_int64)]
        L.tasc_ngram_unigram.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
        L.tasc_ngram_get_stats.argtypes = [C.c_void_p, C.POINTER(NgramStats)]
        L.tasc_tok_enrich.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        L.tasc_model_bigram.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tasc_ngram_from_bigram.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
        L.tasc_ngram_entropy.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(TableEntropy), C.c_void_p]
        L.tasc_ngram_entropy_noalloc.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.tasc_model_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(WeightPtrs), C.POINTER(C.c_void_p)]
        L.tasc_session_create.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                          C.c_size_t, C.POINTER(C.c_void_p)]
        L.tasc_session_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.tasc_draft.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(SpecParams), C.c_void_p, C.c_void_p]
        L.tasc_verify_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p]
        L.tasc_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                    C.POINTER(SpecParams), C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(GenStats), C.c_void_p]
        L.tasc_session_get_tokens.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p]
        L.tasc_session_status.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
        L.tasc_config_set.argtypes = [C.c_int32, C.c_int32]
        L.tasc_profile_phases.argtypes = [C.c_void_p, C.c_int64]
        L.tasc_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.tasc_calibration_mfma.argtypes = [C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.tasc_calibration_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.tasc_calibration_handover.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.tasc_calibration_gemm.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.tasc_profile_enable.argtypes = [C.c_uint32]
        L.tasc_profile_read.argtypes = [C.c_void_p, C.c_void_p]
        L.tasc_profile_durations.argtypes = [C.c_int32, C.c_void_p, C.c_int64, C.POINTER(C.c_int64)]
        for name in ("tasc_ngram_destroy", "tasc_model_destroy", "tasc_session_destroy"):
            getattr(L, name).argtypes = [C.c_void_p]
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _check(status):
    if status != TASC_OK:
        raise TascError(status, lib().tasc_last_error().decode())


def _ptr(a):
    """Raw address of a numpy array (host), a torch tensor (host or device) or None."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        assert a.flags["C_CONTIGUOUS"]
        return a.ctypes.data
    assert a.is_contiguous()
    return a.data_ptr()


def _where(a):
    return TASC_MEM_HOST if isinstance(a, np.ndarray) or not a.is_cuda else TASC_MEM_DEVICE


def _stream(stream):
    if stream is not None:
        return stream
    import torch
    return torch.cuda.current_stream().cuda_stream


class Ngram:
    def __init__(self, handle, n_max):
        self.handle, self.n_max = handle, n_max

    def close(self):
        if self.handle:
            lib().tasc_ngram_destroy(self.handle)
            self.handle = None

    __del__ = close


def tasc_ngram_build(tokens, doc_offsets, vocab, n_max, p_min, stream=None) -> Ngram:
    """tokens: int32 numpy array (host) or cuda tensor; doc_offsets: int64 numpy array."""
    doc_offsets = np.ascontiguousarray(doc_offsets, dtype=np.int64)
    out = C.c_void_p()
    _check(lib().tasc_ngram_build(_ptr(tokens), _ptr(doc_offsets), len(doc_offsets) - 1, vocab, n_max, p_min, _where(tokens),
                                  _stream(stream), C.byref(out)))
    return Ngram(out.value, n_max)


def tasc_ngram_export(ng: Ngram, order: int):
    """Returns (ctx_next int32[R, order], counts uint32[R]), rows sorted by their tokens."""
    n = C.c_int64(0)
    _check(lib().tasc_ngram_export(ng.handle, order, None, None, C.byref(n)))
    rows = np.zeros((n.value, order), dtype=np.int32)
    counts = np.zeros(n.value, dtype=np.uint32)
    n = C.c_int64(n.value)
    _check(lib().tasc_ngram_export(ng.handle, order, _ptr(rows), _ptr(counts), C.byref(n)))
    return rows, counts


def tasc_ngram_export_contexts(ng: Ngram, order: int):
    n = C.c_int64(0)
    _check(lib().tasc_ngram_export_contexts(ng.handle, order, None, None, None, None, C.byref(n)))
    ctx = np.zeros((n.value, order - 1), dtype=np.int32)
    total = np.zeros(n.value, dtype=np.uint32)
    top = np.zeros(n.value, dtype=np.int32)
    top_count = np.zeros(n.value, dtype=np.uint32)
    n = C.c_int64(n.value)
    _check(lib().tasc_ngram_export_contexts(ng.handle, order, _ptr(ctx), _ptr(total), _ptr(top), _ptr(top_count), C.byref(n)))
    return ctx, total, top, top_count


def tasc_ngram_unigram(ng: Ngram, vocab: int):
    fb = C.c_int32(0)
    counts = np.zeros(vocab, dtype=np.uint32)
    _check(lib().tasc_ngram_unigram(ng.handle, C.byref(fb), _ptr(counts)))
    return fb.value, counts


def tasc_ngram_entropy(ng: Ngram, order: int, coverage_ppm: int = 800000, stream=None) -> TableEntropy:
    out = TableEntropy()
    _check(lib().tasc_ngram_entropy(ng.handle, order, coverage_ppm, C.byref(out), _stream(stream)))
    return out


def tasc_ngram_entropy_noalloc(ng: Ngram, order: int, coverage_ppm: int, out_device, stream=None):
    """out_device: cuda uint8 tensor of sizeof(TableEntropy) bytes, written on the stream (no synchronisation)."""
    assert out_device.is_cuda and out_device.numel() * out_device.element_size() >= C.sizeof(TableEntropy)
    _check(lib().tasc_ngram_entropy_noalloc(ng.handle, order, coverage_ppm, _ptr(out_device), _stream(stream)))


def tasc_tok_enrich(tokens, doc_offsets, vocab, n_max, budget, stream=None):
    """tokens: int32 numpy array (host) or cuda tensor.  Returns (merges [(ngram tuple, freq, new id)], final tokens
    (same kind as the input, trimmed), final offsets int64[D + 1], corpus lengths int64[n_merges + 1])."""
    doc_offsets = np.ascontiguousarray(doc_offsets, dtype=np.int64)
    n_docs = doc_offsets.shape[0] - 1
    rows = np.zeros((max(budget, 1), 1 + TASC_MAX_ORDER), dtype=np.int32)
    freq = np.zeros(max(budget, 1), dtype=np.int64)
    lens = np.zeros(budget + 1, dtype=np.int64)
    out_off = np.zeros(n_docs + 1, dtype=np.int64)
    if isinstance(tokens, np.ndarray):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        out = np.zeros(max(tokens.shape[0], 1), dtype=np.int32)
    else:
        import torch
        out = torch.zeros(max(tokens.shape[0], 1), dtype=torch.int32, device=tokens.device)
    n = C.c_int32(0)
    _check(lib().tasc_tok_enrich(_ptr(tokens), _ptr(doc_offsets), n_docs, vocab, n_max, budget, _where(tokens), _stream(stream),
                                 _ptr(rows), _ptr(freq), _ptr(lens), _ptr(out), _ptr(out_off), C.byref(n)))
    m = n.value
    merges = [(tuple(int(t) for t in rows[i, 1:1 + rows[i, 0]]), int(freq[i]), vocab + i) for i in range(m)]
    return merges, out[:int(lens[m])], out_off, lens[:m + 1]


def tasc_model_bigram(model: "Model", s: "Session", next_tok, stream=None):
    """next_tok: cuda int32 tensor [vocab], written in place."""
    _check(lib().tasc_model_bigram(model.handle, s.handle, _ptr(next_tok), _stream(stream)))


def tasc_ngram_from_bigram(next_tok, vocab, n_max, stream=None) -> Ngram:
    out = C.c_void_p()
    _check(lib().tasc_ngram_from_bigram(_ptr(next_tok), _where(next_tok), vocab, n_max, _stream(stream), C.byref(out)))
    return Ngram(out.value, n_max)


def tasc_ngram_get_stats(ng: Ngram) -> NgramStats:
    st = NgramStats()
    _check(lib().tasc_ngram_get_stats(ng.handle, C.byref(st)))
    return st


class Model:
    def __init__(self, handle, desc):
        self.handle, self.desc = handle, desc

    def close(self):
        if self.handle:
            lib().tasc_model_destroy(self.handle)
            self.handle = None

    __del__ = close


def tasc_model_create(cfg, weights, max_pos) -> Model:
    """cfg: object with the model fields of workload.WorkloadConfig; weights: the canonical dict of
    numpy arrays (host) from workload.make_model (uint16 arrays are bf16 bit patterns)."""
    desc = ModelDesc(TASC_BF16 if cfg.dtype == "bf16" else TASC_F32, cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads,
                     cfg.head_dim, cfg.d_ffn, cfg.vocab, max_pos, cfg.rope_theta, cfg.rms_eps)
    L = cfg.n_layers

    alive = []

    def arr(name):
        mats = [np.ascontiguousarray(weights["layers"][l][name]) for l in range(L)]
        alive.append(mats)                                   # the library copies during the call
        a = (C.c_void_p * L)(*[_ptr(m) for m in mats])
        return C.cast(a, C.POINTER(C.c_void_p)), a

    keep = {n: arr(n) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")}
    b = weights.get("bias")
    w = WeightPtrs(TASC_MEM_HOST, _ptr(weights["embed"]), _ptr(weights["lm_head"]), _ptr(weights["gf"]),
                   *[keep[n][0] for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")],
                   _ptr(b["rowptr"]) if b else None, _ptr(b["col"]) if b else None, _ptr(b["val"]) if b else None,
                   _ptr(b["base"]) if b else None)
    out = C.c_void_p()
    _check(lib().tasc_model_create(C.byref(desc), C.byref(w), C.byref(out)))
    return Model(out.value, desc)


class Session:
    def __init__(self, handle, model, batch, max_len, max_rows, kv_pool, workspace):
        self.handle, self.model, self.batch, self.max_len, self.max_rows = handle, model, batch, max_len, max_rows
        self._kv_pool, self._workspace = kv_pool, workspace     # keep the caller-owned buffers alive

    def close(self):
        if self.handle:
            lib().tasc_session_destroy(self.handle)
            self.handle = None

    __del__ = close


def tasc_session_kv_bytes(model: Model, batch, max_len) -> int:
    return lib().tasc_session_kv_bytes(model.handle, batch, max_len)


def tasc_session_workspace_bytes(model: Model, batch, max_len, max_rows) -> int:
    return lib().tasc_session_workspace_bytes(model.handle, batch, max_len, max_rows)


def tasc_session_create(model: Model, batch, max_len, max_rows) -> Session:
    """Allocates the KV pool and the workspace through PyTorch and hands them to the library."""
    import torch
    kvb = tasc_session_kv_bytes(model, batch, max_len)
    wsb = tasc_session_workspace_bytes(model, batch, max_len, max_rows)
    kv = torch.empty(kvb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    out = C.c_void_p()
    _check(lib().tasc_session_create(model.handle, batch, max_len, max_rows, kv.data_ptr(), kvb, ws.data_ptr(), wsb, C.byref(out)))
    return Session(out.value, model, batch, max_len, max_rows, kv, ws)


def tasc_session_prefill(model: Model, s: Session, prompts, prompt_offsets, max_new, stream=None):
    prompt_offsets = np.ascontiguousarray(prompt_offsets, dtype=np.int64)
    _check(lib().tasc_session_prefill(model.handle, s.handle, _ptr(prompts), _ptr(prompt_offsets), _where(prompts), max_new,
                                      _stream(stream)))


def spec_params(k, lambda_q16=49152, p_min_ctx=1, ctx_includes_generated=1) -> SpecParams:
    return SpecParams(k, lambda_q16, p_min_ctx, ctx_includes_generated)


def tasc_draft(ng: Ngram, s: Session, params: SpecParams, drafts, stream=None):
    """drafts: cuda int32 tensor [batch, k], written in place."""
    _check(lib().tasc_draft(ng.handle, s.handle, C.byref(params), _ptr(drafts), _stream(stream)))


def tasc_verify_step(model: Model, s: Session, drafts, k, accept_len=None, emitted=None, logits_dbg=None, stream=None):
    _check(lib().tasc_verify_step(model.handle, s.handle, _ptr(drafts), k, _ptr(accept_len), _ptr(emitted), _ptr(logits_dbg),
                                  _stream(stream)))


def tasc_generate(model: Model, ng, s: Session, prompts, prompt_offsets, max_new, params: SpecParams, out_tokens,
                  trace=None, trace_steps=0, stream=None) -> GenStats:
    prompt_offsets = np.ascontiguousarray(prompt_offsets, dtype=np.int64)
    st = GenStats()
    _check(lib().tasc_generate(model.handle, ng.handle if ng is not None else None, s.handle, _ptr(prompts), _ptr(prompt_offsets),
                               _where(prompts), max_new, C.byref(params), _ptr(out_tokens), _ptr(trace), trace_steps, C.byref(st),
                               _stream(stream)))
    return st


def tasc_session_status(s: Session, stream=None) -> bool:
    """True if a persistent-kernel step of this session ran into a wait time-out since its last prefill."""
    flag = C.c_int32(0)
    _check(lib().tasc_session_status(s.handle, C.byref(flag), _stream(stream)))
    return bool(flag.value)


def tasc_session_get_tokens(s: Session, b: int, stream=None) -> np.ndarray:
    n = C.c_int32(0)
    buf = np.zeros(s.max_len, dtype=np.int32)
    _check(lib().tasc_session_get_tokens(s.handle, b, _ptr(buf), s.max_len, C.byref(n), _stream(stream)))
    return buf[:n.value].copy()


def tasc_profile_enable(classes):
    """classes: iterable of names from KERNEL_CLASSES (empty = off)."""
    mask = 0
    for c in classes:
        mask |= 1 << KERNEL_CLASSES.index(c)
    _check(lib().tasc_profile_enable(mask))


def tasc_profile_read():
    """Returns {class name: (total_ms, launches)} for the classes that recorded something, and clears."""
    n = len(KERNEL_CLASSES)
    ms = np.zeros(n, dtype=np.float64)
    cnt = np.zeros(n, dtype=np.int64)
    _check(lib().tasc_profile_read(_ptr(ms), _ptr(cnt)))
    return {KERNEL_CLASSES[i]: (float(ms[i]), int(cnt[i])) for i in range(n) if cnt[i]}


def tasc_profile_durations(cls_name) -> np.ndarray:
    """Durations (ms) of every recorded launch of one class, in launch order; call before tasc_profile_read."""
    cls = KERNEL_CLASSES.index(cls_name)
    n = C.c_int64(0)
    _check(lib().tasc_profile_durations(cls, None, 0, C.byref(n)))
    out = np.zeros(max(n.value, 1), dtype=np.float64)
    _check(lib().tasc_profile_durations(cls, _ptr(out), out.shape[0], C.byref(n)))
    return out[:n.value]


TASC_CFG_SMALL_PATH, TASC_CFG_SMALL_GRID, TASC_CFG_SMALL_LAYER_WGS, TASC_CFG_SMALL_LAYER_STRIDE, TASC_CFG_TILED_PATH = 0, 1, 2, 3, 4
TASC_CFG_SMALL_XCD_LOCAL = 5
TASC_CFG_SMALL_LAYER_WORKERS = 6
TASC_CFG_SMALL_KERNEL = 7
TASC_CFG_PIPE_SHARE = 8
TASC_CFG_CHAINS = 9
TASC_CFG_STEP_GRAPH = 10


def tasc_config_set(key: int, value: int):
    _check(lib().tasc_config_set(key, value))


def tasc_profile_phases(buf):
    """buf: cuda int64/uint64 tensor (or None to turn the per-phase timestamps off)."""
    _check(lib().tasc_profile_phases(_ptr(buf), 0 if buf is None else buf.numel()))


def tasc_calibration_mfma(iters=2000, stream=None) -> float:
    out = C.c_double(0.0)
    _check(lib().tasc_calibration_mfma(iters, _stream(stream), C.byref(out)))
    return out.value


def tasc_calibration_read(src, passes=1, stream=None) -> float:
    """Read rate (GB/s) of a stream of independent 16-byte loads over the device tensor src (a multiple of 64 KB)."""
    out = C.c_double(0.0)
    _check(lib().tasc_calibration_read(_ptr(src), src.numel() * src.element_size(), passes, _stream(stream), C.byref(out)))
    return out.value


def tasc_calibration_gemm(M, N, K, epilogue=0, slices=1, iters=20, stream=None) -> float:
    """Microseconds per launch of the tiled GEMM at this shape (epilogue 0 store, 1 residual, 2 SwiGLU, 4 partial sums)."""
    out = C.c_double(0.0)
    _check(lib().tasc_calibration_gemm(M, N, K, epilogue, slices, iters, _stream(stream), C.byref(out)))
    return out.value


def tasc_calibration_handover(n_workgroups, stride, nbytes, with_flags=False, stream=None) -> float:
    """Microseconds per hand-over of nbytes among n_workgroups resident workgroups (ids stride * j)."""
    out = C.c_double(0.0)
    _check(lib().tasc_calibration_handover(n_workgroups, stride, nbytes, 1 if with_flags else 0, _stream(stream), C.byref(out)))
    return out.value


def tasc_calibration_copy(dst, src, stream=None):
    """dst, src: cuda uint8 tensors of equal size (a multiple of 16 bytes)."""
    _check(lib().tasc_calibration_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)))
