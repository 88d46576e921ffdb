"""ctypes binding of libpd.so: argument marshalling only.

PyTorch is used for device memory (weights, workspace, logits) and for the
current HIP stream; every step of the method runs inside the library.
"""

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpd.so")

PD_OPT_ATTN_SPLITS, PD_OPT_USE_GRAPH, PD_OPT_PROFILE, PD_OPT_SPLIT_ACT, PD_OPT_PREFILL_CHUNK = 1, 2, 3, 4, 5
PD_OPT_FUSE_NORM = 6
PD_OPT_CONTEXT_SPLIT_ACT = 7
PD_OPT_STREAM_LOADS = 8
PD_OPT_CONTEXT_ATTN = 9
PD_INFO_KERNEL_PATH, PD_INFO_KV_PAIR_LAYERS, PD_INFO_KV_SATURATED, PD_INFO_CONTEXT_PAIRS = 1, 2, 3, 4
PD_INFO_STREAM_LOADS = 5

EXPORTS = ["pd_workspace_bytes", "pd_create", "pd_destroy", "pd_prefill_context", "pd_decode_step",
           "pd_generate", "pd_generate_static", "pd_decode_steps", "pd_reset_decode", "pd_set_option", "pd_profile_read",
           "pd_measure_read_bandwidth", "pd_get_info", "pd_last_error", "pd_encdec_workspace_bytes", "pd_encdec_create", "pd_teacher_forced"]


class PdError(RuntimeError):
    pass


class PdConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layer", "d_model", "n_head", "head_dim", "d_ff", "vocab",
                                         "ffn_kind", "norm_kind", "pos_kind")] + \
               [("rope_base", C.c_float), ("norm_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "bos_id", "eos_id", "max_batch", "max_ctx", "max_sub",
                                         "max_sub_tokens", "max_pos", "kv_pair_layers")]


class PdWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p), ("lm_head", C.c_void_p),
                ("final_norm_g", C.c_void_p), ("final_norm_b", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wqkv", "wo", "w1", "w_up", "w2", "norm1_g",
                                                      "norm1_b", "norm2_g", "norm2_b")]


class PdEncDecConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_enc_layer", "n_dec_layer", "d_model", "n_head", "head_dim", "d_ff",
                                         "vocab", "rel_buckets", "rel_max_distance")] + \
               [("norm_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("bos_id", "eos_id", "max_batch", "max_ctx", "max_sub", "max_sub_tokens")]


_ENCDEC_GLOBAL = ("tok_emb", "lm_head", "enc_rel_bias", "dec_rel_bias", "enc_final_norm_g", "dec_final_norm_g")
_ENCDEC_ENC = ("enc_wqkv", "enc_wo", "enc_w1", "enc_w2", "enc_norm1_g", "enc_norm2_g")
_ENCDEC_DEC = ("dec_wqkv", "dec_wo", "dec_w1", "dec_w2", "cross_wq", "cross_wkv", "cross_wo",
               "dec_norm1_g", "dec_norm3_g", "dec_norm2_g")


class PdEncDecWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _ENCDEC_GLOBAL] + \
               [(n, C.POINTER(C.c_void_p)) for n in _ENCDEC_ENC + _ENCDEC_DEC]


_lib = None


def load():
    """Loads libpd.so; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise PdError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    lib.pd_workspace_bytes.restype = C.c_size_t
    lib.pd_workspace_bytes.argtypes = [C.POINTER(PdConfig)]
    lib.pd_create.argtypes = [C.POINTER(PdConfig), C.POINTER(PdWeights), vp, C.c_size_t, vp, C.POINTER(vp)]
    lib.pd_destroy.argtypes = [vp]
    lib.pd_prefill_context.argtypes = [vp, i32p] + [C.c_int] * 6 + [vp]
    lib.pd_decode_step.argtypes = [vp, i32p, i32p, vp, i32p, vp]
    lib.pd_generate.argtypes = [vp, i32p] + [C.c_int] * 6 + [i32p, i32p, i32p, vp]
    lib.pd_generate_static.argtypes = [C.POINTER(PdConfig), C.POINTER(PdWeights), i32p] + [C.c_int] * 6 + \
                                      [i32p, i32p, i32p, vp]
    lib.pd_decode_steps.argtypes = [vp, C.c_int, vp]
    lib.pd_reset_decode.argtypes = [vp, vp]
    lib.pd_set_option.argtypes = [vp, C.c_int, C.c_int]
    lib.pd_profile_read.argtypes = [vp, C.POINTER(C.c_double), i32p]
    lib.pd_measure_read_bandwidth.argtypes = [vp, C.c_size_t, C.c_size_t, C.c_int, vp, C.POINTER(C.c_double)]
    lib.pd_get_info.argtypes = [vp, C.c_int, vp, C.POINTER(C.c_int64)]
    lib.pd_last_error.restype = C.c_char_p
    lib.pd_teacher_forced.argtypes = [vp, i32p, C.c_int, vp, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_double),
                                      i32p, vp]
    lib.pd_encdec_workspace_bytes.restype = C.c_size_t
    lib.pd_encdec_workspace_bytes.argtypes = [C.POINTER(PdEncDecConfig)]
    lib.pd_encdec_create.argtypes = [C.POINTER(PdEncDecConfig), C.POINTER(PdEncDecWeights), vp, C.c_size_t, vp,
                                     C.POINTER(vp)]
    for name in EXPORTS:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise PdError(f"libpd error {rc}: {load().pd_last_error().decode()}")


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _config(shape, max_batch, max_ctx, max_sub, max_sub_tokens, max_pos, kv_pair_layers):
    return PdConfig(
        n_layer=shape.n_layer, d_model=shape.d_model, n_head=shape.n_head, head_dim=shape.head_dim,
        d_ff=shape.d_ff, vocab=shape.vocab, ffn_kind=shape.ffn_kind, norm_kind=shape.norm_kind,
        pos_kind=shape.pos_kind, rope_base=shape.rope_base, norm_eps=shape.norm_eps,
        dtype=shape.dtype, bos_id=shape.bos_id, eos_id=shape.eos_id, max_batch=max_batch,
        max_ctx=max_ctx, max_sub=max_sub, max_sub_tokens=max_sub_tokens, max_pos=max_pos,
        kv_pair_layers=kv_pair_layers)


def _upload_weights(torch, device, shape, weights):
    """Copies the weights to the device; returns (PdWeights, tensors to keep alive, pointer arrays)."""
    keep, arrays = [], []

    def dev(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            t = torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
        keep.append(t)
        return t.data_ptr()

    w = PdWeights()
    for name in ("tok_emb", "pos_emb", "lm_head", "final_norm_g", "final_norm_b"):
        setattr(w, name, dev(weights.get(name)))
    for name in ("wqkv", "wo", "w1", "w_up", "w2", "norm1_g", "norm1_b", "norm2_g", "norm2_b"):
        ptrs = [dev(lw.get(name)) for lw in weights["layers"]]
        if all(p is None for p in ptrs):
            setattr(w, name, None)
            continue
        arr = (C.c_void_p * shape.n_layer)(*ptrs)
        arrays.append(arr)
        setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
    return w, keep, arrays


class PipelinedDecoder:
    """Owns the device copies of the weights and the workspace of one pd_ctx.

    shape: object with the model fields of pd_config (n_layer, d_model, ...),
    weights: dict of numpy arrays as produced by pd_inputs.make_weights
    (uint16 = bf16 bit patterns, float32 otherwise).
    kv_pair_layers: number of leading layers whose cache keeps keys and values as pairs of halves
    (-1: the library chooses from the shape).
    """

    def __init__(self, shape, weights, max_batch, max_ctx, max_sub, max_sub_tokens, max_pos,
                 device="cuda:0", kv_pair_layers=-1):
        import torch
        self.torch = torch
        self.lib = load()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = _config(shape, max_batch, max_ctx, max_sub, max_sub_tokens, max_pos, kv_pair_layers)
        self.vocab = shape.vocab
        # device tensors and pointer arrays referenced by the library
        w, self._keep, self._arrays = _upload_weights(torch, self.device, shape, weights)
        nbytes = self.lib.pd_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise PdError(f"invalid configuration: {self.lib.pd_last_error().decode()}")
        self.workspace_bytes = nbytes
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.ctx = C.c_void_p()
        _check(self.lib.pd_create(C.byref(self.cfg), C.byref(w), base, nbytes, self._stream(),
                                  C.byref(self.ctx)))
        self.B = self.S = self.M = 0

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "ctx", None) is not None and self.ctx.value:
            self.torch.cuda.synchronize(self.device)
            self.lib.pd_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the three calls of the boundary ---------------------------------------
    def prefill_context(self, ctx_tokens, n_sub, delta_t, sub_tokens, time_max):
        a, p = _i32(ctx_tokens)
        assert a.ndim == 2
        _check(self.lib.pd_prefill_context(self.ctx, p, a.shape[0], a.shape[1], n_sub, delta_t,
                                           sub_tokens, time_max, self._stream()))
        self.B, self.S, self.M = a.shape[0], n_sub, sub_tokens

    def decode_step(self, force=None, want_tokens=True, want_logits=False, want_done=True):
        """Returns (tokens int32 [B][S] or None, logits torch fp32 [B][S][V] or None, all_done or None)."""
        fp = None
        if force is not None:
            fa, fp = _i32(force)
            assert fa.shape == (self.B, self.S)
        toks, tp = (None, None)
        if want_tokens:
            toks = np.full((self.B, self.S), -2, dtype=np.int32)
            tp = toks.ctypes.data_as(C.POINTER(C.c_int32))
        logits, lp = None, None
        if want_logits:
            logits = self.torch.full((self.B, self.S, self.vocab), float("nan"), dtype=self.torch.float32,
                                     device=self.device)
            lp = C.c_void_p(logits.data_ptr())
        done = C.c_int32(0)
        _check(self.lib.pd_decode_step(self.ctx, fp, tp, lp, C.byref(done) if want_done else None,
                                       self._stream()))
        return toks, logits, (bool(done.value) if want_done else None)

    def generate(self, ctx_tokens, n_sub, delta_t, sub_tokens, time_max):
        """Returns (tokens int32 [B][S][M] padded -1, lens int32 [B][S], steps int32 [B])."""
        a, p = _i32(ctx_tokens)
        B = a.shape[0]
        toks = np.full((B, n_sub, sub_tokens), -2, dtype=np.int32)
        lens = np.zeros((B, n_sub), dtype=np.int32)
        steps = np.zeros((B,), dtype=np.int32)
        i32p = C.POINTER(C.c_int32)
        _check(self.lib.pd_generate(self.ctx, p, B, a.shape[1], n_sub, delta_t, sub_tokens, time_max,
                                    toks.ctypes.data_as(i32p), lens.ctypes.data_as(i32p),
                                    steps.ctypes.data_as(i32p), self._stream()))
        self.B, self.S, self.M = B, n_sub, sub_tokens
        return toks, lens, steps

    def teacher_forced(self, targets):
        """pd_teacher_forced.  targets: per request a list of subsequences (lists of token ids as fed:
        <bos>, Y_i, <eos>).  Returns (logits: per request a torch fp32 [rows][V] in subsequence-major
        order, nll: per request float32 [rows], loss float64 [B])."""
        assert len(targets) == self.B
        max_len = max(len(s) for t in targets for s in t)
        rows_cap = max(sum(len(s) for s in t) for t in targets)
        arr = np.full((self.B, self.S, max_len), -1, dtype=np.int32)
        for b, t in enumerate(targets):
            assert len(t) <= self.S
            for i, s in enumerate(t):
                arr[b, i, :len(s)] = s
        logits = self.torch.full((self.B, rows_cap, self.vocab), float("nan"), dtype=self.torch.float32,
                                 device=self.device)
        nll = np.zeros((self.B, rows_cap), dtype=np.float32)
        loss = np.zeros((self.B,), dtype=np.float64)
        rows = np.zeros((self.B,), dtype=np.int32)
        i32p = C.POINTER(C.c_int32)
        _check(self.lib.pd_teacher_forced(self.ctx, arr.ctypes.data_as(i32p), max_len, C.c_void_p(logits.data_ptr()),
                                          rows_cap, nll.ctypes.data_as(C.POINTER(C.c_float)),
                                          loss.ctypes.data_as(C.POINTER(C.c_double)), rows.ctypes.data_as(i32p),
                                          self._stream()))
        return [logits[b, :rows[b]] for b in range(self.B)], [nll[b, :rows[b]] for b in range(self.B)], loss

    # -- helpers ---------------------------------------------------------------
    def decode_steps(self, n):
        _check(self.lib.pd_decode_steps(self.ctx, n, self._stream()))

    def reset_decode(self):
        _check(self.lib.pd_reset_decode(self.ctx, self._stream()))

    def set_option(self, key, value):
        _check(self.lib.pd_set_option(self.ctx, key, value))

    def get_info(self, key):
        v = C.c_int64(0)
        _check(self.lib.pd_get_info(self.ctx, key, self._stream(), C.byref(v)))
        return v.value

    def profile_read(self):
        us, n = C.c_double(0), C.c_int32(0)
        _check(self.lib.pd_profile_read(self.ctx, C.byref(us), C.byref(n)))
        return us.value, n.value


class EncDecPipelinedDecoder(PipelinedDecoder):
    """The encoder-decoder form behind the same calls: prefill_context encodes the inputs (Eq. 1),
    decode_step / generate run Algorithm 1 over the decoder.

    shape: object with the fields of pd_encdec_config's model part (pd_inputs.EncDecConfig);
    weights: the `device` dict of pd_inputs.encdec_to_bf16 (uint16 = bf16 bit patterns)."""

    def __init__(self, shape, weights, max_batch, max_ctx, max_sub, max_sub_tokens, device="cuda:0"):
        import torch
        self.torch = torch
        self.lib = load()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = PdEncDecConfig(
            n_enc_layer=shape.n_enc_layer, n_dec_layer=shape.n_dec_layer, d_model=shape.d_model,
            n_head=shape.n_head, head_dim=shape.head_dim, d_ff=shape.d_ff, vocab=shape.vocab,
            rel_buckets=shape.rel_buckets, rel_max_distance=shape.rel_max_distance, norm_eps=shape.norm_eps,
            bos_id=shape.bos_id, eos_id=shape.eos_id, max_batch=max_batch, max_ctx=max_ctx, max_sub=max_sub,
            max_sub_tokens=max_sub_tokens)
        self.vocab = shape.vocab
        self._keep, self._arrays = [], []

        def dev(a):
            if a.dtype == np.uint16:
                t = torch.from_numpy(a.view(np.int16)).to(self.device).view(torch.bfloat16)
            else:
                t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device)
            self._keep.append(t)
            return t.data_ptr()

        def per_layer(layers, key):
            arr = (C.c_void_p * len(layers))(*[dev(lw[key]) for lw in layers])
            self._arrays.append(arr)
            return C.cast(arr, C.POINTER(C.c_void_p))

        w = PdEncDecWeights()
        for name, key in zip(_ENCDEC_GLOBAL, ("tok_emb", "lm_head", "enc_rel_bias", "dec_rel_bias", "enc_final_g",
                                              "dec_final_g")):
            setattr(w, name, dev(weights[key]))
        for name, key in zip(_ENCDEC_ENC, ("wqkv", "wo", "w1", "w2", "norm1_g", "norm2_g")):
            setattr(w, name, per_layer(weights["enc_layers"], key))
        for name, key in zip(_ENCDEC_DEC, ("wqkv", "wo", "w1", "w2", "cq", "ckv", "co", "norm1_g", "norm3_g",
                                           "norm2_g")):
            setattr(w, name, per_layer(weights["dec_layers"], key))
        nbytes = self.lib.pd_encdec_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise PdError(f"invalid configuration: {self.lib.pd_last_error().decode()}")
        self.workspace_bytes = nbytes
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.ctx = C.c_void_p()
        _check(self.lib.pd_encdec_create(C.byref(self.cfg), C.byref(w), base, nbytes, self._stream(),
                                         C.byref(self.ctx)))
        self.B = self.S = self.M = 0


def generate_static(shape, weights, ctx_tokens, n_sub, delta_t, sub_tokens, time_max, max_pos,
                    device="cuda:0", kv_pair_layers=-1):
    """pd_generate_static: the whole of Algorithm 1 in the library's own static workspace (no device
    allocation inside the library; the weights are uploaded here, by the caller's side).
    Returns (tokens int32 [B][S][M] padded -1, lens int32 [B][S], steps int32 [B])."""
    import torch
    lib = load()
    device = torch.device(device)
    torch.cuda.set_device(device)
    a, p = _i32(ctx_tokens)
    B, L = a.shape
    cfg = _config(shape, B, L, n_sub, sub_tokens, max_pos, kv_pair_layers)
    w, keep, arrays = _upload_weights(torch, device, shape, weights)
    toks = np.full((B, n_sub, sub_tokens), -2, dtype=np.int32)
    lens = np.zeros((B, n_sub), dtype=np.int32)
    steps = np.zeros((B,), dtype=np.int32)
    i32p = C.POINTER(C.c_int32)
    stream = C.c_void_p(torch.cuda.current_stream(device).cuda_stream)
    _check(lib.pd_generate_static(C.byref(cfg), C.byref(w), p, B, L, n_sub, delta_t, sub_tokens, time_max,
                                  toks.ctypes.data_as(i32p), lens.ctypes.data_as(i32p),
                                  steps.ctypes.data_as(i32p), stream))
    del keep, arrays
    return toks, lens, steps


def measure_read_bandwidth(dev_ptr, buf_bytes, chunk_bytes, iters, stream=None):
    """GB/s of a kernel that only reads `chunk_bytes` per launch from the device buffer at `dev_ptr`."""
    out = C.c_double(0)
    _check(load().pd_measure_read_bandwidth(C.c_void_p(dev_ptr), buf_bytes, chunk_bytes, iters,
                                            C.c_void_p(stream or 0), C.byref(out)))
    return out.value
