"""ctypes binding of include/areal.h and include/areal_host.h.

Argument marshalling only: every step of the generation path runs in the HIP
library.  PyTorch appears here solely to own device buffers and the stream.
Importing this module without a built library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libareal.so")

OK, E_INVAL, E_NOMEM, E_STATE, E_HIP = 0, -1, -2, -3, -4
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
KV_BLOCK_TOKENS = 16
(K_EMBED, K_RMSNORM, K_GEMM_QKV, K_ROPE_KVWRITE, K_ATTN_DECODE, K_ATTN_PREFILL, K_GEMM_O,
 K_GEMM_GATEUP, K_GEMM_DOWN, K_GEMM_LMHEAD, K_SAMPLER, K_ATTN_MERGE) = range(12)


class ArealError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"areal error {code}: {msg}")
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rope_theta", C.c_float), ("rms_eps", C.c_float),
        ("max_seqs", C.c_int32), ("max_seq_len", C.c_int32), ("max_batch_tokens", C.c_int32),
        ("convert_weights", C.c_int32),
        ("kv_arena", C.c_void_p), ("kv_arena_bytes", C.c_uint64),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64),
        ("hip_stream", C.c_void_p)]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("embed", C.c_void_p), ("lm_head", C.c_void_p),
                ("final_norm", C.c_void_p)] + [(n, _PP) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn",
                 "bq", "bk", "bv")]


_I32P = C.POINTER(C.c_int32)
_I64P = C.POINTER(C.c_int64)

_SIGNATURES = {
    # include/areal.h
    "areal_workspace_bytes": (C.c_uint64, [C.POINTER(ModelCfg)]),
    "areal_kv_block_bytes": (C.c_uint64, [C.POINTER(ModelCfg)]),
    "areal_create": (C.c_int, [C.POINTER(ModelCfg), C.POINTER(C.c_void_p)]),
    "areal_destroy": (C.c_int, [C.c_void_p]),
    "areal_last_error": (C.c_char_p, [C.c_void_p]),
    "areal_load_weights": (C.c_int, [C.c_void_p, C.POINTER(Weights), C.c_uint64]),
    "areal_prefill": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, _I32P, C.c_void_p]),
    "areal_decode_step": (C.c_int, [C.c_void_p, C.c_int32, _I32P, C.c_void_p, C.c_void_p]),
    "areal_append_tokens": (C.c_int, [C.c_void_p, C.c_int32, _I32P, C.c_void_p]),
    "areal_sample_logprob": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, _I32P, _I32P, C.c_float,
                                       C.c_float, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p]),
    "areal_sample_logprob_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_float, C.c_float, C.c_uint64, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]),
    "areal_update_weights_interrupt": (C.c_int, [C.c_void_p, C.POINTER(Weights), C.c_uint64, _I32P,
                                                 _I32P, C.c_void_p, _I64P]),
    "areal_gate_create": (C.c_void_p, [C.c_int64, C.c_int64]),
    "areal_gate_destroy": (None, [C.c_void_p]),
    "areal_gate_submit": (C.c_int64, [C.c_void_p, C.c_int64]),
    "areal_gate_budget": (C.c_int64, [C.c_void_p]),
    "areal_gate_set_version": (C.c_int, [C.c_void_p, C.c_int64]),
    "areal_gate_submitted": (C.c_int64, [C.c_void_p]),
    "areal_dynamic_batching": (C.c_int32, [C.c_int32, _I32P, C.c_int64, C.c_int32, _I32P]),
    "areal_ppo_objective": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_float, C.c_void_p, C.c_void_p]),
    "areal_recompute_logprob": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_float, C.c_void_p,
                                          C.c_int32, C.c_void_p]),
    "areal_free_seq": (C.c_int, [C.c_void_p, C.c_int32]),
    "areal_seq_len": (C.c_int, [C.c_void_p, C.c_int32, _I32P]),
    "areal_get_tokens": (C.c_int, [C.c_void_p, C.c_int32, _I32P]),
    "areal_get_versions": (C.c_int, [C.c_void_p, C.c_int32, _I64P]),
    "areal_kv_blocks": (C.c_int, [C.c_void_p, _I64P, _I64P]),
    "areal_decode_set_counters": (C.c_int, [C.c_void_p, _I64P, _I64P, _I64P]),
    "areal_adopt_seq": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]),
    "areal_adopt_seq_shared": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "areal_profile_begin": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]),
    "areal_profile_end": (C.c_int, [C.c_void_p, _I64P, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    # include/areal_ops.h
    "areal_op_gemm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "areal_op_gemm_num_configs": (C.c_int, []),
    "areal_op_gemm_choose": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _I32P, _I32P]),
    "areal_op_stream_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    # include/areal_host.h
    "areal_kvalloc_create": (C.c_void_p, [C.c_int64, C.c_int32, C.c_int32]),
    "areal_kvalloc_destroy": (None, [C.c_void_p]),
    "areal_kvalloc_reserve": (C.c_int, [C.c_void_p, C.c_int32, C.c_int64]),
    "areal_kvalloc_release": (None, [C.c_void_p, C.c_int32]),
    "areal_kvalloc_share": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]),
    "areal_kvalloc_free_blocks": (C.c_int64, [C.c_void_p]),
    "areal_kvalloc_table": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, C.c_int32]),
    "areal_kvalloc_shuffle": (None, [C.c_void_p, C.c_uint64]),
    "areal_plan_passes": (C.c_int32, [C.c_int32, _I32P, C.c_int32, _I32P, C.c_int32]),
}

_HOST_NAMES = [n for n in _SIGNATURES if n.startswith(("areal_kvalloc_", "areal_gate_"))] + [
    "areal_plan_passes", "areal_dynamic_batching"]

_lib = None
_host_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ArealError(E_STATE, f"{LIB_PATH} is missing: run `python -m paper_2505_24298_amd.build` "
                                      "(or __graft_entry__.build()) first; there is no CPU fallback")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def host_lib():
    """The host-only entry points (include/areal_host.h).  They live in the main library;
    AREAL_HOST_LIB names another build of the same source to take them from instead (the
    sanitizer build of the CPU tests)."""
    global _host_lib
    if _host_lib is None:
        alt = os.environ.get("AREAL_HOST_LIB")
        if not alt:
            _host_lib = lib()
        else:
            l = C.CDLL(alt)
            for name in _HOST_NAMES:
                fn = getattr(l, name)
                fn.restype, fn.argtypes = _SIGNATURES[name]
            _host_lib = l
    return _host_lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_I32P)


def make_cfg(shape, max_seqs, max_seq_len, max_batch_tokens, convert_weights=True):
    cfg = ModelCfg()
    for k in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab"):
        setattr(cfg, k, int(shape[k]))
    cfg.rope_theta = float(shape["rope_theta"])
    cfg.rms_eps = float(shape["rms_eps"])
    cfg.max_seqs, cfg.max_seq_len, cfg.max_batch_tokens = int(max_seqs), int(max_seq_len), int(max_batch_tokens)
    cfg.convert_weights = int(bool(convert_weights))
    return cfg


class Areal:
    """One library context plus the torch buffers it borrows.  Method names are
    the C entry points without the prefix."""

    def __init__(self, shape, max_seqs, max_seq_len, max_batch_tokens, kv_blocks,
                 convert_weights=True, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.shape = dict(shape)
        self.vocab = int(shape["vocab"])
        self.max_seqs = int(max_seqs)
        self.L = lib()
        cfg = make_cfg(shape, max_seqs, max_seq_len, max_batch_tokens, convert_weights)
        ws_bytes = self.L.areal_workspace_bytes(C.byref(cfg))
        blk_bytes = self.L.areal_kv_block_bytes(C.byref(cfg))
        if ws_bytes == 0 or blk_bytes == 0:
            raise ArealError(E_INVAL, "invalid model configuration")
        torch.cuda.set_device(self.device)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.kv_arena = torch.zeros(int(kv_blocks) * blk_bytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), ws_bytes
        cfg.kv_arena, cfg.kv_arena_bytes = self.kv_arena.data_ptr(), self.kv_arena.numel()
        cfg.hip_stream = self.stream.cuda_stream
        self.cfg = cfg
        self.ctx = C.c_void_p()
        rc = self.L.areal_create(C.byref(cfg), C.byref(self.ctx))
        if rc != OK:
            raise ArealError(rc, self.L.areal_last_error(None).decode())
        self._weights_keepalive = []

    def close(self):
        if getattr(self, "ctx", None):
            self.L.areal_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != OK:
            raise ArealError(rc, self.L.areal_last_error(self.ctx).decode())

    # -- weights -----------------------------------------------------------
    def _weights_struct(self, w):
        """w: dict like synth.make_weights but of torch device tensors (all
        of one dtype: float32, bfloat16 or float16)."""
        torch = self.torch
        dt = w["embed"].dtype
        codes = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16, torch.float16: DTYPE_F16}
        if dt not in codes:
            raise ArealError(E_INVAL, "weights must be float32, bfloat16 or float16 tensors")
        keep = []

        def ptr(t):
            assert t.is_cuda and t.is_contiguous() and t.dtype == dt
            keep.append(t)
            return t.data_ptr()

        s = Weights()
        s.dtype = codes[dt]
        s.embed, s.lm_head, s.final_norm = ptr(w["embed"]), ptr(w["lm_head"]), ptr(w["final_norm"])
        nl = len(w["layers"])
        names = ["wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn"]
        if w["layers"][0].get("bq") is not None:
            names += ["bq", "bk", "bv"]
        for n in names:
            arr = (C.c_void_p * nl)(*[ptr(lw[n]) for lw in w["layers"]])
            keep.append(arr)
            setattr(s, n, C.cast(arr, _PP))
        return s, keep

    def load_weights(self, w, version):
        s, keep = self._weights_struct(w)
        self._check(self.L.areal_load_weights(self.ctx, C.byref(s), int(version)))
        self._weights_keepalive = [keep]

    def update_weights_interrupt(self, w, version, logits_out=None):
        torch = self.torch
        s, keep = self._weights_struct(w)
        n_live = C.c_int32()
        ids = np.zeros(self.max_seqs, dtype=np.int32)
        retok = C.c_int64()
        if logits_out is None:
            logits_out = torch.empty((self.max_seqs, self.vocab), dtype=torch.float32, device=self.device)
        self._check(self.L.areal_update_weights_interrupt(
            self.ctx, C.byref(s), int(version), C.byref(n_live), ids.ctypes.data_as(_I32P),
            logits_out.data_ptr(), C.byref(retok)))
        # the previous set may still be read by queued work: keep both alive
        self._weights_keepalive = self._weights_keepalive[-1:] + [keep]
        n = n_live.value
        return ids[:n].copy(), logits_out[:n], retok.value

    def ppo_objective(self, logp_theta, logp_prox, logp_behav, adv, eps, mask=None, per_token=False):
        """Decoupled PPO objective over device float32 arrays: returns (sum, clipped tokens,
        counted tokens) as a host tuple and, with per_token, the per-token objective tensor."""
        torch = self.torch
        n = logp_theta.numel()
        for t in (logp_theta, logp_prox, logp_behav, adv):
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n
        sums = torch.zeros(3, dtype=torch.float64, device=self.device)
        obj = torch.empty(n, dtype=torch.float32, device=self.device) if per_token else None
        if mask is not None:
            assert mask.is_cuda and mask.dtype == torch.uint8 and mask.numel() == n
        self._check(self.L.areal_ppo_objective(self.ctx, n, logp_theta.data_ptr(), logp_prox.data_ptr(),
                                               logp_behav.data_ptr(), adv.data_ptr(),
                                               None if mask is None else mask.data_ptr(), float(eps),
                                               None if obj is None else obj.data_ptr(), sums.data_ptr()))
        s = sums.cpu().numpy()
        return (float(s[0]), int(s[1]), int(s[2])), obj

    def recompute_logprob(self, seqs, temperature=1.0, scratch_rows=256, scratch=None):
        """Log-prob of every token of every sequence given the tokens before it
        (packed float32 device tensor; first token of each sequence = 0)."""
        torch = self.torch
        cu = np.zeros(len(seqs) + 1, dtype=np.int32)
        cu[1:] = np.cumsum([len(p) for p in seqs])
        toks, toks_p = _i32(np.concatenate([np.asarray(p, dtype=np.int32) for p in seqs])
                            if len(seqs) else np.zeros(0, dtype=np.int32))
        if scratch is None:
            scratch = torch.empty((scratch_rows, self.vocab), dtype=torch.float32, device=self.device)
        assert scratch.is_cuda and scratch.dtype == torch.float32 and scratch.is_contiguous()
        out = torch.empty(int(cu[-1]), dtype=torch.float32, device=self.device)
        self._check(self.L.areal_recompute_logprob(self.ctx, len(seqs), toks_p, cu.ctypes.data_as(_I32P),
                                                   float(temperature), scratch.data_ptr(),
                                                   int(scratch.shape[0]), out.data_ptr()))
        return out

    # -- generate ------------------------------------------------------------
    def prefill(self, seq_ids, prompts, logits_out=None):
        torch = self.torch
        ids, ids_p = _i32(seq_ids)
        cu = np.zeros(len(prompts) + 1, dtype=np.int32)
        cu[1:] = np.cumsum([len(p) for p in prompts])
        toks, toks_p = _i32(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts])
                            if len(prompts) else np.zeros(0, dtype=np.int32))
        if logits_out is None:
            logits_out = torch.empty((len(ids), self.vocab), dtype=torch.float32, device=self.device)
        self._check(self.L.areal_prefill(self.ctx, len(ids), ids_p, toks_p, cu.ctypes.data_as(_I32P),
                                         logits_out.data_ptr()))
        return logits_out

    def decode_step(self, seq_ids, tokens_in, logits_out=None):
        torch = self.torch
        ids, ids_p = _i32(seq_ids)
        assert tokens_in.is_cuda and tokens_in.dtype == torch.int32 and tokens_in.numel() >= len(ids)
        if logits_out is None:
            logits_out = torch.empty((len(ids), self.vocab), dtype=torch.float32, device=self.device)
        self._check(self.L.areal_decode_step(self.ctx, len(ids), ids_p, tokens_in.data_ptr(),
                                             logits_out.data_ptr()))
        return logits_out

    def append_tokens(self, seq_ids, tokens_in):
        torch = self.torch
        ids, ids_p = _i32(seq_ids)
        assert tokens_in.is_cuda and tokens_in.dtype == torch.int32 and tokens_in.numel() >= len(ids)
        self._check(self.L.areal_append_tokens(self.ctx, len(ids), ids_p, tokens_in.data_ptr()))

    def sample_logprob(self, logits, seq_ids, positions, temperature=1.0, top_p=1.0, seed=0,
                       forced_tokens=None, out=None):
        torch = self.torch
        n = logits.shape[0]
        assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
        ids, ids_p = _i32(seq_ids)
        pos, pos_p = _i32(positions)
        if out is None:
            out = (torch.empty(n, dtype=torch.int32, device=self.device),
                   torch.empty(n, dtype=torch.float32, device=self.device),
                   torch.empty(n, dtype=torch.float32, device=self.device))
        toks, lb, lf = out
        fp = None
        if forced_tokens is not None:
            assert forced_tokens.is_cuda and forced_tokens.dtype == torch.int32
            fp = forced_tokens.data_ptr()
        self._check(self.L.areal_sample_logprob(self.ctx, n, logits.data_ptr(), ids_p, pos_p,
                                                float(temperature), float(top_p), int(seed), fp,
                                                toks.data_ptr(), lb.data_ptr(), lf.data_ptr()))
        return toks, lb, lf

    def free_seq(self, seq_id):
        self._check(self.L.areal_free_seq(self.ctx, int(seq_id)))

    def adopt_seq(self, seq_id, length, fill_token=0, src_id=-1, n_shared_blocks=0):
        self._check(self.L.areal_adopt_seq_shared(self.ctx, int(seq_id), int(length), int(fill_token),
                                                  int(src_id), int(n_shared_blocks)))

    def seq_len(self, seq_id):
        v = C.c_int32()
        self._check(self.L.areal_seq_len(self.ctx, int(seq_id), C.byref(v)))
        return v.value

    def get_tokens(self, seq_id):
        out = np.zeros(self.seq_len(seq_id), dtype=np.int32)
        self._check(self.L.areal_get_tokens(self.ctx, int(seq_id), out.ctypes.data_as(_I32P)))
        return out

    def get_versions(self, seq_id):
        out = np.zeros(self.seq_len(seq_id), dtype=np.int64)
        self._check(self.L.areal_get_versions(self.ctx, int(seq_id), out.ctypes.data_as(_I64P)))
        return out

    def profile_begin(self, kernel_class, layer=0, every=1):
        self._check(self.L.areal_profile_begin(self.ctx, int(kernel_class), int(layer), int(every)))

    def profile_end(self):
        n, ms, units = C.c_int64(), C.c_double(), C.c_double()
        self._check(self.L.areal_profile_end(self.ctx, C.byref(n), C.byref(ms), C.byref(units)))
        return n.value, ms.value, units.value

    def kv_blocks(self):
        t, f = C.c_int64(), C.c_int64()
        self._check(self.L.areal_kv_blocks(self.ctx, C.byref(t), C.byref(f)))
        return t.value, f.value

    def decode_set_counters(self):
        r, rt, st = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self.L.areal_decode_set_counters(self.ctx, C.byref(r), C.byref(rt), C.byref(st)))
        return r.value, rt.value, st.value


def sample_logprob_static(logits, seq_ids, positions, temperature=1.0, top_p=1.0, seed=0, forced_tokens=None,
                          out=None):
    """areal_sample_logprob_static on torch device tensors (current stream); allocates only
    the outputs, and not even those when `out` is given."""
    import torch
    n, vocab = logits.shape
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
    for t in (seq_ids, positions, forced_tokens):
        assert t is None or (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous())
    if out is None:
        out = (torch.empty(n, dtype=torch.int32, device=logits.device),
               torch.empty(n, dtype=torch.float32, device=logits.device),
               torch.empty(n, dtype=torch.float32, device=logits.device))
    p = lambda t: None if t is None else t.data_ptr()
    rc = lib().areal_sample_logprob_static(torch.cuda.current_stream().cuda_stream, n, vocab, logits.data_ptr(),
                                           p(seq_ids), p(positions), float(temperature), float(top_p), int(seed),
                                           p(forced_tokens), out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr())
    if rc != OK:
        raise ArealError(rc, lib().areal_last_error(None).decode())
    return out


def op_gemm(A, W0, W1, C_out, mode, cfg=-1, splits=-1):
    """areal_op_gemm on torch tensors (current stream)."""
    import torch
    M, K = A.shape
    N = W0.shape[0]
    rc = lib().areal_op_gemm(torch.cuda.current_stream().cuda_stream, A.data_ptr(), W0.data_ptr(),
                             None if W1 is None else W1.data_ptr(), C_out.data_ptr(), M, N, K, mode, cfg, splits)
    if rc != OK:
        raise ArealError(rc, "areal_op_gemm")


def op_stream_read(buf, offset, nbytes, sink):
    """areal_op_stream_read over bytes [offset, offset + nbytes) of the torch uint8 tensor `buf`
    (current stream); `sink`: a device tensor of at least 16 bytes."""
    import torch
    rc = lib().areal_op_stream_read(torch.cuda.current_stream().cuda_stream, buf.data_ptr() + int(offset),
                                    int(nbytes), sink.data_ptr())
    if rc != OK:
        raise ArealError(rc, lib().areal_last_error(None).decode())


def weights_to_device(w, device="cuda:0", bf16=True, f16=False):
    """numpy weight dict (synth.make_weights) -> dict of torch device tensors.
    With bf16 the values must already be bf16-representable (exact cast); f16
    rounds to half precision (the layout a context without convert_weights takes)."""
    import torch
    dt = torch.float16 if f16 else (torch.bfloat16 if bf16 else torch.float32)

    def cv(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dt).contiguous()

    out = dict(embed=cv(w["embed"]), lm_head=cv(w["lm_head"]), final_norm=cv(w["final_norm"]), layers=[])
    for lw in w["layers"]:
        out["layers"].append({k: cv(v) for k, v in lw.items()})
    return out
