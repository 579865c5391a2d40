"""ctypes binding of libspd (argument marshalling only; every step runs in the HIP kernels).

Function names and arguments mirror include/spd.h.  torch is used for device memory
and the current stream, nothing else.  There is no fallback: if the shared library
has not been built, importing this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2404_08856_amd.build, "
                      "or __graft_entry__.build()); there is no CPU fallback")
_lib = ctypes.CDLL(LIB_PATH)

SPD_OK = 0
SPD_ERR_INVALID_ARG, SPD_ERR_SHAPE, SPD_ERR_CAPACITY, SPD_ERR_HIP = -1, -2, -3, -4
SPD_TARGET_IS_PROBS, SPD_DRAFT_IS_PROBS = 1, 2
SPD_MAX_ROWS, SPD_MAX_M = 64, 8

EXPORTS = ["spd_last_error", "spd_model_bytes", "spd_model_create", "spd_model_destroy", "spd_kv_set_len",
           "spd_kv_get_len", "spd_prefill", "spd_prefill_tokens", "spd_verify_forward", "spd_draft_step",
           "spd_accept_workspace_bytes", "spd_speculative_accept", "spd_trace_enable", "spd_trace_read",
           "spd_model_set_tuning", "spd_kv_lens_to_device", "spd_kv_lens_from_device", "spd_draft_step_strided",
           "spd_block_finish", "spd_device_status", "spd_speculative_accept_static", "spd_kv_export", "spd_probe_read_chain"]
TRACE_KINDS = ["qkv", "o", "gate_up", "down", "lm_head", "attention", "embed"]
PROJECTIONS = ["qkv", "o", "gate_up", "down", "lm_head"]


class SpdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libspd error {code}: {msg}")
        self.code = code


class spd_model_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float),
                ("tied_embeddings", ctypes.c_int32), ("max_seqs", ctypes.c_int32),
                ("max_positions", ctypes.c_int32)]


class spd_tuning(ctypes.Structure):
    _fields_ = [("separate_qkv_attention", ctypes.c_int32), ("attention_slices", ctypes.c_int32),
                ("gemm_waves", ctypes.c_int32 * 5), ("gemm_grid_cap", ctypes.c_int32 * 5),
                ("gemm_general_kernel", ctypes.c_int32 * 5), ("gemm_ring", ctypes.c_int32 * 5), ("batch_kernel", ctypes.c_int32),
                ("wait_spin_limit", ctypes.c_uint32)]


_PP = ctypes.POINTER(ctypes.c_void_p)


class spd_weights(ctypes.Structure):
    _fields_ = [("embed", ctypes.c_void_p), ("lm_head", ctypes.c_void_p), ("final_norm", ctypes.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP),
                ("mlp_norm", _PP), ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP)]


_vp, _i32, _f32, _u32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_uint32, ctypes.c_size_t
_szp = ctypes.POINTER(ctypes.c_size_t)
_lib.spd_last_error.restype = ctypes.c_char_p
_lib.spd_last_error.argtypes = []
_lib.spd_model_bytes.argtypes = [ctypes.POINTER(spd_model_config), _szp, _szp, _szp]
_lib.spd_model_create.argtypes = [ctypes.POINTER(spd_model_config), ctypes.POINTER(spd_weights), _vp, _sz, _vp, _sz,
                                  _vp, _sz, _vp, ctypes.POINTER(_vp)]
_lib.spd_model_destroy.argtypes = [_vp]
_lib.spd_model_set_tuning.argtypes = [_vp, ctypes.POINTER(spd_tuning)]
_lib.spd_kv_set_len.argtypes = [_vp, ctypes.POINTER(_i32), _i32]
_lib.spd_kv_get_len.argtypes = [_vp, ctypes.POINTER(_i32), _i32]
_lib.spd_kv_export.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.spd_prefill.argtypes = [_vp, _i32, _vp, _i32, _vp, _vp]
_lib.spd_prefill_tokens.argtypes = [_vp, _i32, _vp, _i32, _vp, _vp]
_lib.spd_verify_forward.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp]
_lib.spd_draft_step.argtypes = [_vp, _vp, _i32, _i32, _f32, _vp, _vp, _vp, _vp]
_lib.spd_accept_workspace_bytes.argtypes = [_i32, _i32, _i32, _szp]
_lib.spd_speculative_accept.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _f32, _u32, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.spd_speculative_accept_static.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _f32, _u32, _vp, _vp, _vp, _vp]
_lib.spd_probe_read_chain.argtypes = [_vp, _sz, _szp, _i32, _i32, _vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), _vp]
_lib.spd_trace_enable.argtypes = [_vp, _i32]
_lib.spd_trace_read.argtypes = [_vp, _i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i32)]
_lib.spd_kv_lens_to_device.argtypes = [_vp, _vp]
_lib.spd_kv_lens_from_device.argtypes = [_vp, _vp]
_lib.spd_device_status.argtypes = [_vp, _vp]
_lib.spd_draft_step_strided.argtypes = [_vp, _vp, _i32, _i32, _i32, _f32, _vp, _i32, _vp, _sz, _vp, _i32, _vp]
_lib.spd_block_finish.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
for _name in EXPORTS:
    if _name != "spd_last_error":
        getattr(_lib, _name).restype = _i32


def spd_last_error():
    return _lib.spd_last_error().decode()


def _check(rc):
    if rc != SPD_OK:
        raise SpdError(rc, spd_last_error())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return ctypes.c_void_p(t.data_ptr())


def _raw(t, dtype):
    """Data pointer of a device tensor that may be a strided view into a larger buffer."""
    assert t.is_cuda and t.dtype == dtype
    return ctypes.c_void_p(t.data_ptr())


def make_config(shape, max_seqs, max_positions):
    """spd_model_config from a synth.ModelShape-like object."""
    return spd_model_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                            shape.vocab, shape.rms_eps, shape.rope_theta, int(shape.tied_embeddings),
                            max_seqs, max_positions)


def spd_model_bytes(cfg):
    p, k, w = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(_lib.spd_model_bytes(ctypes.byref(cfg), ctypes.byref(p), ctypes.byref(k), ctypes.byref(w)))
    return p.value, k.value, w.value


class Model:
    """Owns the three device buffers (torch allocations) and the spd_model handle."""

    def __init__(self, cfg, weights, device="cuda"):
        """weights: dict as produced by synth.make_weights, tensors on `device`."""
        self.cfg = cfg
        pb, kb, wb = spd_model_bytes(cfg)
        self.packed = torch.empty(pb, dtype=torch.uint8, device=device)
        self.kv = torch.zeros(kb, dtype=torch.uint8, device=device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=device)
        L = cfg.n_layers
        assert len(weights["layers"]) == L

        def arr(key, dtype):
            a = (ctypes.c_void_p * L)()
            for l, lw in enumerate(weights["layers"]):
                a[l] = _ptr(lw[key], dtype).value
            return a

        bf, f32 = torch.bfloat16, torch.float32
        keep = [arr("attn_norm", f32), arr("wq", bf), arr("wk", bf), arr("wv", bf), arr("wo", bf),
                arr("mlp_norm", f32), arr("w_gate", bf), arr("w_up", bf), arr("w_down", bf)]
        w = spd_weights(_ptr(weights["embed"], bf), _ptr(weights.get("lm_head"), bf), _ptr(weights["final_norm"], f32),
                        *[ctypes.cast(a, _PP) for a in keep])
        handle = ctypes.c_void_p()
        _check(_lib.spd_model_create(ctypes.byref(cfg), ctypes.byref(w), _ptr(self.packed), pb, _ptr(self.kv), kb,
                                     _ptr(self.workspace), wb, _stream(), ctypes.byref(handle)))
        self.handle = handle
        torch.cuda.current_stream().synchronize()     # re-tiling done: the caller may drop `weights`

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:      # _lib is gone at interpreter shutdown
            _lib.spd_model_destroy(self.handle)
        self.handle = None

    def __del__(self):
        self.close()

    # --- thin wrappers, same names as the C entry points ---------------------------------
    def spd_model_set_tuning(self, separate_qkv_attention=0, attention_slices=0, gemm_waves=None, gemm_grid_cap=None,
                             gemm_general_kernel=None, gemm_ring=None, batch_kernel=0, wait_spin_limit=0):
        """Kernel-selection knobs for tests and sweeps; the per-projection dicts are keyed by PROJECTIONS."""
        t = spd_tuning()
        t.separate_qkv_attention, t.attention_slices, t.wait_spin_limit = int(separate_qkv_attention), int(attention_slices), int(wait_spin_limit)
        t.batch_kernel = int(batch_kernel)
        for field, given in (("gemm_waves", gemm_waves), ("gemm_grid_cap", gemm_grid_cap), ("gemm_general_kernel", gemm_general_kernel),
                             ("gemm_ring", gemm_ring)):
            for name, value in (given or {}).items():
                getattr(t, field)[PROJECTIONS.index(name)] = int(value)
        _check(_lib.spd_model_set_tuning(self.handle, ctypes.byref(t)))

    def spd_kv_set_len(self, lens):
        a = (ctypes.c_int32 * len(lens))(*[int(x) for x in lens])
        _check(_lib.spd_kv_set_len(self.handle, a, len(lens)))

    def spd_kv_get_len(self, n_seqs):
        a = (ctypes.c_int32 * n_seqs)()
        _check(_lib.spd_kv_get_len(self.handle, a, n_seqs))
        return list(a)

    def spd_kv_export(self, layer, seq, pos0, k_out, v_out):
        n = k_out.shape[0]
        assert k_out.shape == v_out.shape == (n, self.cfg.n_heads, self.cfg.head_dim)
        _check(_lib.spd_kv_export(self.handle, layer, seq, pos0, n, _ptr(k_out, torch.float32), _ptr(v_out, torch.float32), _stream()))

    def spd_prefill(self, seq, embeds, last_logits=None):
        _check(_lib.spd_prefill(self.handle, seq, _ptr(embeds, torch.float32), embeds.shape[0],
                                _ptr(last_logits, torch.float32), _stream()))

    def spd_prefill_tokens(self, seq, tokens, last_logits=None):
        _check(_lib.spd_prefill_tokens(self.handle, seq, _ptr(tokens, torch.int32), tokens.shape[0],
                                       _ptr(last_logits, torch.float32), _stream()))

    def spd_verify_forward(self, tokens, logits_out):
        n_seqs, M = tokens.shape
        assert logits_out.shape == (n_seqs, M, self.cfg.vocab)
        _check(_lib.spd_verify_forward(self.handle, _ptr(tokens, torch.int32), n_seqs, M,
                                       _ptr(logits_out, torch.float32), _stream()))

    def spd_draft_step(self, tokens_in, temperature, u_draft, D_row_out, token_out):
        n_seqs, n_in = tokens_in.shape
        assert D_row_out.shape == (n_seqs, self.cfg.vocab) and token_out.shape == (n_seqs,) and u_draft.shape == (n_seqs,)
        _check(_lib.spd_draft_step(self.handle, _ptr(tokens_in, torch.int32), n_seqs, n_in, float(temperature),
                                   _ptr(u_draft, torch.float32), _ptr(D_row_out, torch.float32),
                                   _ptr(token_out, torch.int32), _stream()))


    def spd_draft_step_strided(self, tokens_in, in_stride, n_seqs, n_in, temperature, u_draft, u_stride,
                               D_row_out, D_stride, token_out, token_stride):
        """tokens_in, u_draft, D_row_out, token_out: device tensors (views into larger buffers are fine:
        only their data pointers are used; the strides are in elements between sequences)."""
        _check(_lib.spd_draft_step_strided(self.handle, _raw(tokens_in, torch.int32), in_stride, n_seqs, n_in,
                                           float(temperature), _raw(u_draft, torch.float32), u_stride,
                                           _raw(D_row_out, torch.float32), D_stride, _raw(token_out, torch.int32),
                                           token_stride, _stream()))

    def spd_device_status(self):
        _check(_lib.spd_device_status(self.handle, _stream()))

    def spd_kv_lens_to_device(self):
        _check(_lib.spd_kv_lens_to_device(self.handle, _stream()))

    def spd_kv_lens_from_device(self):
        _check(_lib.spd_kv_lens_from_device(self.handle, _stream()))

    def spd_trace_enable(self, enable):
        _check(_lib.spd_trace_enable(self.handle, int(bool(enable))))

    def spd_trace_read(self):
        """{kind: (milliseconds summed over launches, launches)} since the last read; waits for the events."""
        n = len(TRACE_KINDS)
        ms = (ctypes.c_double * n)()
        cnt = (ctypes.c_int32 * n)()
        _check(_lib.spd_trace_read(self.handle, n, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(TRACE_KINDS)}


def spd_block_finish(target, draft, target_logits, draft_probs, verify_tokens, u, temperature, n_accepted_out,
                     next_token_out, draft_in_out, out_tokens=None, n_out=None, workspace=None):
    n_seqs, g1, vocab = target_logits.shape
    gamma = g1 - 1
    assert draft_probs.shape == (n_seqs, gamma, vocab) and verify_tokens.shape == (n_seqs, g1) and u.shape == (n_seqs, g1)
    assert draft_in_out.shape == (n_seqs, 2)
    if workspace is None:
        workspace = torch.empty(spd_accept_workspace_bytes(n_seqs, gamma, vocab), dtype=torch.uint8, device=target_logits.device)
    cap = 0 if out_tokens is None else out_tokens.shape[1]
    _check(_lib.spd_block_finish(target.handle, draft.handle, _ptr(target_logits, torch.float32), _ptr(draft_probs, torch.float32),
                                 _ptr(verify_tokens, torch.int32), _ptr(u, torch.float32), n_seqs, gamma, float(temperature),
                                 _ptr(n_accepted_out, torch.int32), _ptr(next_token_out, torch.int32),
                                 _ptr(draft_in_out, torch.int32), _ptr(out_tokens, torch.int32), cap, _ptr(n_out, torch.int32),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    return workspace


def spd_accept_workspace_bytes(n_seqs, gamma, vocab):
    b = ctypes.c_size_t()
    _check(_lib.spd_accept_workspace_bytes(n_seqs, gamma, vocab, ctypes.byref(b)))
    return b.value


def spd_speculative_accept(target, draft, draft_tokens, u, temperature, flags, n_accepted_out, next_token_out,
                           accept_prob_out=None, workspace=None):
    n_seqs, g1, vocab = target.shape
    gamma = g1 - 1
    assert draft.shape == (n_seqs, gamma, vocab) and draft_tokens.shape == (n_seqs, gamma) and u.shape == (n_seqs, g1)
    if workspace is None:
        workspace = torch.empty(spd_accept_workspace_bytes(n_seqs, gamma, vocab), dtype=torch.uint8, device=target.device)
    _check(_lib.spd_speculative_accept(_ptr(target, torch.float32), _ptr(draft, torch.float32),
                                       _ptr(draft_tokens, torch.int32), _ptr(u, torch.float32), n_seqs, gamma, vocab,
                                       float(temperature), int(flags), _ptr(n_accepted_out, torch.int32),
                                       _ptr(next_token_out, torch.int32), _ptr(accept_prob_out, torch.float32),
                                       _ptr(workspace), workspace.numel(), _stream()))


def spd_speculative_accept_static(target, draft, draft_tokens, u, temperature, flags, n_accepted_out, next_token_out,
                                  accept_prob_out=None):
    """spd_speculative_accept without a workspace argument (scratch memory inside the library); allocates nothing."""
    n_seqs, g1, vocab = target.shape
    gamma = g1 - 1
    assert draft.shape == (n_seqs, gamma, vocab) and draft_tokens.shape == (n_seqs, gamma) and u.shape == (n_seqs, g1)
    _check(_lib.spd_speculative_accept_static(_ptr(target, torch.float32), _ptr(draft, torch.float32),
                                              _ptr(draft_tokens, torch.int32), _ptr(u, torch.float32), n_seqs, gamma, vocab,
                                              float(temperature), int(flags), _ptr(n_accepted_out, torch.int32),
                                              _ptr(next_token_out, torch.int32), _ptr(accept_prob_out, torch.float32), _stream()))


def spd_probe_read_chain(buffer, stage_bytes, reps=20):
    """(per-kernel microseconds, microseconds per chain) of plain read kernels of the given sizes over `buffer` (a uint8 device tensor)."""
    n = len(stage_bytes)
    sizes = (ctypes.c_size_t * n)(*[int(b) for b in stage_bytes])
    sink = torch.zeros(1024, dtype=torch.int32, device=buffer.device)
    us = (ctypes.c_double * n)()
    chain = ctypes.c_double()
    _check(_lib.spd_probe_read_chain(_ptr(buffer, torch.uint8), buffer.numel(), sizes, n, int(reps), _ptr(sink), us, ctypes.byref(chain), _stream()))
    return list(us), chain.value
