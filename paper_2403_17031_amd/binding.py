"""ctypes binding of librlhf_rollout.so.  Argument marshalling only: every step of the rollout
and rescoring path runs in the library's HIP kernels.  PyTorch provides device memory and the
stream handle, nothing else.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librlhf_rollout.so")

EXPORTS = (
    "rlhf_create", "rlhf_destroy", "rlhf_workspace_bytes", "rollout_generate", "score_sequences",
    "rlhf_debug_logits_rows", "rlhf_profile_enable", "rlhf_profile_read", "rlhf_last_rollout_phases",
    "rlhf_last_error", "rlhf_ppo_assemble_rewards", "rlhf_ppo_gae", "rlhf_ppo_whiten", "rlhf_ppo_loss", "rlhf_adamw_step",
    "rlhf_head_backward", "rlhf_head_backward_workspace_bytes", "rlhf_mlp_backward", "rlhf_mlp_backward_workspace_bytes", "rlhf_attention_backward", "rlhf_forward_keep", "rlhf_policy_backward", "rlhf_policy_backward_workspace_bytes",
    "rlhf_attention_branch_backward", "rlhf_attention_branch_backward_workspace_bytes",
    "rlhf_attention_backward_noalloc", "rlhf_weight_image_bytes", "rlhf_refresh_weights",
    "rlhf_ppo_update", "rlhf_ppo_update_workspace_bytes", "score_responses", "rlhf_score_responses_workspace_bytes",
)

_PER_LAYER = ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv", "w_o", "b_o", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class RlhfError(RuntimeError):
    pass


# Debug aid (tests): when True, every Policy fills its workspace and every output it allocates with 0xFF bytes
# (NaN as fp32 and fp16, -1 as an integer) before each call, so that a kernel reading a region that this call has
# not written -- which on a reused workspace sees plausible values from the previous call -- shows up in the results.
POISON = False


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "rotary_dims", "d_ff",
                                         "vocab", "dtype", "eos_id", "pad_id")] + \
               [("ln_eps", C.c_float), ("rope_base", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [("embed_in", C.c_void_p)] + [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER] + \
               [("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p), ("embed_out", C.c_void_p), ("value_w", C.c_void_p),
                ("value_b", C.c_float)]


class _Grads(C.Structure):  # rlhf_grads: the mirror of rlhf_weights, float arrays
    _fields_ = [("embed_in", C.c_void_p)] + [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER] + \
               [("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p), ("embed_out", C.c_void_p), ("value_w", C.c_void_p),
                ("value_b", C.c_void_p)]


class _UpdateConfig(C.Structure):  # rlhf_ppo_update_config
    _fields_ = [("epochs", C.c_int32), ("n_minibatches", C.c_int32), ("cliprange", C.c_float),
                ("cliprange_value", C.c_float), ("vf_coef", C.c_float), ("temperature", C.c_float),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("first_step", C.c_int32), ("grad_scale", C.c_float)]


class _TrainState(C.Structure):  # rlhf_train_state
    _fields_ = [("grads", _Grads), ("master", _Grads), ("exp_avg", _Grads), ("exp_avg_sq", _Grads)]


_lib = None


def load_library():
    """Loads the built library; raises if it has not been built (python -m paper_2403_17031_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RlhfError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_17031_amd.build`")
    # PyTorch ships its own HIP runtime under the same soname; it must be the one already loaded
    # when this library is opened, or the process ends up with two runtimes and no visible device
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64, f32, sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_float, C.c_size_t
    lib.rlhf_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, sz, C.POINTER(vp)]
    lib.rlhf_weight_image_bytes.argtypes = [C.POINTER(_Config), C.POINTER(sz)]
    lib.rlhf_refresh_weights.argtypes = [vp, vp]
    lib.rlhf_destroy.argtypes = [vp]
    lib.rlhf_destroy.restype = None
    lib.rlhf_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz)]
    lib.rollout_generate.argtypes = [vp, vp, vp, i32, i32, u64, u64, f32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.score_sequences.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.score_responses.argtypes = [vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.rlhf_score_responses_workspace_bytes.argtypes = [vp, i32, i32, i32, C.POINTER(sz)]
    lib.rlhf_debug_logits_rows.argtypes = [vp, vp, vp, i32, i32, C.POINTER(i32), i32, vp, vp, sz, vp]
    lib.rlhf_profile_enable.argtypes = [vp, i32]
    lib.rlhf_profile_read.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                      C.POINTER(C.c_int64), C.POINTER(i32)]
    lib.rlhf_last_rollout_phases.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.rlhf_ppo_assemble_rewards.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, vp, vp, vp, vp, vp]
    lib.rlhf_ppo_gae.argtypes = [vp, vp, C.c_int64, vp, i32, i32, f32, f32, vp, vp, vp]
    lib.rlhf_ppo_whiten.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.rlhf_ppo_loss.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp, vp, vp]
    lib.rlhf_head_backward_workspace_bytes.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
    lib.rlhf_head_backward.argtypes = [vp, vp, vp, vp, vp, i32, C.c_float, C.c_float] + [vp] * 6 + [vp, C.c_size_t, vp]
    lib.rlhf_mlp_backward_workspace_bytes.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
    lib.rlhf_mlp_backward.argtypes = [vp, i32, vp, vp, i32] + [vp] * 7 + [vp, C.c_size_t, vp]
    lib.rlhf_attention_branch_backward_workspace_bytes.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
    lib.rlhf_attention_branch_backward.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32] + [vp] * 7 + [vp, C.c_size_t, vp]
    lib.rlhf_forward_keep.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, C.c_size_t, vp]
    lib.rlhf_policy_backward_workspace_bytes.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
    lib.rlhf_policy_backward.argtypes = [vp, vp, C.c_int64, vp, vp, i32, i32, i32, vp, vp, vp, C.c_float, C.c_float,
                                         C.POINTER(_Grads), vp, C.c_size_t, vp]
    lib.rlhf_attention_backward.argtypes = [vp] * 5 + [i32] * 6 + [vp] * 5 + [vp]
    lib.rlhf_ppo_update_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz)]
    lib.rlhf_ppo_update.argtypes = [vp, C.POINTER(_UpdateConfig), C.POINTER(_TrainState), vp, vp, i32, i32, i32,
                                    vp, vp, vp, vp, vp, C.POINTER(i32), i32, vp, vp, sz, vp]
    lib.rlhf_attention_backward_noalloc.argtypes = [vp] * 5 + [i32] * 6 + [vp] * 3 + [vp]
    lib.rlhf_adamw_step.argtypes = [vp, vp, vp, vp, vp, u64, i32] + [C.c_double] * 6 + [vp]
    lib.rlhf_last_error.restype = C.c_char_p
    for n in EXPORTS:
        if n not in ("rlhf_destroy", "rlhf_last_error"):
            getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def exported_symbols():
    lib = load_library()
    return [n for n in EXPORTS if hasattr(lib, n)]


def _check(rc):
    if rc != 0:
        raise RlhfError(f"rlhf error {rc}: {load_library().rlhf_last_error().decode()}")


class Policy:
    """A model resident on the GPU plus a workspace; wraps one rlhf_handle."""

    def __init__(self, cfg, weights: dict, device="cuda:0"):
        """cfg: synth.ModelConfig-like object; weights: name -> float32 numpy array (already rounded to
        bf16 values when cfg.dtype == 'bf16'), plus scalar 'value_b'."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.lib = load_library()
        self.tdtype = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
        self._dev = {}
        for name, arr in weights.items():
            if name == "value_b":
                continue
            t = torch.from_numpy(np.ascontiguousarray(arr))
            # the values are exactly representable in the storage type, so this conversion is lossless
            self._dev[name] = t.to(self.device, dtype=self.tdtype).contiguous()
        c = _Config(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.rotary_dims, cfg.d_ff, cfg.vocab,
                    0 if cfg.dtype == "fp32" else 1, cfg.eos_id, cfg.pad_id, cfg.ln_eps, cfg.rope_base)
        w = _Weights()
        self._arrays = []
        for n in _PER_LAYER:
            arr = (C.c_void_p * max(cfg.n_layers, 1))(*[self._dev[f"layers.{l}.{n}"].data_ptr()
                                                         for l in range(cfg.n_layers)])
            self._arrays.append(arr)
            setattr(w, n, C.cast(arr, C.POINTER(C.c_void_p)))
        for n in ("embed_in", "lnf_g", "lnf_b", "embed_out"):
            setattr(w, n, self._dev[n].data_ptr())
        w.value_w = self._dev["value_w"].data_ptr() if "value_w" in self._dev else None
        w.value_b = float(weights.get("value_b", 0.0))
        self._value_b = float(weights.get("value_b", 0.0))
        self._train = None
        self._has_value = "value_w" in self._dev
        self._h = C.c_void_p()
        nimg = C.c_size_t()
        _check(self.lib.rlhf_weight_image_bytes(C.byref(c), C.byref(nimg)))
        # the fp16 image the matrix products of a bf16 model read: caller-owned, like every other buffer
        self._image = torch.empty(max(nimg.value, 1), dtype=torch.uint8, device=self.device)
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_create(C.byref(c), C.byref(w), self._image.data_ptr(), nimg.value, C.byref(self._h)))
        self._ws = None

    def close(self):
        if getattr(self, "_h", None):
            self.lib.rlhf_destroy(self._h)
            self._h = None
            self._image = None

    def refresh_weights(self):
        """After the weight tensors in self._dev were changed in place (an optimizer step): re-convert the
        matrices into the fp16 image the products read."""
        with self.torch.cuda.device(self.device):
            _check(self.lib.rlhf_refresh_weights(self._h, self._stream()))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ workspace
    def workspace_bytes(self, B, Lq, max_new, L_score):
        out = C.c_size_t()
        _check(self.lib.rlhf_workspace_bytes(self._h, B, Lq, max_new, L_score, C.byref(out)))
        return out.value

    def _workspace(self, nbytes):
        torch = self.torch
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = None
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        if POISON:
            self._ws.fill_(255)
        return self._ws

    def _out(self, shape, dtype):
        """An output buffer for a call (poisoned like the workspace when the debug switch is on)."""
        t = self.torch.empty(shape, dtype=dtype, device=self.device)
        if POISON:
            t.view(self.torch.uint8).fill_(255)
        return t

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    # ------------------------------------------------------------------ calls
    def rollout_generate(self, queries, pad_mask, seed, temperature, max_new_tokens, seq_id_base=0,
                         return_mask=False):
        """queries int32 [B, Lq], pad_mask uint8 [B, Lq] (torch CUDA tensors or numpy arrays).
        Returns CUDA tensors: tokens int32 [B, Lq+N], logprobs float32 [B, N], lengths int32 [B]
        (and with return_mask=True the uint8 [B, Lq+N] mask that score_sequences takes)."""
        torch = self.torch
        q = self._to_dev(queries, torch.int32)
        m = self._to_dev(pad_mask, torch.uint8)
        B, Lq = q.shape
        N = int(max_new_tokens)
        ws = self._workspace(self.workspace_bytes(B, Lq, max(N, 1), 0))
        toks = self._out((B, Lq + max(N, 0)), torch.int32)
        lps = self._out((B, max(N, 0)), torch.float32)
        lens = self._out((B,), torch.int32)
        omask = self._out((B, Lq + max(N, 0)), torch.uint8) if return_mask else None
        with torch.cuda.device(self.device):
            _check(self.lib.rollout_generate(self._h, q.data_ptr(), m.data_ptr(), B, Lq, C.c_uint64(seed),
                                             C.c_uint64(seq_id_base), temperature, N, toks.data_ptr(),
                                             lps.data_ptr(), lens.data_ptr(),
                                             omask.data_ptr() if return_mask else None, ws.data_ptr(), ws.numel(),
                                             self._stream()))
        return (toks, lps, lens, omask) if return_mask else (toks, lps, lens)

    def score_sequences(self, tokens, mask, temperature, want_values=True):
        """tokens int32 [B, L], mask uint8 [B, L].  Returns (logprobs, values) float32 [B, L] CUDA tensors."""
        torch = self.torch
        t = self._to_dev(tokens, torch.int32)
        m = self._to_dev(mask, torch.uint8)
        B, L = t.shape
        ws = self._workspace(self.workspace_bytes(B, 0, 0, L))
        lp = self._out((B, L), torch.float32)
        val = self._out((B, L), torch.float32) if want_values else None
        with torch.cuda.device(self.device):
            _check(self.lib.score_sequences(self._h, t.data_ptr(), m.data_ptr(), B, L, temperature, lp.data_ptr(),
                                            val.data_ptr() if want_values else None, ws.data_ptr(), ws.numel(),
                                            self._stream()))
        return lp, val

    def score_responses(self, tokens, mask, first_col, temperature, want_values=True):
        """score_sequences restricted to the response: logprobs of the columns from first_col on, values from
        column first_col - 1 on, zeros before.  Returns (logprobs, values) float32 [B, L] CUDA tensors."""
        torch = self.torch
        t = self._to_dev(tokens, torch.int32)
        m = self._to_dev(mask, torch.uint8)
        B, L = t.shape
        out = C.c_size_t()
        _check(self.lib.rlhf_score_responses_workspace_bytes(self._h, B, L, int(first_col), C.byref(out)))
        ws = self._workspace(out.value)
        lp = self._out((B, L), torch.float32)
        val = self._out((B, L), torch.float32) if want_values else None
        with torch.cuda.device(self.device):
            _check(self.lib.score_responses(self._h, t.data_ptr(), m.data_ptr(), B, L, int(first_col), temperature,
                                            lp.data_ptr(), val.data_ptr() if want_values else None, ws.data_ptr(),
                                            ws.numel(), self._stream()))
        return lp, val

    def head_backward(self, x_final, targets, d_logprobs, d_values, temperature, grad_scale=1.0):
        """x_final float32 [T, d], targets int32 [T] (-1: no term), d_logprobs / d_values float32 [T].  Returns a
        dict of CUDA float32 tensors: d_x [T, d], d_lnf_g [d], d_lnf_b [d], d_embed_out [V, d], and, if the model
        has a value head, d_value_w [d] and d_value_b [1]; each is grad_scale times the gradient."""
        torch = self.torch
        x = self._to_dev(x_final, torch.float32)
        y = self._to_dev(targets, torch.int32)
        gl = self._to_dev(d_logprobs, torch.float32)
        T, d = x.shape
        if d != self.cfg.d_model or y.numel() != T or gl.numel() != T:
            raise RlhfError("head_backward: x_final must be [T, d_model], targets and d_logprobs [T]")
        has_v = self._has_value
        gv = self._to_dev(d_values, torch.float32) if has_v else None
        if has_v and gv.numel() != T:
            raise RlhfError("head_backward: d_values must be [T]")
        out = C.c_size_t()
        _check(self.lib.rlhf_head_backward_workspace_bytes(self._h, T, C.byref(out)))
        ws = self._workspace(out.value)
        new = lambda *shape: self._out(shape, torch.float32)
        res = dict(d_x=new(T, d), d_lnf_g=new(d), d_lnf_b=new(d), d_embed_out=new(self.cfg.vocab, d))
        if has_v:
            res.update(d_value_w=new(d), d_value_b=new(1))
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_head_backward(
                self._h, x.data_ptr(), y.data_ptr(), gl.data_ptr(), gv.data_ptr() if has_v else None, T, temperature,
                grad_scale, res["d_x"].data_ptr(), res["d_lnf_g"].data_ptr(), res["d_lnf_b"].data_ptr(),
                res["d_embed_out"].data_ptr(), res["d_value_w"].data_ptr() if has_v else None,
                res["d_value_b"].data_ptr() if has_v else None, ws.data_ptr(), ws.numel(), self._stream()))
        return res

    def mlp_backward(self, layer, x_in, d_out):
        """x_in, d_out float32 [T, d].  Returns a dict of CUDA float32 tensors: d_x [T, d] (the MLP branch's term
        only), d_ln2_g, d_ln2_b [d], d_w_fc1 [d_ff, d], d_b_fc1 [d_ff], d_w_fc2 [d, d_ff], d_b_fc2 [d]."""
        torch = self.torch
        x = self._to_dev(x_in, torch.float32)
        g = self._to_dev(d_out, torch.float32)
        T, d = x.shape
        F = self.cfg.d_ff
        if d != self.cfg.d_model or tuple(g.shape) != (T, d):
            raise RlhfError("mlp_backward: x_in and d_out must both be [T, d_model]")
        out = C.c_size_t()
        _check(self.lib.rlhf_mlp_backward_workspace_bytes(self._h, T, C.byref(out)))
        ws = self._workspace(out.value)
        new = lambda *shape: self._out(shape, torch.float32)
        res = dict(d_x=new(T, d), d_ln2_g=new(d), d_ln2_b=new(d), d_w_fc1=new(F, d), d_b_fc1=new(F),
                   d_w_fc2=new(d, F), d_b_fc2=new(d))
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_mlp_backward(self._h, int(layer), x.data_ptr(), g.data_ptr(), T,
                                              *[res[k].data_ptr() for k in ("d_x", "d_ln2_g", "d_ln2_b", "d_w_fc1",
                                                                            "d_b_fc1", "d_w_fc2", "d_b_fc2")],
                                              ws.data_ptr(), ws.numel(), self._stream()))
        return res

    def attention_branch_backward(self, layer, x_in, d_out, cu_seqlens, max_len=None):
        """x_in, d_out float32 [T, d]; cu_seqlens int32 [B+1].  Returns a dict of CUDA float32 tensors: d_x [T, d]
        (the attention branch's term only), d_ln1_g, d_ln1_b [d], d_w_qkv [3d, d], d_b_qkv [3d], d_w_o [d, d],
        d_b_o [d]."""
        torch = self.torch
        x = self._to_dev(x_in, torch.float32)
        g = self._to_dev(d_out, torch.float32)
        cu = self._to_dev(cu_seqlens if isinstance(cu_seqlens, torch.Tensor) else np.asarray(cu_seqlens, dtype=np.int32),
                          torch.int32)
        T, d = x.shape
        if d != self.cfg.d_model or tuple(g.shape) != (T, d) or cu.dim() != 1 or cu.numel() < 2:
            raise RlhfError("attention_branch_backward: x_in and d_out must be [T, d_model], cu_seqlens [B+1]")
        if max_len is None:
            max_len = int((cu[1:] - cu[:-1]).max().item())
        out = C.c_size_t()
        _check(self.lib.rlhf_attention_branch_backward_workspace_bytes(self._h, T, C.byref(out)))
        ws = self._workspace(out.value)
        new = lambda *shape: self._out(shape, torch.float32)
        names = ("d_x", "d_ln1_g", "d_ln1_b", "d_w_qkv", "d_b_qkv", "d_w_o", "d_b_o")
        res = dict(d_x=new(T, d), d_ln1_g=new(d), d_ln1_b=new(d), d_w_qkv=new(3 * d, d), d_b_qkv=new(3 * d),
                   d_w_o=new(d, d), d_b_o=new(d))
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_attention_branch_backward(self._h, int(layer), x.data_ptr(), g.data_ptr(), cu.data_ptr(),
                                                           cu.numel() - 1, T, max(int(max_len), 1),
                                                           *[res[k].data_ptr() for k in names], ws.data_ptr(),
                                                           ws.numel(), self._stream()))
        return res

    def forward_keep(self, tokens, mask):
        """The scoring forward pass, keeping the residual stream at the input of every layer and after the last.
        Returns (x_keep float32 [(n_layers + 1), B*L, d], cu_seqlens int32 [B+1], packed_tokens int32 [B*L])."""
        torch = self.torch
        t = self._to_dev(tokens, torch.int32)
        m = self._to_dev(mask, torch.uint8)
        B, L = t.shape
        ws = self._workspace(self.workspace_bytes(B, 0, 0, L))
        x_keep = self._out((self.cfg.n_layers + 1, B * L, self.cfg.d_model), torch.float32)
        cu = self._out((B + 1,), torch.int32)
        ptok = self._out((B * L,), torch.int32)
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_forward_keep(self._h, t.data_ptr(), m.data_ptr(), B, L, x_keep.data_ptr(), cu.data_ptr(),
                                              ptok.data_ptr(), ws.data_ptr(), ws.numel(), self._stream()))
        return x_keep, cu, ptok

    def policy_backward(self, x_keep, cu_seqlens, packed_tokens, targets, d_logprobs, d_values, temperature,
                        grad_scale=1.0, max_len=None):
        """x_keep, cu_seqlens, packed_tokens from forward_keep; targets int32 [T], d_logprobs / d_values float32 [T]
        over the T = cu_seqlens[-1] packed rows.  Returns {weight name: CUDA float32 gradient (times grad_scale)}."""
        torch = self.torch
        cfg = self.cfg
        cu = self._to_dev(cu_seqlens, torch.int32)
        T = int(cu[-1].item())
        B = cu.numel() - 1
        if max_len is None:
            max_len = int((cu[1:] - cu[:-1]).max().item())
        y = self._to_dev(targets, torch.int32)
        gl = self._to_dev(d_logprobs, torch.float32)
        gv = self._to_dev(d_values, torch.float32) if self._has_value else None
        if y.numel() != T or gl.numel() != T or (gv is not None and gv.numel() != T):
            raise RlhfError("policy_backward: targets, d_logprobs and d_values must have one entry per packed row")
        d, F, V = cfg.d_model, cfg.d_ff, cfg.vocab
        new = lambda *shape: self._out(shape, torch.float32)
        shapes = dict(ln1_g=(d,), ln1_b=(d,), ln2_g=(d,), ln2_b=(d,), w_qkv=(3 * d, d), b_qkv=(3 * d,), w_o=(d, d),
                      b_o=(d,), w_fc1=(F, d), b_fc1=(F,), w_fc2=(d, F), b_fc2=(d,))
        res = dict(embed_in=new(V, d), lnf_g=new(d), lnf_b=new(d), embed_out=new(V, d))
        if self._has_value:
            res.update(value_w=new(d), value_b=new(1))
        for l in range(cfg.n_layers):
            for n in _PER_LAYER:
                res[f"layers.{l}.{n}"] = new(*shapes[n])
        g = _Grads()
        keep = []
        for n in _PER_LAYER:
            arr = (C.c_void_p * max(cfg.n_layers, 1))(*[res[f"layers.{l}.{n}"].data_ptr() for l in range(cfg.n_layers)])
            keep.append(arr)
            setattr(g, n, C.cast(arr, C.POINTER(C.c_void_p)))
        for n in ("embed_in", "lnf_g", "lnf_b", "embed_out"):
            setattr(g, n, res[n].data_ptr())
        g.value_w = res["value_w"].data_ptr() if self._has_value else None
        g.value_b = res["value_b"].data_ptr() if self._has_value else None
        out = C.c_size_t()
        _check(self.lib.rlhf_policy_backward_workspace_bytes(self._h, T, C.byref(out)))
        ws = self._workspace(out.value)
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_policy_backward(self._h, x_keep.data_ptr(), x_keep.stride(0), cu.data_ptr(),
                                                 packed_tokens.data_ptr(), B, T, max(int(max_len), 1), y.data_ptr(),
                                                 gl.data_ptr(), gv.data_ptr() if gv is not None else None, temperature,
                                                 grad_scale, C.byref(g), ws.data_ptr(), ws.numel(), self._stream()))
        return res

    # ------------------------------------------------------------------ training
    def _grads_struct(self, tensors, keep):
        """An rlhf_grads-shaped struct over {weight name: CUDA float32 tensor} (with a [1] tensor 'value_b')."""
        g = _Grads()
        for n in _PER_LAYER:
            arr = (C.c_void_p * max(self.cfg.n_layers, 1))(*[tensors[f"layers.{l}.{n}"].data_ptr()
                                                             for l in range(self.cfg.n_layers)])
            keep.append(arr)
            setattr(g, n, C.cast(arr, C.POINTER(C.c_void_p)))
        for n in ("embed_in", "lnf_g", "lnf_b", "embed_out", "value_w", "value_b"):
            setattr(g, n, tensors[n].data_ptr())
        return g

    def train_state(self):
        """Allocates (once) what rlhf_ppo_update keeps between calls: fp32 master weights initialised from the
        model's weights, zero moments and gradient buffers.  Returns the dict of dicts of CUDA tensors."""
        torch = self.torch
        if getattr(self, "_train", None) is None:
            if not self._has_value:
                raise RlhfError("the update needs a model with a value head")
            names = [n for n in self._dev]
            master = {n: self._dev[n].float().contiguous() for n in names}
            master["value_b"] = torch.full((1,), self._value_b, dtype=torch.float32, device=self.device)
            zeros = lambda: {n: torch.zeros_like(t) for n, t in master.items()}
            self._train = dict(master=master, exp_avg=zeros(), exp_avg_sq=zeros(), grads=zeros(), steps=0)
        return self._train

    def ppo_update(self, tokens, mask, query_len, old_logprobs, advantages, old_values, returns, kept, temperature,
                   epochs=4, n_minibatches=1, cliprange=0.2, cliprange_value=0.2, vf_coef=0.1, lr=3e-6, beta1=0.9,
                   beta2=0.999, eps=1e-5, weight_decay=0.01, grad_scale=None, keep_preactivations=True):
        """One PPO update (K iterations over mini-batches) through rlhf_ppo_update.  tokens int32 / mask uint8
        [B, Lq+N]; old_logprobs, advantages, old_values, returns float32 [B, N]; kept int32 [B].  Updates this
        policy's weights in place (and the optimizer state from train_state()).  Returns the loss statistics, a
        CUDA float tensor [epochs * n_minibatches, 8] in the order of PPO_LOSS_STATS."""
        torch = self.torch
        t = self._to_dev(tokens, torch.int32)
        m = self._to_dev(mask, torch.uint8)
        B, L = t.shape
        Lq = int(query_len)
        N = L - Lq
        arrs = [self._to_dev(a, torch.float32) for a in (old_logprobs, advantages, old_values, returns)]
        if any(tuple(a.shape) != (B, N) for a in arrs):
            raise RlhfError("ppo_update: old_logprobs, advantages, old_values and returns must be [B, L - query_len]")
        k = self._to_dev(kept, torch.int32)
        if B % n_minibatches:
            raise RlhfError("ppo_update: n_minibatches must divide the batch")
        Bm = B // n_minibatches
        counts = m.view(n_minibatches, Bm * L).sum(1, dtype=torch.int32).cpu().numpy().astype(np.int32)
        max_len = int(m.sum(1).max().item())
        n_kept = int(k.clamp(min=0, max=N).view(n_minibatches, Bm).sum(1).max().item())
        if grad_scale is None:
            grad_scale = 1.0 if self.cfg.dtype == "fp32" else 64.0 * max(n_kept, 1)
        st = self.train_state()
        keep = []
        ts = _TrainState(self._grads_struct(st["grads"], keep), self._grads_struct(st["master"], keep),
                         self._grads_struct(st["exp_avg"], keep), self._grads_struct(st["exp_avg_sq"], keep))
        uc = _UpdateConfig(epochs, n_minibatches, cliprange, cliprange_value, vf_coef, temperature, lr, beta1, beta2, eps,
                           weight_decay, st["steps"] + 1, grad_scale)
        need = C.c_size_t()
        _check(self.lib.rlhf_ppo_update_workspace_bytes(self._h, Bm, L, N, int(counts.max()), C.byref(need)))
        # Workspace beyond the minimum lets the loop keep FC1's pre-activations instead of recomputing them (one
        # [T_max, d_ff] fp16 slice per layer): as many layers as leave 16 GB of the device free.
        want = need.value
        if keep_preactivations and self.cfg.dtype != "fp32":
            per_layer = (int(counts.max()) * self.cfg.d_ff * 2 + 255) // 256 * 256
            free_b, _ = torch.cuda.mem_get_info()
            have = self._ws.numel() if self._ws is not None else 0
            room = free_b + have - need.value - (16 << 30)
            want += max(0, min(self.cfg.n_layers, room // per_layer)) * per_layer + 256
        ws = self._workspace(want)
        stats = self._out((epochs * n_minibatches, 8), torch.float32)
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_ppo_update(self._h, C.byref(uc), C.byref(ts), t.data_ptr(), m.data_ptr(), B, Lq, N,
                                            *[a.data_ptr() for a in arrs], k.data_ptr(),
                                            counts.ctypes.data_as(C.POINTER(C.c_int32)), max(max_len, 1),
                                            stats.data_ptr(), ws.data_ptr(), want, self._stream()))
        st["steps"] += epochs * n_minibatches
        return stats

    def debug_logits_rows(self, tokens, mask, rows_bt):
        torch = self.torch
        t = self._to_dev(tokens, torch.int32)
        m = self._to_dev(mask, torch.uint8)
        B, L = t.shape
        rows = np.ascontiguousarray(np.asarray(rows_bt, dtype=np.int32).reshape(-1, 2))
        n = rows.shape[0]
        ws = self._workspace(self.workspace_bytes(B, 0, 0, L))
        out = self._out((n, self.cfg.vocab), torch.float32)
        with torch.cuda.device(self.device):
            _check(self.lib.rlhf_debug_logits_rows(self._h, t.data_ptr(), m.data_ptr(), B, L,
                                                   rows.ctypes.data_as(C.POINTER(C.c_int32)), n, out.data_ptr(),
                                                   ws.data_ptr(), ws.numel(), self._stream()))
        return out

    # ------------------------------------------------------------------ timing aids
    def profile_enable(self, on=True):
        _check(self.lib.rlhf_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        cap = 64
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_int64 * cap)()
        n = C.c_int32()
        _check(self.lib.rlhf_profile_read(self._h, cap, names, ms, cnt, C.byref(n)))
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(min(n.value, cap))}

    def last_rollout_phases(self):
        a, b = C.c_double(), C.c_double()
        _check(self.lib.rlhf_last_rollout_phases(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def _to_dev(self, x, dtype):
        torch = self.torch
        if isinstance(x, np.ndarray):
            x = torch.from_numpy(np.ascontiguousarray(x))
        return x.to(self.device, dtype=dtype).contiguous()


# ---------------------------------------------------------------------- PPO signals (stateless)
def _dev_f32(torch, a, device):
    t = a if isinstance(a, torch.Tensor) else torch.as_tensor(np.ascontiguousarray(a))
    return t.to(device=device, dtype=torch.float32).contiguous()


def _dev_i32(torch, a, device):
    t = a if isinstance(a, torch.Tensor) else torch.as_tensor(np.ascontiguousarray(a))
    return t.to(device=device, dtype=torch.int32).contiguous()


def _cur_stream(torch, device):
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def ppo_assemble_rewards(logprobs, ref_logprobs, rm_values, tokens, query_len, eos_id, pad_id, beta=0.05,
                         missing_eos_score=-1.0, device="cuda:0"):
    """logprobs [B, N] (rollout_generate); ref_logprobs, rm_values [B, Lq+N] (score_sequences with the
    reference policy's / the reward model's weights); tokens int32 [B, Lq+N].
    Returns CUDA tensors (rewards [B, N], scores [B], kl [B], kept int32 [B])."""
    import torch
    lib = load_library()
    dev = torch.device(device)
    lp = _dev_f32(torch, logprobs, dev)
    ref = _dev_f32(torch, ref_logprobs, dev)
    rm = _dev_f32(torch, rm_values, dev)
    tok = _dev_i32(torch, tokens, dev)
    B, N = lp.shape
    Lq = int(query_len)
    if tuple(ref.shape) != (B, Lq + N) or tuple(rm.shape) != (B, Lq + N) or tuple(tok.shape) != (B, Lq + N):
        raise RlhfError("ppo_assemble_rewards: ref_logprobs, rm_values and tokens must be [B, query_len + N]")
    rewards = torch.empty((B, N), dtype=torch.float32, device=dev)
    scores = torch.empty((B,), dtype=torch.float32, device=dev)
    kl = torch.empty((B,), dtype=torch.float32, device=dev)
    kept = torch.empty((B,), dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.rlhf_ppo_assemble_rewards(lp.data_ptr(), ref.data_ptr(), rm.data_ptr(), tok.data_ptr(), B, Lq, N,
                                             int(eos_id), int(pad_id), float(beta), float(missing_eos_score),
                                             rewards.data_ptr(), scores.data_ptr(), kl.data_ptr(), kept.data_ptr(),
                                             _cur_stream(torch, dev)))
    return rewards, scores, kl, kept


def ppo_gae(rewards, values, kept, gamma=1.0, lam=0.95, value_offset=0, device="cuda:0"):
    """rewards [B, N]; values [B, >= value_offset + N], the value of response token t read at column
    value_offset + t; kept int32 [B].  Returns CUDA tensors (advantages, returns), both [B, N]."""
    import torch
    lib = load_library()
    dev = torch.device(device)
    r = _dev_f32(torch, rewards, dev)
    v = _dev_f32(torch, values, dev)
    k = _dev_i32(torch, kept, dev)
    B, N = r.shape
    off = int(value_offset)
    if v.shape[0] != B or off < 0 or v.shape[1] < off + N or k.shape[0] != B:
        raise RlhfError("ppo_gae: values must be [B, >= value_offset + N] and kept [B]")
    adv = torch.empty((B, N), dtype=torch.float32, device=dev)
    ret = torch.empty((B, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.rlhf_ppo_gae(r.data_ptr(), v.data_ptr() + 4 * off, v.shape[1], k.data_ptr(), B, N, float(gamma),
                                float(lam), adv.data_ptr(), ret.data_ptr(), _cur_stream(torch, dev)))
    return adv, ret


def ppo_whiten(x, kept=None, shift_mean=True, device="cuda:0"):
    """x [B, N]; kept int32 [B] or None (dense).  Returns a CUDA tensor [B, N]."""
    import torch
    lib = load_library()
    dev = torch.device(device)
    xv = _dev_f32(torch, x, dev)
    B, N = xv.shape
    k = None if kept is None else _dev_i32(torch, kept, dev)
    if k is not None and k.shape[0] != B:
        raise RlhfError("ppo_whiten: kept must be [B]")
    out = torch.empty((B, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.rlhf_ppo_whiten(xv.data_ptr(), None if k is None else k.data_ptr(), B, N, 1 if shift_mean else 0,
                                   out.data_ptr(), _cur_stream(torch, dev)))
    return out


PPO_LOSS_STATS = ("loss", "pg_loss", "vf_loss", "approx_kl", "pg_clipfrac", "vf_clipfrac", "ratio_mean", "n_tokens")


def ppo_loss(new_logprobs, old_logprobs, advantages, new_values, old_values, returns, kept, cliprange=0.2,
             cliprange_value=0.2, vf_coef=0.1, device="cuda:0"):
    """All arrays [B, N] over the response positions, kept int32 [B].  Returns (stats, d_logprobs,
    d_values): stats a CUDA float tensor [8] in the order of PPO_LOSS_STATS, the gradients CUDA
    tensors [B, N]."""
    import torch
    lib = load_library()
    dev = torch.device(device)
    arrs = [_dev_f32(torch, a, dev) for a in (new_logprobs, old_logprobs, advantages, new_values, old_values, returns)]
    B, N = arrs[0].shape
    if any(a.shape != (B, N) for a in arrs):
        raise RlhfError("ppo_loss: all six arrays must be [B, N]")
    k = _dev_i32(torch, kept, dev)
    if k.shape[0] != B:
        raise RlhfError("ppo_loss: kept must be [B]")
    d_lp = torch.empty((B, N), dtype=torch.float32, device=dev)
    d_v = torch.empty((B, N), dtype=torch.float32, device=dev)
    stats = torch.empty(8, dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.rlhf_ppo_loss(*[a.data_ptr() for a in arrs], k.data_ptr(), B, N, cliprange, cliprange_value, vf_coef,
                                 d_lp.data_ptr(), d_v.data_ptr(), stats.data_ptr(), _cur_stream(torch, dev)))
    return stats, d_lp, d_v



def linear_lr(base_lr, update_index, total_updates):
    """Learning rate of update `update_index` (0-based) of `total_updates` under the linear schedule."""
    if total_updates <= 0:
        raise ValueError("total_updates must be positive")
    k = min(max(int(update_index), 0), int(total_updates))
    return base_lr * (1.0 - k / total_updates)


def attention_backward(q, k, v, d_out, cu_seqlens, n_heads, max_len=None, noalloc=False, out=None):
    """q, k, v, d_out: CUDA tensors [T, n_heads*head_dim], all float32 or all float16, contiguous; cu_seqlens int32
    [B+1] (CUDA or host).  Returns (dq, dk, dv) in the inputs' dtype.  noalloc=True goes through
    rlhf_attention_backward_noalloc (the library's own fixed scratch); out: optional (dq, dk, dv) to write into."""
    import torch
    lib = load_library()
    ts = (q, k, v, d_out)
    if any((not isinstance(t, torch.Tensor)) or not t.is_cuda or not t.is_contiguous() or t.dim() != 2 for t in ts):
        raise RlhfError("attention_backward: q, k, v, d_out must be contiguous 2-D CUDA tensors")
    if any(t.dtype != q.dtype or t.shape != q.shape for t in ts) or q.dtype not in (torch.float32, torch.float16):
        raise RlhfError("attention_backward: q, k, v, d_out must share shape and dtype (float32 or float16)")
    T, d = q.shape
    if d % n_heads:
        raise RlhfError("attention_backward: the width must be a multiple of n_heads")
    dev = q.device
    cu = torch.as_tensor(cu_seqlens, dtype=torch.int32).to(dev).contiguous()
    B = cu.numel() - 1
    if max_len is None:
        max_len = int((cu[1:] - cu[:-1]).max().item())
    dq, dk, dv = out if out is not None else (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q))
    if noalloc:
        with torch.cuda.device(dev):
            _check(lib.rlhf_attention_backward_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_out.data_ptr(),
                                                       cu.data_ptr(), B, T, n_heads, d // n_heads,
                                                       0 if q.dtype == torch.float32 else 1, max(int(max_len), 1),
                                                       dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                                       _cur_stream(torch, dev)))
        return dq, dk, dv
    lse = torch.empty(T * n_heads, dtype=torch.float32, device=dev)
    delta = torch.empty(T * n_heads, dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.rlhf_attention_backward(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_out.data_ptr(), cu.data_ptr(),
                                           B, T, n_heads, d // n_heads, 0 if q.dtype == torch.float32 else 1,
                                           max(int(max_len), 1), lse.data_ptr(), delta.data_ptr(), dq.data_ptr(),
                                           dk.data_ptr(), dv.data_ptr(), _cur_stream(torch, dev)))
    return dq, dk, dv


def adamw_step(param, grad, exp_avg, exp_avg_sq, step, lr=3e-6, beta1=0.9, beta2=0.999, eps=1e-5, weight_decay=0.01,
               grad_scale=1.0, param_bf16=None):
    """In-place AdamW update of CUDA float32 tensors (any shape, contiguous, same number of elements);
    param_bf16: optional CUDA bfloat16 tensor that receives the rounded parameters."""
    import torch
    lib = load_library()
    ts = (param, grad, exp_avg, exp_avg_sq)
    if any((not isinstance(t, torch.Tensor)) or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous()
           for t in ts):
        raise RlhfError("adamw_step: param, grad and the moments must be contiguous CUDA float32 tensors")
    n = param.numel()
    if any(t.numel() != n for t in ts):
        raise RlhfError("adamw_step: all arrays must have the same number of elements")
    if param_bf16 is not None and (param_bf16.dtype != torch.bfloat16 or not param_bf16.is_cuda or
                                   not param_bf16.is_contiguous() or param_bf16.numel() != n):
        raise RlhfError("adamw_step: param_bf16 must be a contiguous CUDA bfloat16 tensor of the same size")
    dev = param.device
    with torch.cuda.device(dev):
        _check(lib.rlhf_adamw_step(param.data_ptr(), grad.data_ptr(), exp_avg.data_ptr(), exp_avg_sq.data_ptr(),
                                   None if param_bf16 is None else param_bf16.data_ptr(), n, int(step), lr, beta1, beta2,
                                   eps, weight_decay, grad_scale, _cur_stream(torch, dev)))
