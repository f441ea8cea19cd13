"""ctypes binding of libdllm.so: same names as include/dllm.h, argument marshalling only.

`Engine` is a convenience that owns the torch tensors (weights, KV pool, workspace) a context
borrows.  Every step of the path runs inside the library's kernels; nothing here computes.
The library must be built (python -m paper_2601_07568_amd.build); loading fails loudly if not.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdllm.so")

DLLM_OK, DLLM_EINVAL, DLLM_ESHAPE, DLLM_ENOSPACE, DLLM_EHIP = 0, -1, -2, -3, -4
DLLM_F32, DLLM_BF16 = 0, 1
STATUS_BAD_TOKEN, STATUS_BAD_PAGE, STATUS_ROWS_CAP, STATUS_BAD_LENGTH = 1, 2, 4, 8


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                          "d_ff", "vocab", "mask_id")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "page_tokens", "max_pages_per_seq", "n_pages",
                                          "max_batch", "max_q", "max_tokens")]


class LayerW(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate",
                                          "w_up", "w_down")]


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(LayerW))]


_lib = None


def lib() -> C.CDLL:
    """Loads libdllm.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_07568_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    pcfg = C.POINTER(Config)
    sig = {
        "dllm_workspace_bytes": (sz, [pcfg]),
        "dllm_kv_pool_bytes": (sz, [pcfg]),
        "dllm_create": (i32, [C.POINTER(vp), pcfg, C.POINTER(Weights), vp, sz, vp, sz]),
        "dllm_destroy": (None, [vp]),
        "dllm_packed_weight_bytes": (sz, [pcfg]),
        "dllm_pack_weights": (i32, [vp, vp, vp, sz]),
        "dllm_prefill_kv": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp]),
        "dllm_denoise_step": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]),
        "dllm_denoise_step_static": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]),
        "dllm_static_scratch_bytes": (sz, []),
        "dllm_unmask": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, f32, i32, vp, vp]),
        "dllm_unmask_entropy": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, f32, i32, vp, vp]),
        "dllm_denoise_step_var": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "dllm_denoise_step_live": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "dllm_gather_rows": (i32, [vp, vp, i32, i32, vp, vp, vp, vp, i32]),
        "dllm_scatter_rows": (i32, [vp, vp, i32, i32, vp, vp, vp, vp]),
        "dllm_fsm_plan": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, i32, vp, vp, vp]),
        "dllm_fsm_window": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp]),
        "dllm_fsm_round_windows": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]),
        "dllm_fsm_pack": (i32, [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]),
        "dllm_refresh_cache_dev": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "dllm_fsm_unpack": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "dllm_fsm_scatter": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]),
        "dllm_unmask_traced": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, f32, i32, i32, i32, vp, vp, vp]),
        "dllm_noisy_sequence": (i32, [vp, vp, i32, i32, vp, vp, vp, i32, C.c_double, vp]),
        "dllm_eos_scan": (i32, [vp, vp, i32, i32, vp, i32, vp, vp, vp, vp]),
        "dllm_unmask_blocks": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, f32, i32, vp, vp, vp]),
        "dllm_fsm_update": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, C.c_double, C.c_double, i32, i32, vp, vp]),
        "dllm_refresh_cache": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "dllm_debug_logits": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, vp]),
        "dllm_debug_hidden": (i32, [vp, vp, i32, i32, i32, vp, vp, vp, i32, vp]),
        "dllm_reset_status": (i32, [vp, vp]),
        "dllm_read_status": (i32, [vp, vp, C.POINTER(C.c_int32)]),
        "dllm_set_kernel_mode": (i32, [vp, i32]),
        "dllm_profile_enable": (i32, [vp, i32]),
        "dllm_profile_read": (i32, [vp, vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                    C.POINTER(C.c_double)]),
        "dllm_probe_hbm_read": (i32, [vp, vp, vp, sz, vp]),
        "dllm_probe_mfma": (i32, [vp, vp, i32, i32, vp, C.POINTER(C.c_double)]),
        "dllm_strerror": (C.c_char_p, [i32]),
        "dllm_last_hip_error": (C.c_char_p, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


class DllmError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        super().__init__(f"dllm error {code}: {lib().dllm_strerror(code).decode()} {detail}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_config(ms, page_tokens, max_pages_per_seq, n_pages, max_batch, max_q, max_tokens) -> Config:
    return Config(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ff, ms.vocab,
                  ms.mask_id, ms.rms_eps, ms.rope_base, DLLM_BF16 if ms.dtype == "bf16" else DLLM_F32,
                  page_tokens, max_pages_per_seq, n_pages, max_batch, max_q, max_tokens)


class Engine:
    """Owns device tensors and a dllm context.  `weights` provides .layer(l) -> dict of numpy arrays
    (float32, or uint16 bfloat16 bits) and ["tok_emb"|"final_norm"|"lm_head"]; alternatively pass
    device tensors through `device_weights` = (globals dict, list of layer dicts)."""

    def __init__(self, ms, weights=None, *, page_tokens=32, max_pages_per_seq=8, n_pages=16, max_batch=1,
                 max_q=32, max_tokens=0, device="cuda:0", device_weights=None, pack=True):
        import torch
        self.torch, self.ms, self.device = torch, ms, torch.device(device)
        self.cfg = make_config(ms, page_tokens, max_pages_per_seq, n_pages, max_batch, max_q, max_tokens)
        L = lib()
        self.tdtype = torch.bfloat16 if ms.dtype == "bf16" else torch.float32

        def up(a):
            t = torch.from_numpy(np.ascontiguousarray(a))
            if a.dtype == np.uint16:
                t = t.view(torch.bfloat16)
            return t.to(self.device)

        if device_weights is not None:
            self.g, self.layers = device_weights
        else:
            self.g = {k: up(weights[k]) for k in ("tok_emb", "final_norm", "lm_head")}
            self.layers = [{k: up(v) for k, v in weights.layer(l).items()} for l in range(ms.n_layers)]
        self._lw = (LayerW * max(1, ms.n_layers))()
        for l, lw in enumerate(self.layers):
            for name, _ in LayerW._fields_:
                assert lw[name].dtype == self.tdtype and lw[name].is_contiguous()
                setattr(self._lw[l], name, lw[name].data_ptr())
        self._w = Weights(self.g["tok_emb"].data_ptr(), self.g["final_norm"].data_ptr(),
                          self.g["lm_head"].data_ptr(), self._lw)
        ws_bytes = L.dllm_workspace_bytes(C.byref(self.cfg))
        kv_bytes = L.dllm_kv_pool_bytes(C.byref(self.cfg))
        if ws_bytes == 0:
            raise DllmError(DLLM_ESHAPE, "(configuration rejected)")
        self.workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=self.device)
        self._ws_off = (-self.workspace.data_ptr()) % 256
        self.kv_pool = torch.zeros(max(kv_bytes, 1), dtype=torch.uint8, device=self.device)
        self.ctx = C.c_void_p()
        rc = L.dllm_create(C.byref(self.ctx), C.byref(self.cfg), C.byref(self._w), self.kv_pool.data_ptr(),
                           kv_bytes, self.workspace.data_ptr() + self._ws_off, ws_bytes)
        if rc != DLLM_OK:
            raise DllmError(rc)
        self._check(L.dllm_reset_status(self.ctx, self._stream()))
        self.packed = None
        if ms.dtype == "bf16" and pack:
            pb = L.dllm_packed_weight_bytes(C.byref(self.cfg))
            self.packed = torch.empty(pb + 256, dtype=torch.uint8, device=self.device)
            off = (-self.packed.data_ptr()) % 256
            self._check(L.dllm_pack_weights(self.ctx, self._stream(), self.packed.data_ptr() + off, pb))

    # -- helpers
    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _check(self, rc):
        if rc != DLLM_OK:
            raise DllmError(rc, lib().dllm_last_hip_error(self.ctx).decode() if rc == DLLM_EHIP else "")

    def close(self):
        if self.ctx:
            lib().dllm_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def i32(self, a):
        return self.torch.as_tensor(np.asarray(a, dtype=np.int32)).to(self.device)

    def kv_slab(self, layer, which):
        """View of the pool as [n_pages, n_kv_heads, page_tokens, head_dim] of layer, which (0=K, 1=V);
        the V slab is stored [.., head_dim, page_tokens] and is returned transposed back."""
        c = self.cfg
        es = 2 if self.ms.dtype == "bf16" else 4
        n = c.n_pages * c.n_kv_heads * c.page_tokens * c.head_dim
        off = (layer * 2 + which) * n * es
        flat = self.kv_pool[off:off + n * es].view(self.tdtype)
        if which == 1:
            return flat.view(c.n_pages, c.n_kv_heads, c.head_dim, c.page_tokens).transpose(2, 3)
        return flat.view(c.n_pages, c.n_kv_heads, c.page_tokens, c.head_dim)

    # -- the calls of include/dllm.h
    def prefill_kv(self, tokens, cu_seqlens, block_table, n_cache=None, *, total_tokens, max_seqlen):
        B = cu_seqlens.numel() - 1
        self._check(lib().dllm_prefill_kv(self.ctx, self._stream(), B, total_tokens, max_seqlen, _ptr(tokens),
                                          _ptr(cu_seqlens), _ptr(n_cache), _ptr(block_table)))

    def denoise_step(self, q_tokens, prefix_len, block_table, cand, conf, entropy=None, *, max_prefix_len):
        B, Q = q_tokens.shape
        self._check(lib().dllm_denoise_step(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                            _ptr(prefix_len), _ptr(block_table), _ptr(cand), _ptr(conf),
                                            _ptr(entropy)))

    def denoise_step_static(self, q_tokens, prefix_len, block_table, cand, conf, entropy=None, *, max_prefix_len):
        B, Q = q_tokens.shape
        self._check(lib().dllm_denoise_step_static(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                                   _ptr(prefix_len), _ptr(block_table), _ptr(cand), _ptr(conf),
                                                   _ptr(entropy)))

    def unmask(self, q_tokens, cand, conf, threshold, min_unmask, block_len=None, n_unmasked=None,
               n_remaining=None):
        B, Q = q_tokens.shape
        self._check(lib().dllm_unmask(self.ctx, self._stream(), B, Q, block_len or Q, _ptr(q_tokens), _ptr(cand),
                                      _ptr(conf), threshold, min_unmask, _ptr(n_unmasked), _ptr(n_remaining)))

    def unmask_entropy(self, q_tokens, cand, entropy, theta, min_unmask, block_len=None, n_unmasked=None,
                       n_remaining=None):
        B, Q = q_tokens.shape
        self._check(lib().dllm_unmask_entropy(self.ctx, self._stream(), B, Q, block_len or Q, _ptr(q_tokens),
                                              _ptr(cand), _ptr(entropy), theta, min_unmask, _ptr(n_unmasked),
                                              _ptr(n_remaining)))

    def unmask_blocks(self, q_tokens, cand, stat, threshold, floor, by_entropy, block_len, n_unmasked=None,
                      n_remaining=None):
        B, Q = q_tokens.shape
        self._check(lib().dllm_unmask_blocks(self.ctx, self._stream(), B, Q, block_len, _ptr(q_tokens), _ptr(cand),
                                             _ptr(stat), threshold, 1 if by_entropy else 0, _ptr(floor),
                                             _ptr(n_unmasked), _ptr(n_remaining)))

    def unmask_traced(self, q_tokens, cand, stat, threshold, min_unmask, step_index, order, by_entropy=False,
                      block_len=None, n_unmasked=None, n_remaining=None):
        B, Q = q_tokens.shape
        self._check(lib().dllm_unmask_traced(self.ctx, self._stream(), B, Q, block_len or Q, _ptr(q_tokens),
                                             _ptr(cand), _ptr(stat), threshold, 1 if by_entropy else 0, min_unmask,
                                             step_index, _ptr(order), _ptr(n_unmasked), _ptr(n_remaining)))

    def noisy_sequence(self, y, order, window_start, k, t, out):
        B, n = y.shape
        self._check(lib().dllm_noisy_sequence(self.ctx, self._stream(), B, n, _ptr(y), _ptr(order),
                                              _ptr(window_start), k, t, _ptr(out)))

    def eos_scan(self, gen_tokens, eos_id, finished, first_eos=None, active_index=None, n_active=None):
        B, n = gen_tokens.shape
        self._check(lib().dllm_eos_scan(self.ctx, self._stream(), B, n, _ptr(gen_tokens), eos_id, _ptr(finished),
                                        _ptr(first_eos), _ptr(active_index), _ptr(n_active)))

    def denoise_step_var(self, q_tokens, prefix_len, q_valid, block_table, cand, conf, entropy=None, *, max_prefix_len):
        B, Q = q_tokens.shape
        self._check(lib().dllm_denoise_step_var(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                                _ptr(prefix_len), _ptr(q_valid), _ptr(block_table), _ptr(cand),
                                                _ptr(conf), _ptr(entropy)))

    def denoise_step_live(self, q_tokens, prefix_len, q_valid, n_live, block_table, cand, conf, entropy=None, *,
                          max_prefix_len):
        B, Q = q_tokens.shape
        self._check(lib().dllm_denoise_step_live(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                                 _ptr(prefix_len), _ptr(q_valid), _ptr(n_live), _ptr(block_table),
                                                 _ptr(cand), _ptr(conf), _ptr(entropy)))

    def gather_rows(self, index, n_index, src, dst, fill=0):
        B = src.shape[0]
        self._check(lib().dllm_gather_rows(self.ctx, self._stream(), B, src.numel() // B, _ptr(index), _ptr(n_index),
                                           _ptr(src), _ptr(dst), fill))

    def scatter_rows(self, index, n_index, src, dst):
        B = src.shape[0]
        self._check(lib().dllm_scatter_rows(self.ctx, self._stream(), B, src.numel() // B, _ptr(index), _ptr(n_index),
                                            _ptr(src), _ptr(dst)))

    def fsm_plan(self, state, counter, base_len, block_len, refresh_every, rounds_since, nocache, n_commit_next):
        B, NB = state.shape
        self._check(lib().dllm_fsm_plan(self.ctx, self._stream(), B, NB, block_len, _ptr(state), _ptr(counter),
                                        _ptr(base_len), refresh_every, _ptr(rounds_since), _ptr(nocache),
                                        _ptr(n_commit_next)))

    def fsm_window(self, gen_tokens, state, base_len, block_len, W, pad_token, win_tokens, win_floor, prefix_len,
                   q_valid, win_lo):
        B, NB = state.shape
        self._check(lib().dllm_fsm_window(self.ctx, self._stream(), B, NB, block_len, W, _ptr(gen_tokens), _ptr(state),
                                          _ptr(base_len), pad_token, _ptr(win_tokens), _ptr(win_floor),
                                          _ptr(prefix_len), _ptr(q_valid), _ptr(win_lo)))

    def fsm_round_windows(self, gen_tokens, state, base_len, nocache, block_len, W, pad_token, win_tokens, win_floor,
                          prefix_len, q_valid, q_valid_cached, win_lo):
        B, NB = state.shape
        self._check(lib().dllm_fsm_round_windows(self.ctx, self._stream(), B, NB, block_len, W, _ptr(gen_tokens),
                                                 _ptr(state), _ptr(base_len), _ptr(nocache), pad_token,
                                                 _ptr(win_tokens), _ptr(win_floor), _ptr(prefix_len), _ptr(q_valid),
                                                 _ptr(q_valid_cached), _ptr(win_lo)))

    def fsm_pack(self, prompt_tokens, gen_tokens, state, base_len, nocache, n_commit_plan, block_len, W, pad_token,
                 tokens, cu_seqlens, n_commit, *, max_seqlen):
        B, NB = state.shape
        self._check(lib().dllm_fsm_pack(self.ctx, self._stream(), B, NB, block_len, W, prompt_tokens.shape[1],
                                        tokens.numel(), max_seqlen, _ptr(prompt_tokens), _ptr(gen_tokens), _ptr(state),
                                        _ptr(base_len), _ptr(nocache), _ptr(n_commit_plan), pad_token, _ptr(tokens),
                                        _ptr(cu_seqlens), _ptr(n_commit)))

    def refresh_cache_dev(self, tokens, cu_seqlens, block_table, n_commit, cand=None, conf=None, entropy=None,
                          *, max_seqlen):
        B = cu_seqlens.numel() - 1
        self._check(lib().dllm_refresh_cache_dev(self.ctx, self._stream(), B, tokens.numel(), max_seqlen, _ptr(tokens),
                                                 _ptr(cu_seqlens), _ptr(n_commit), _ptr(block_table), _ptr(cand),
                                                 _ptr(conf), _ptr(entropy)))

    def fsm_unpack(self, cu_seqlens, prefix_len, q_valid, nocache, packed_cand, packed_conf, packed_entropy, cand, conf,
                   entropy=None):
        B, Q = cand.shape
        self._check(lib().dllm_fsm_unpack(self.ctx, self._stream(), B, Q, packed_cand.numel(), _ptr(cu_seqlens),
                                          _ptr(prefix_len), _ptr(q_valid), _ptr(nocache), _ptr(packed_cand),
                                          _ptr(packed_conf), _ptr(packed_entropy), _ptr(cand), _ptr(conf),
                                          _ptr(entropy)))

    def fsm_scatter(self, win_tokens, win_lo, q_valid, gen_tokens, n_blocks, block_len, W):
        B = win_lo.numel()
        self._check(lib().dllm_fsm_scatter(self.ctx, self._stream(), B, n_blocks, block_len, W, _ptr(win_tokens),
                                           _ptr(win_lo), _ptr(q_valid), _ptr(gen_tokens)))

    def fsm_update(self, gen_tokens, state, counter, block_len, add_at, full_at, delay, nocache_round,
                   floor_next=None, summary=None):
        B, NB = state.shape
        self._check(lib().dllm_fsm_update(self.ctx, self._stream(), B, NB, block_len, _ptr(gen_tokens), _ptr(state),
                                          _ptr(counter), add_at, full_at, delay,
                                          -1 if nocache_round is None else (1 if nocache_round else 0),
                                          _ptr(floor_next), _ptr(summary)))

    def refresh_cache(self, tokens, cu_seqlens, block_table, n_commit=None, cand=None, conf=None, entropy=None,
                      *, total_tokens, max_seqlen):
        B = cu_seqlens.numel() - 1
        self._check(lib().dllm_refresh_cache(self.ctx, self._stream(), B, total_tokens, max_seqlen, _ptr(tokens),
                                             _ptr(cu_seqlens), _ptr(n_commit), _ptr(block_table), _ptr(cand),
                                             _ptr(conf), _ptr(entropy)))

    def debug_logits(self, q_tokens, prefix_len, block_table, *, max_prefix_len):
        B, Q = q_tokens.shape
        out = self.torch.empty(B, Q, self.ms.vocab, dtype=self.torch.float32, device=self.device)
        self._check(lib().dllm_debug_logits(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                            _ptr(prefix_len), _ptr(block_table), _ptr(out)))
        return out

    def debug_hidden(self, q_tokens, prefix_len, block_table, n_layers_run, *, max_prefix_len):
        B, Q = q_tokens.shape
        out = self.torch.empty(B, Q, self.ms.d_model, dtype=self.torch.float32, device=self.device)
        self._check(lib().dllm_debug_hidden(self.ctx, self._stream(), B, Q, max_prefix_len, _ptr(q_tokens),
                                            _ptr(prefix_len), _ptr(block_table), n_layers_run, _ptr(out)))
        return out

    def read_status(self) -> int:
        v = C.c_int32(-1)
        self._check(lib().dllm_read_status(self.ctx, self._stream(), C.byref(v)))
        return v.value

    def reset_status(self):
        self._check(lib().dllm_reset_status(self.ctx, self._stream()))

    def profile_enable(self, on: bool):
        self._check(lib().dllm_profile_enable(self.ctx, 1 if on else 0))

    def profile_read(self, cls: int):
        """(launches, total milliseconds, total algorithmic bytes) of kernel class cls."""
        n, ms, by = C.c_int32(0), C.c_double(0), C.c_double(0)
        self._check(lib().dllm_profile_read(self.ctx, self._stream(), cls, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value

    def probe_hbm_read(self, buf, sink):
        self._check(lib().dllm_probe_hbm_read(self.ctx, self._stream(), _ptr(buf), buf.numel() * buf.element_size(),
                                              _ptr(sink)))

    def probe_mfma(self, iters, sink, random_bits=False) -> float:
        fl = C.c_double(0)
        self._check(lib().dllm_probe_mfma(self.ctx, self._stream(), iters, int(random_bits), _ptr(sink), C.byref(fl)))
        return fl.value

    def set_kernel_mode(self, mode: int):
        self._check(lib().dllm_set_kernel_mode(self.ctx, mode))
