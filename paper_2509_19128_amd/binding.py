"""ctypes binding of include/pl.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

__all__ = [
    "PL_OK", "PL_E_INVAL", "PL_E_NOSLOT", "PL_E_NOKV", "PL_E_BUSY", "PL_E_STATE", "PL_E_CTX", "PL_E_HIP",
    "PL_E_NOMEM", "PL_SWAP_ASYNC", "PL_SWAP_WAIT", "PL_SWAP_RECOMPUTE_KV", "PL_DEVICE_NONE", "PL_BF16", "PL_F32", "PlError", "ModelCfg", "StepOut", "Stats",
    "lib", "library_path", "Engine", "operand_order", "pl_attention_decode", "pl_attention_workspace_bytes", "pl_kv_pack_host",
    "pl_gemm_bf16", "pl_debug_gemm_cfg", "pl_debug_gemm_plan", "pl_debug_gemm_planned", "pl_sample", "pl_sample_static", "pl_sample_workspace_bytes", "pl_debug_stream_read", "pl_is_ess", "EXPORTS",
]

PL_OK, PL_E_INVAL, PL_E_NOSLOT, PL_E_NOKV, PL_E_BUSY, PL_E_STATE, PL_E_CTX, PL_E_HIP, PL_E_NOMEM = 0, -1, -2, -3, -4, -5, -6, -7, -8
PL_SWAP_ASYNC, PL_SWAP_WAIT, PL_SWAP_RECOMPUTE_KV = 0, 1, 2
PL_DEVICE_NONE = -1
PL_BF16, PL_F32 = 0, 1

# every symbol include/pl.h declares
EXPORTS = [
    "pl_create", "pl_destroy", "pl_last_error", "pl_weight_count", "pl_weight_layout", "pl_weight_nbytes",
    "pl_pack_weights", "pl_load_weights", "pl_swap_weights", "pl_swap_poll", "pl_add_sequence", "pl_prefill", "pl_prefill_async", "pl_retire_sequence",
    "pl_num_active", "pl_decode_step", "pl_get_stats", "pl_debug_get_logits", "pl_debug_read_kv",
    "pl_debug_write_kv", "pl_debug_add_sequence_at", "pl_debug_set_history", "pl_debug_set_poison", "pl_debug_set_graphs", "pl_debug_kv_pool", "pl_debug_set_profile", "pl_debug_gemm_cfg", "pl_debug_gemm_plan", "pl_debug_gemm_planned", "pl_debug_stream_read", "pl_attention_workspace_bytes",
    "pl_attention_decode", "pl_kv_pack_host", "pl_gemm_bf16", "pl_sample_workspace_bytes", "pl_sample", "pl_sample_static", "pl_is_ess",
]


class PlError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"pl error {code}: {msg}")
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("max_batch", C.c_int32),
                ("max_context", C.c_int32), ("kv_pool_tokens", C.c_int64), ("kv_page_tokens", C.c_int32),
                ("n_weight_buffers", C.c_int32), ("seed", C.c_uint64), ("device", C.c_int32), ("dtype", C.c_int32), ("tie_embeddings", C.c_int32)]


class StepOut(C.Structure):
    _fields_ = [("n", C.c_int32), ("slot", C.POINTER(C.c_int32)), ("seq_id", C.POINTER(C.c_uint64)),
                ("token", C.POINTER(C.c_int32)), ("logprob", C.POINTER(C.c_float)),
                ("weight_version", C.POINTER(C.c_uint32)), ("position", C.POINTER(C.c_int32)),
                ("emitted", C.POINTER(C.c_uint8)), ("finished", C.POINTER(C.c_uint8)),
                ("step_ms", C.c_float), ("swap_stall_ms", C.c_float)]


class Stats(C.Structure):
    _fields_ = [("steps", C.c_uint64), ("tokens_emitted", C.c_uint64), ("slot_steps", C.c_uint64),
                ("swaps", C.c_uint64), ("gpu_ms_total", C.c_double), ("algorithmic_bytes", C.c_double),
                ("last_swap_copy_ms", C.c_float), ("active_version", C.c_uint32),
                ("kv_pages_free", C.c_int64), ("kv_pages_total", C.c_int64),
                ("attn_ms", C.c_double), ("gemm_ms", C.c_double), ("sample_ms", C.c_double), ("other_ms", C.c_double),
                ("attn_launches", C.c_uint64), ("gemm_launches", C.c_uint64), ("attn_kv_bytes", C.c_double),
                ("attn_shared_ms", C.c_double), ("attn_shared_kv_bytes", C.c_double), ("attn_shared_launches", C.c_uint64),
                ("host_enqueue_ms", C.c_double), ("host_wait_ms", C.c_double),
                ("prefill_passes", C.c_uint64), ("prefill_positions", C.c_uint64), ("prefill_ms", C.c_double),
                ("recompute_passes", C.c_uint64), ("recompute_positions", C.c_uint64), ("recompute_ms", C.c_double)]


_lib = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpl.so")


def lib():
    """The loaded library.  Builds it on first use if no built library is present; raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    L = C.CDLL(path)
    vp, i32, i64, u32, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float
    P = C.POINTER
    sigs = {
        "pl_create": (C.c_int, [P(ModelCfg), P(vp)]),
        "pl_destroy": (None, [vp]),
        "pl_last_error": (C.c_char_p, []),
        "pl_weight_count": (i32, [vp]),
        "pl_weight_layout": (C.c_int, [vp, i32, P(C.c_char_p), P(i64), P(i64)]),
        "pl_weight_nbytes": (i64, [vp]),
        "pl_pack_weights": (C.c_int, [vp, C.c_char_p, vp, i32, vp]),
        "pl_load_weights": (C.c_int, [vp, vp, i64]),
        "pl_swap_weights": (C.c_int, [vp, vp, i64, u32, P(u32)]),
        "pl_swap_poll": (C.c_int, [vp, P(i32), P(u32)]),
        "pl_add_sequence": (C.c_int, [vp, u64, vp, i32, i32, f32, P(i32)]),
        "pl_prefill": (C.c_int, [vp, i32, P(i32)]),
        "pl_prefill_async": (C.c_int, [vp, i32, P(i32)]),
        "pl_debug_set_history": (C.c_int, [vp, i32, vp, i32]),
        "pl_retire_sequence": (C.c_int, [vp, i32]),
        "pl_num_active": (i32, [vp]),
        "pl_decode_step": (C.c_int, [vp, vp, P(StepOut)]),
        "pl_get_stats": (C.c_int, [vp, P(Stats)]),
        "pl_debug_get_logits": (C.c_int, [vp, vp, i64]),
        "pl_debug_read_kv": (C.c_int, [vp, i32, i32, vp, vp, i32]),
        "pl_debug_write_kv": (C.c_int, [vp, i32, i32, vp, vp, i32]),
        "pl_debug_add_sequence_at": (C.c_int, [vp, u64, vp, i32, i32, f32, i32, i32, i32, P(i32)]),
        "pl_debug_kv_pool": (C.c_int, [vp, P(vp), P(i64)]),
        "pl_debug_set_profile": (C.c_int, [vp, i32]),
        "pl_debug_set_poison": (C.c_int, [vp, i32]),
        "pl_debug_set_graphs": (C.c_int, [vp, i32]),
        "pl_debug_stream_read": (i64, [vp, i64, i32, vp]),
        "pl_debug_gemm_cfg": (C.c_int, [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]),
        "pl_debug_gemm_plan": (C.c_int, [i32, i32, i32, i32, vp, vp, vp, vp]),
        "pl_debug_gemm_planned": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]),
        "pl_attention_workspace_bytes": (i64, [i32, i32, i32, i32, i32]),
        "pl_attention_decode": (C.c_int, [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp]),
        "pl_kv_pack_host": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32]),
        "pl_gemm_bf16": (C.c_int, [vp, vp, vp, i32, i32, i32, i32, i32, vp]),
        "pl_sample_workspace_bytes": (i64, [i32, i32]),
        "pl_sample": (C.c_int, [vp, i32, i32, vp, vp, vp, vp, u64, vp, vp, vp, vp]),
        "pl_sample_static": (C.c_int, [vp, i32, i32, vp, vp, vp, vp, u64, vp, vp, vp]),
        "pl_is_ess": (C.c_int, [vp, vp, vp, i32, f32, vp, vp, vp, vp, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise PlError(rc, lib().pl_last_error().decode())


def operand_order(w):
    """[N, K] matrix -> the flat MFMA-operand-ordered image the GEMM kernels stream (layout only)."""
    n, k = w.shape
    assert n % 32 == 0 and k % 64 == 0, (n, k)
    return np.ascontiguousarray(w.reshape(n // 32, 32, k // 64, 2, 4, 8).transpose(2, 0, 4, 3, 1, 5)).reshape(-1)


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


class Engine:
    """Owns one pl_engine*.  Methods are the ABI calls with numpy marshalling."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, max_batch,
                 max_context, kv_pool_tokens, rope_theta=1.0e4, rms_eps=1.0e-6, kv_page_tokens=0,
                 n_weight_buffers=2, seed=0, device=0, dtype=PL_BF16, tie_embeddings=0):
        self.cfg = ModelCfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_theta,
                            rms_eps, max_batch, max_context, kv_pool_tokens, kv_page_tokens, n_weight_buffers,
                            seed, device, dtype, tie_embeddings)
        self._h = C.c_void_p()
        _check(lib().pl_create(C.byref(self.cfg), C.byref(self._h)))
        B = max_batch
        self._o = dict(slot=np.zeros(B, np.int32), seq_id=np.zeros(B, np.uint64), token=np.zeros(B, np.int32),
                       logprob=np.zeros(B, np.float32), weight_version=np.zeros(B, np.uint32),
                       position=np.zeros(B, np.int32), emitted=np.zeros(B, np.uint8), finished=np.zeros(B, np.uint8))
        self._out = StepOut()
        for k, v in self._o.items():
            setattr(self._out, k, v.ctypes.data_as(dict(StepOut._fields_)[k]))

    @classmethod
    def from_model(cls, m, **kw):
        """m: any object with the decoder shape attributes (e.g. synth.ModelCfg)."""
        return cls(n_layers=m.n_layers, d_model=m.d_model, n_q_heads=m.n_q_heads, n_kv_heads=m.n_kv_heads,
                   head_dim=m.head_dim, d_ffn=m.d_ffn, vocab=m.vocab, rope_theta=m.rope_theta, rms_eps=m.rms_eps, **kw)

    def close(self):
        if self._h:
            lib().pl_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- weights ------------------------------------------------------------------------------
    def weight_nbytes(self):
        return int(lib().pl_weight_nbytes(self._h))

    def weight_layout(self):
        out = []
        for i in range(lib().pl_weight_count(self._h)):
            name, off, shp = C.c_char_p(), C.c_int64(), (C.c_int64 * 2)()
            _check(lib().pl_weight_layout(self._h, i, C.byref(name), C.byref(off), shp))
            out.append((name.value.decode(), off.value, (shp[0], shp[1])))
        return out

    def pack_weights(self, tensors, to_bits):
        """Flat uint16 (bf16 bits) blob from per-tensor fp32 arrays named wq/wk/wv/wo/wg/wu/wd/g1/g2
        per layer plus embed/gf/lm_head; `to_bits` converts fp32 -> bf16 bit patterns.  Row
        concatenation, the 32-row gate/up interleave and the operand ordering are layout only."""
        if self.cfg.dtype == PL_F32:
            return self.pack_weights_c(tensors)          # fp32 test build: row-major fp32, no bf16 conversion
        blob = np.empty(self.weight_nbytes() // 2, np.uint16)
        for name, off, (r, c) in self.weight_layout():
            if name.endswith("w_qkv"):
                p = name[:-5]
                src = np.concatenate([tensors[p + "wq"], tensors[p + "wk"], tensors[p + "wv"]], axis=0)
            elif name.endswith("w_gu"):
                p = name[:-4]
                g, u = tensors[p + "wg"], tensors[p + "wu"]
                f, d = g.shape
                src = np.stack([g.reshape(f // 32, 32, d), u.reshape(f // 32, 32, d)], axis=1).reshape(2 * f, d)
            elif name.endswith("w_o"):
                src = tensors[name[:-3] + "wo"]
            elif name.endswith("w_d"):
                src = tensors[name[:-3] + "wd"]
            else:
                src = tensors[name]
            assert src.size == r * c, (name, src.shape, r, c)
            bits = to_bits(np.ascontiguousarray(src, np.float32)).reshape(src.shape)
            blob[off:off + r * c] = bits.reshape(-1) if (c == 1 or name == "embed") else operand_order(bits)
        return blob

    def pack_weights_c(self, tensors):
        """The blob through the library's host helper pl_pack_weights (fp32 sources): uint16 bf16 bit
        patterns, or float32 for an engine of the fp32 test build."""
        f32 = self.cfg.dtype == PL_F32
        blob = np.zeros(self.weight_nbytes() // (4 if f32 else 2), np.float32 if f32 else np.uint16)
        for name, w in tensors.items():
            if name == "lm_head" and self.cfg.tie_embeddings:
                continue
            w = np.ascontiguousarray(w, np.float32)
            _check(lib().pl_pack_weights(self._h, name.encode(), _np_ptr(w), 1, _np_ptr(blob)))
        return blob

    def unpack_weights(self, blob, from_bits, names=None):
        """Inverse of pack_weights: per-tensor fp32 arrays (wq/wk/wv/wo/wg/wu/wd/g1/g2, embed, gf, lm_head)
        from a flat uint16 blob.  `names`: restrict to these blob tensors (e.g. one layer at a time)."""
        cfg, out = self.cfg, {}
        qd, kvd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        for name, off, (r, c) in self.weight_layout():
            if names is not None and name not in names:
                continue
            bits = np.asarray(blob[off:off + r * c])
            if c == 1:
                out[name] = from_bits(bits).reshape(r)
                continue
            if name != "embed":
                bits = bits.reshape(c // 64, r // 32, 4, 2, 32, 8).transpose(1, 4, 0, 3, 2, 5).reshape(r, c)
            w = from_bits(np.ascontiguousarray(bits)).reshape(r, c)
            if name.endswith("w_qkv"):
                p = name[:-5]
                out[p + "wq"], out[p + "wk"], out[p + "wv"] = w[:qd], w[qd:qd + kvd], w[qd + kvd:]
            elif name.endswith("w_gu"):
                p = name[:-4]
                gu = w.reshape(r // 64, 2, 32, c)
                out[p + "wg"], out[p + "wu"] = gu[:, 0].reshape(r // 2, c), gu[:, 1].reshape(r // 2, c)
            elif name.endswith("w_o"):
                out[name[:-3] + "wo"] = w
            elif name.endswith("w_d"):
                out[name[:-3] + "wd"] = w
            else:
                out[name] = w
        return out

    def load_weights(self, src, nbytes=None):
        """src: numpy array (host) or an integer device/host address with nbytes."""
        if isinstance(src, np.ndarray):
            _check(lib().pl_load_weights(self._h, _np_ptr(src), src.nbytes))
        else:
            _check(lib().pl_load_weights(self._h, C.c_void_p(int(src)), int(nbytes)))

    def swap_weights(self, src, nbytes=None, flags=PL_SWAP_WAIT):
        v = C.c_uint32()
        if isinstance(src, np.ndarray):
            self._keep = src          # must stay alive until the flip
            _check(lib().pl_swap_weights(self._h, _np_ptr(src), src.nbytes, flags, C.byref(v)))
        else:
            _check(lib().pl_swap_weights(self._h, C.c_void_p(int(src)), int(nbytes), flags, C.byref(v)))
        return v.value

    def swap_poll(self):
        r, v = C.c_int32(), C.c_uint32()
        _check(lib().pl_swap_poll(self._h, C.byref(r), C.byref(v)))
        return bool(r.value), v.value

    # ---- sequences ----------------------------------------------------------------------------
    def add_sequence(self, seq_id, prompt, max_new, temperature=1.0):
        p = np.ascontiguousarray(prompt, np.int32)
        s = C.c_int32()
        _check(lib().pl_add_sequence(self._h, seq_id, _np_ptr(p), p.size, max_new, temperature, C.byref(s)))
        return s.value

    def debug_add_sequence_at(self, seq_id, prompt, n_prompt, max_new, temperature, context_len, n_emitted, last_token):
        p = None if prompt is None else np.ascontiguousarray(prompt, np.int32)
        s = C.c_int32()
        _check(lib().pl_debug_add_sequence_at(self._h, seq_id, None if p is None else _np_ptr(p), n_prompt, max_new,
                                              temperature, context_len, n_emitted, last_token, C.byref(s)))
        return s.value

    def prefill(self, slot):
        """Read the slot's prompt except its last token in batched passes; returns the positions read."""
        n = C.c_int32()
        _check(lib().pl_prefill(self._h, slot, C.byref(n)))
        return n.value

    def prefill_async(self, slot):
        """Start reading the slot's prompt in the background; returns the positions that will be read."""
        n = C.c_int32()
        _check(lib().pl_prefill_async(self._h, slot, C.byref(n)))
        return n.value

    def debug_set_history(self, slot, tokens):
        t = np.ascontiguousarray(tokens, np.int32)
        _check(lib().pl_debug_set_history(self._h, slot, _np_ptr(t), t.size))

    def retire_sequence(self, slot):
        _check(lib().pl_retire_sequence(self._h, slot))

    def num_active(self):
        return int(lib().pl_num_active(self._h))

    # ---- step -----------------------------------------------------------------------------------
    def decode_step(self, forced=None):
        """Returns a dict of arrays (views trimmed to n entries; valid until the next step)."""
        f = None if forced is None else np.ascontiguousarray(forced, np.int32)
        _check(lib().pl_decode_step(self._h, None if f is None else _np_ptr(f), C.byref(self._out)))
        n = self._out.n
        r = {k: v[:n] for k, v in self._o.items()}
        r["n"], r["step_ms"], r["swap_stall_ms"] = n, self._out.step_ms, self._out.swap_stall_ms
        return r

    def stats(self):
        s = Stats()
        _check(lib().pl_get_stats(self._h, C.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}

    # ---- hooks ------------------------------------------------------------------------------------
    def debug_get_logits(self, n):
        out = np.empty((n, self.cfg.vocab), np.float32)
        _check(lib().pl_debug_get_logits(self._h, _np_ptr(out), out.size))
        return out

    def debug_read_kv(self, slot, layer, n_ctx):
        shp = (n_ctx, self.cfg.n_kv_heads, self.cfg.head_dim)
        k, v = np.empty(shp, np.float32), np.empty(shp, np.float32)
        _check(lib().pl_debug_read_kv(self._h, slot, layer, _np_ptr(k), _np_ptr(v), n_ctx))
        return k, v

    def debug_write_kv(self, slot, layer, k, v):
        k, v = np.ascontiguousarray(k, np.float32), np.ascontiguousarray(v, np.float32)
        _check(lib().pl_debug_write_kv(self._h, slot, layer, _np_ptr(k), _np_ptr(v), k.shape[0]))

    def debug_set_profile(self, level):
        _check(lib().pl_debug_set_profile(self._h, int(level)))

    def debug_set_graphs(self, on):
        _check(lib().pl_debug_set_graphs(self._h, int(bool(on))))

    def debug_set_poison(self, on):
        _check(lib().pl_debug_set_poison(self._h, int(bool(on))))

    def debug_kv_pool(self):
        p, n = C.c_void_p(), C.c_int64()
        _check(lib().pl_debug_kv_pool(self._h, C.byref(p), C.byref(n)))
        return p.value, n.value


# ---- kernel-level entry points: device addresses as integers (e.g. torch tensor .data_ptr()) --------

def pl_attention_workspace_bytes(n_seq, n_q_heads, n_kv_heads, hd, max_ctx):
    return int(lib().pl_attention_workspace_bytes(n_seq, n_q_heads, n_kv_heads, hd, max_ctx))


def pl_attention_decode(q, kv_pages, page_table, ctx_len, out, workspace, n_seq, n_q_heads, n_kv_heads, hd,
                        page_tokens, pages_per_seq, max_ctx, stream=0):
    _check(lib().pl_attention_decode(q, kv_pages, page_table, ctx_len, out, workspace, n_seq, n_q_heads, n_kv_heads,
                                     hd, page_tokens, pages_per_seq, max_ctx, stream))


def pl_kv_pack_host(pages_host, page_ids, k, v, first_pos, n_kv_heads, hd, page_tokens):
    page_ids = np.ascontiguousarray(page_ids, np.int32)
    k, v = np.ascontiguousarray(k, np.float32), np.ascontiguousarray(v, np.float32)
    assert pages_host.dtype == np.uint16 and pages_host.flags.c_contiguous
    _check(lib().pl_kv_pack_host(_np_ptr(pages_host), _np_ptr(page_ids), _np_ptr(k), _np_ptr(v), first_pos,
                                 k.shape[0], n_kv_heads, hd, page_tokens))


def pl_debug_stream_read(ptr, nbytes, nontemporal=False, stream=0):
    r = int(lib().pl_debug_stream_read(ptr, nbytes, int(bool(nontemporal)), stream))
    if r < 0:
        raise PlError(r, lib().pl_last_error().decode())
    return r


def pl_gemm_bf16(x, w, y, M, N, K, mode=0, splits=1, stream=0):
    _check(lib().pl_gemm_bf16(x, w, y, M, N, K, mode, splits, stream))


def pl_debug_gemm_cfg(cfg, x, w, y, ws, M, N, K, mode, splits, n_begin, n_end, paired=False, stream=0):
    _check(lib().pl_debug_gemm_cfg(cfg, x, w, y, ws, M, N, K, mode, splits, n_begin, n_end, int(bool(paired)), stream))


def pl_debug_gemm_plan(M_max, N, K, mode):
    """(splits, n_main, rem_splits, ws_elems) an engine of max_batch = M_max fixes for this product."""
    sp, nm, rs, ws = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
    _check(lib().pl_debug_gemm_plan(M_max, N, K, mode, C.byref(sp), C.byref(nm), C.byref(rs), C.byref(ws)))
    return sp.value, nm.value, rs.value, ws.value


def pl_debug_gemm_planned(x, w, y, ws, M_max, M, N, K, mode, stream=0):
    _check(lib().pl_debug_gemm_planned(x, w, y, ws, M_max, M, N, K, mode, stream))


def pl_sample_workspace_bytes(n, vocab):
    return int(lib().pl_sample_workspace_bytes(n, vocab))


def pl_sample(logits, n, vocab, seq_id, position, inv_temperature, forced, seed, token, logprob, workspace, stream=0):
    _check(lib().pl_sample(logits, n, vocab, seq_id, position, inv_temperature, forced, seed, token, logprob,
                           workspace, stream))


def pl_sample_static(logits, n, vocab, seq_id, position, inv_temperature, forced, seed, token, logprob, stream=0):
    _check(lib().pl_sample_static(logits, n, vocab, seq_id, position, inv_temperature, forced, seed, token, logprob, stream))


def pl_is_ess(logp_pi, logp_mu, seq_offsets, n_seq, c, w_out, seq_sums, ess_seq, totals, stream=0):
    """Device pointers (ints); see include/pl.h."""
    _check(lib().pl_is_ess(logp_pi, logp_mu, seq_offsets, n_seq, c, w_out, seq_sums, ess_seq, totals, stream))
