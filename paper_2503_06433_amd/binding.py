"""ctypes binding of include/seesaw_rt.h: same names, argument marshalling only.

The library is loaded from this directory and nothing else: if it is missing the
import of a Context fails loudly (there is no fallback path)."""
import ctypes as C
import os

import numpy as np

SS_F32, SS_BF16, SS_F16 = 0, 1, 2
SS_PP, SS_TP = 0, 1
SS_ATTN, SS_MLP, SS_BOTH, SS_NO_RESIDUAL = 1, 2, 3, 4
SS_OUT, SS_IN = 0, 1
SS_HOST, SS_DEVICE = 0, 1
SS_OK, SS_EINVAL, SS_ENOMEM, SS_ENOENT, SS_EHIP = 0, -1, -2, -3, -4

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path():
    return os.path.join(_HERE, "libseesaw_rt.so")


class SeesawError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("seesaw_rt error %d: %s" % (code, text))
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("n_layers", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32), ("page_size", C.c_int32)]


class RuntimeCfg(C.Structure):
    _fields_ = [("gpu_kv_pages", C.c_int64), ("host_tier_bytes", C.c_int64), ("pinned_bytes", C.c_int64),
                ("device", C.c_int32), ("max_seq_len", C.c_int32)]


class ShardDesc(C.Structure):
    _fields_ = [("mode", C.c_int32), ("k", C.c_int32), ("shard", C.c_int32),
                ("layer_begin", C.c_int32), ("layer_end", C.c_int32)]

    def __init__(self, mode, k, shard, layer_begin, layer_end):
        super().__init__(mode, k, shard, layer_begin, layer_end)


class _Batch(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("seq_ids", C.POINTER(C.c_int64)), ("q_lens", C.POINTER(C.c_int32)),
                ("kv_lens_before", C.POINTER(C.c_int32))]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")] + \
               [("location", C.c_int32)]


_lib = None


class OfflineCfg(C.Structure):
    _fields_ = [("prefill", ShardDesc), ("decode", ShardDesc), ("max_prefill_tokens", C.c_int32),
                ("max_decode_seqs", C.c_int32), ("reshard_weights", C.c_int32), ("swap_in_group", C.c_int32)]


class OfflineStats(C.Structure):
    _fields_ = [("prefill_batches", C.c_int64), ("decode_steps", C.c_int64), ("to_decode", C.c_int64),
                ("to_prefill", C.c_int64), ("tokens", C.c_int64), ("prefill_seconds", C.c_double),
                ("decode_seconds", C.c_double), ("switch_seconds", C.c_double), ("total_seconds", C.c_double)]


def load_library():
    """Loads libseesaw_rt.so and declares every entry point of seesaw_rt.h."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2503_06433_amd.build`" % path)
    lib = C.CDLL(path)
    P, I, L, V = C.POINTER, C.c_int, C.c_int64, C.c_void_p
    D = P(ShardDesc)
    sig = {
        "ss_create": (I, [P(ModelCfg), P(RuntimeCfg), P(V)]),
        "ss_destroy": (I, [V]),
        "ss_last_error": (C.c_char_p, [V]),
        "ss_load_layer": (I, [V, D, I, P(_LayerWeights)]),
        "ss_host_weights_put": (I, [V, I, P(_LayerWeights)]),
        "ss_reshard_weights": (I, [V, D, D, V]),
        "ss_weights_wait": (I, [V, D]),
        "ss_weights_shard_bytes": (L, [V, D]),
        "ss_weights_read": (I, [V, D, I, I, V]),
        "ss_layer_prefill": (I, [V, D, I, I, P(_Batch), V, V, V]),
        "ss_layer_decode": (I, [V, D, I, I, P(_Batch), V, V, V]),
        "ss_layers_prefill": (I, [V, D, P(_Batch), V, V, V]),
        "ss_layers_decode": (I, [V, D, P(_Batch), V, V, V]),
        "ss_kv_swap": (I, [V, D, I, P(L), I, V]),
        "ss_kv_reshard": (I, [V, D, D, P(L), I, V]),
        "ss_sync": (I, [V]),
        "ss_kv_jobs_issued": (L, [V]),
        "ss_kv_wait": (I, [V, L]),
        "ss_kv_free": (I, [V, D, P(L), I]),
        "ss_host_tier_release": (I, [V, P(L), I]),
        "ss_kv_export_dev": (I, [V, D, P(L), I, V, V]),
        "ss_kv_import_dev": (I, [V, D, P(L), P(C.c_int32), I, V, V]),
        "ss_kv_page_table": (I, [V, D, L, P(C.c_int32), P(C.c_int32)]),
        "ss_kv_seq_len": (I, [V, D, L, P(C.c_int32)]),
        "ss_kv_read": (I, [V, D, L, I, V]),
        "ss_host_tier_read": (I, [V, L, I, V]),
        "ss_host_tier_used_bytes": (L, [V]),
        "ss_kv_free_pages": (L, [V, D]),
        "ss_load_head": (I, [V, V, V, V]),
        "ss_embed": (I, [V, P(C.c_int32), I, V, V]),
        "ss_lm_head": (I, [V, V, I, V, V]),
        "ss_lm_head_noalloc": (I, [V, V, I, V, V]),
        "ss_get_config": (I, [V, P(ModelCfg), P(RuntimeCfg)]),
        "ss_offline_run": (I, [V, P(OfflineCfg), C.c_int32, P(C.c_int32), P(C.c_int32), P(C.c_int32), P(C.c_int32),
                               P(C.c_int32), L, P(L), P(OfflineStats), V]),
        "ss_prof_enable": (I, [V, I]),
        "ss_prof_read": (I, [V, I, P(C.c_double), P(L)]),
        "ss_prof_reset": (I, [V]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


EXPORTED = ("ss_create ss_destroy ss_last_error ss_load_layer ss_host_weights_put ss_reshard_weights ss_weights_wait "
            "ss_weights_shard_bytes ss_weights_read ss_layer_prefill ss_layer_decode ss_layers_prefill ss_layers_decode ss_kv_swap "
            "ss_kv_reshard ss_sync ss_kv_jobs_issued ss_kv_wait ss_kv_free ss_host_tier_release ss_kv_export_dev ss_kv_import_dev "
            "ss_kv_page_table ss_kv_seq_len ss_kv_read ss_host_tier_read ss_host_tier_used_bytes "
            "ss_kv_free_pages ss_load_head ss_embed ss_lm_head ss_lm_head_noalloc ss_get_config ss_offline_run ss_prof_enable ss_prof_read ss_prof_reset").split()


W_NAMES = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")     # index = SS_W_* of the header


def _ptr(x):
    """Raw address of a torch tensor, a numpy array, or an int."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Context:
    """One GPU's runtime.  Methods carry the C names without the ss_ prefix."""

    def __init__(self, model, runtime):
        self.lib = load_library()
        self.model, self.runtime = model, runtime
        self.h = C.c_void_p()
        rc = self.lib.ss_create(C.byref(model), C.byref(runtime), C.byref(self.h))
        if rc != SS_OK:
            raise SeesawError(rc, "ss_create failed")

    def _ck(self, rc):
        if rc != SS_OK:
            raise SeesawError(rc, self.lib.ss_last_error(self.h).decode())

    def destroy(self):
        if self.h:
            self.lib.ss_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- weights
    def load_layer(self, desc, layer, weights, location=SS_HOST):
        """weights: dict name -> numpy array (host) or torch tensor (device)."""
        keep = {k: (np.ascontiguousarray(v) if isinstance(v, np.ndarray) else v.contiguous()) for k, v in weights.items()}
        lw = _LayerWeights(*[_ptr(keep[n]) for n in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")], location)
        self._ck(self.lib.ss_load_layer(self.h, C.byref(desc), layer, C.byref(lw)))

    def host_weights_put(self, layer, weights, location=SS_HOST):
        """Copies a layer's full weights (dict as for load_layer) into the library's CPU copy of the model."""
        keep = {k: (np.ascontiguousarray(v) if isinstance(v, np.ndarray) else v.contiguous()) for k, v in weights.items()}
        lw = _LayerWeights(*[_ptr(keep[n]) for n in W_NAMES], location)
        self._ck(self.lib.ss_host_weights_put(self.h, layer, C.byref(lw)))

    def reshard_weights(self, src, dst, stream=0):
        """src may be None (nothing is released)."""
        self._ck(self.lib.ss_reshard_weights(self.h, C.byref(src) if src is not None else None, C.byref(dst), stream))

    def weights_wait(self, desc):
        self._ck(self.lib.ss_weights_wait(self.h, C.byref(desc)))

    def weights_shard_bytes(self, desc):
        n = self.lib.ss_weights_shard_bytes(self.h, C.byref(desc))
        if n < 0:
            self._ck(int(n))
        return int(n)

    def weights_read(self, desc, layer, which, n_elems):
        """Raw storage bits (uint16 for bf16, float32 for fp32) of the slice `which` the shard holds."""
        out = np.empty(n_elems, dtype=np.float32 if self.model.dtype == SS_F32 else np.uint16)
        self._ck(self.lib.ss_weights_read(self.h, C.byref(desc), layer, which, out.ctypes.data))
        return out

    def offline_run(self, prefill, decode, prompts, out_lens, max_prefill_tokens, max_decode_seqs, reshard_weights=True,
                    stream=0, trace_cap=1 << 20, swap_in_group=0):
        """prompts: list of int arrays.  Returns (tokens per request, trace as [(code, [ids])], stats dict)."""
        cfg = OfflineCfg(prefill, decode, max_prefill_tokens, max_decode_seqs, 1 if reshard_weights else 0, swap_in_group)
        n = len(prompts)
        p_lens = _i32([len(p) for p in prompts])
        p_toks = _i32(np.concatenate([np.asarray(p) for p in prompts]) if n else [])
        o_lens = _i32(out_lens)
        toks = np.zeros(max(int(o_lens.sum()), 1), dtype=np.int32)
        trace = np.zeros(trace_cap, dtype=np.int32)
        tlen = C.c_int64(0)
        st = OfflineStats()
        i32p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
        self._ck(self.lib.ss_offline_run(self.h, C.byref(cfg), n, i32p(p_lens), i32p(p_toks), i32p(o_lens), i32p(toks),
                                         i32p(trace), trace_cap, C.byref(tlen), C.byref(st), stream))
        out, o = [], 0
        for k in o_lens:
            out.append(toks[o:o + int(k)].copy())
            o += int(k)
        rec, i = [], 0
        while i < tlen.value:
            cnt = int(trace[i + 1])
            rec.append((int(trace[i]), [int(v) for v in trace[i + 2:i + 2 + cnt]]))
            i += 2 + cnt
        return out, rec, {f: getattr(st, f) for f, _ in OfflineStats._fields_}

    def load_head(self, embed, gf, wlm):
        e, g, w = (np.ascontiguousarray(a) for a in (embed, gf, wlm))
        self._ck(self.lib.ss_load_head(self.h, _ptr(e), _ptr(g), _ptr(w)))

    # ---- layers
    def _batch(self, seq_ids, q_lens, kv_before):
        s, q, b = _i64(seq_ids), _i32(q_lens), _i32(kv_before)
        bt = _Batch(len(s), s.ctypes.data_as(C.POINTER(C.c_int64)), q.ctypes.data_as(C.POINTER(C.c_int32)),
                    b.ctypes.data_as(C.POINTER(C.c_int32)))
        return bt, (s, q, b)

    def layer_prefill(self, desc, layer, phase, seq_ids, q_lens, kv_before, x_in, out, stream=0):
        bt, keep = self._batch(seq_ids, q_lens, kv_before)
        self._ck(self.lib.ss_layer_prefill(self.h, C.byref(desc), layer, phase, C.byref(bt), _ptr(x_in), _ptr(out), stream))

    def layer_decode(self, desc, layer, phase, seq_ids, kv_before, x_in, out, stream=0):
        bt, keep = self._batch(seq_ids, np.ones(len(seq_ids), dtype=np.int32), kv_before)
        self._ck(self.lib.ss_layer_decode(self.h, C.byref(desc), layer, phase, C.byref(bt), _ptr(x_in), _ptr(out), stream))

    def layers_prefill(self, desc, seq_ids, q_lens, kv_before, x_in, out, stream=0):
        bt, keep = self._batch(seq_ids, q_lens, kv_before)
        self._ck(self.lib.ss_layers_prefill(self.h, C.byref(desc), C.byref(bt), _ptr(x_in), _ptr(out), stream))

    def layers_decode(self, desc, seq_ids, kv_before, x_in, out, stream=0):
        bt, keep = self._batch(seq_ids, np.ones(len(seq_ids), dtype=np.int32), kv_before)
        self._ck(self.lib.ss_layers_decode(self.h, C.byref(desc), C.byref(bt), _ptr(x_in), _ptr(out), stream))

    # ---- KV movement
    def kv_swap(self, desc, direction, seq_ids, stream=0):
        s = _i64(seq_ids)
        self._ck(self.lib.ss_kv_swap(self.h, C.byref(desc), direction, s.ctypes.data_as(C.POINTER(C.c_int64)), len(s), stream))

    def kv_reshard(self, src, dst, seq_ids, stream=0):
        s = _i64(seq_ids)
        self._ck(self.lib.ss_kv_reshard(self.h, C.byref(src), C.byref(dst), s.ctypes.data_as(C.POINTER(C.c_int64)), len(s), stream))

    def sync(self):
        self._ck(self.lib.ss_sync(self.h))

    def kv_jobs_issued(self):
        return self.lib.ss_kv_jobs_issued(self.h)

    def kv_wait(self, n_jobs):
        self._ck(self.lib.ss_kv_wait(self.h, n_jobs))

    def kv_free(self, desc, seq_ids):
        s = _i64(seq_ids)
        self._ck(self.lib.ss_kv_free(self.h, C.byref(desc), s.ctypes.data_as(C.POINTER(C.c_int64)), len(s)))

    def host_tier_release(self, seq_ids):
        s = _i64(seq_ids)
        self._ck(self.lib.ss_host_tier_release(self.h, s.ctypes.data_as(C.POINTER(C.c_int64)), len(s)))

    def kv_export_dev(self, desc, seq_ids, staging, stream=0):
        s = _i64(seq_ids)
        self._ck(self.lib.ss_kv_export_dev(self.h, C.byref(desc), s.ctypes.data_as(C.POINTER(C.c_int64)), len(s), _ptr(staging), stream))

    def kv_import_dev(self, desc, seq_ids, lens, staging, stream=0):
        s, l = _i64(seq_ids), _i32(lens)
        self._ck(self.lib.ss_kv_import_dev(self.h, C.byref(desc), s.ctypes.data_as(C.POINTER(C.c_int64)),
                                           l.ctypes.data_as(C.POINTER(C.c_int32)), len(s), _ptr(staging), stream))

    # ---- inspection
    def kv_page_table(self, desc, seq):
        n = C.c_int32(0)
        self._ck(self.lib.ss_kv_page_table(self.h, C.byref(desc), seq, None, C.byref(n)))
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        n2 = C.c_int32(n.value)
        self._ck(self.lib.ss_kv_page_table(self.h, C.byref(desc), seq, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n2)))
        return out[: n.value]

    def kv_seq_len(self, desc, seq):
        n = C.c_int32(0)
        self._ck(self.lib.ss_kv_seq_len(self.h, C.byref(desc), seq, C.byref(n)))
        return n.value

    def _np_dtype(self):
        return np.float32 if self.model.dtype == SS_F32 else np.uint16

    def kv_read(self, desc, seq, layer, heads_local):
        s = self.kv_seq_len(desc, seq)
        out = np.zeros((2, heads_local, s, self.model.head_dim), dtype=self._np_dtype())
        self._ck(self.lib.ss_kv_read(self.h, C.byref(desc), seq, layer, out.ctypes.data))
        return out

    def host_tier_read(self, seq, layer, length):
        out = np.zeros((2, self.model.n_kv_heads, length, self.model.head_dim), dtype=self._np_dtype())
        self._ck(self.lib.ss_host_tier_read(self.h, seq, layer, out.ctypes.data))
        return out

    def host_tier_used_bytes(self):
        return self.lib.ss_host_tier_used_bytes(self.h)

    def kv_free_pages(self, desc):
        return self.lib.ss_kv_free_pages(self.h, C.byref(desc))

    # ---- tiny-model helpers
    def embed(self, token_ids, x_out, stream=0):
        t = _i32(token_ids)
        self._ck(self.lib.ss_embed(self.h, t.ctypes.data_as(C.POINTER(C.c_int32)), len(t), _ptr(x_out), stream))

    def lm_head(self, x, n, logits, stream=0):
        self._ck(self.lib.ss_lm_head(self.h, _ptr(x), n, _ptr(logits), stream))

    def lm_head_noalloc(self, x, n, logits, stream=0):
        self._ck(self.lib.ss_lm_head_noalloc(self.h, _ptr(x), n, _ptr(logits), stream))

    # ---- timing hooks
    def prof_enable(self, on):
        self._ck(self.lib.ss_prof_enable(self.h, int(on)))

    def prof_reset(self):
        self._ck(self.lib.ss_prof_reset(self.h))

    def prof_read(self, cls):
        ms, n = C.c_double(0), C.c_int64(0)
        self._ck(self.lib.ss_prof_read(self.h, cls, C.byref(ms), C.byref(n)))
        return ms.value, n.value
