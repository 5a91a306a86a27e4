"""ctypes binding over the C ABI in include/mc.h (argument marshalling only).

Every step of the path runs in the library's HIP kernels.  PyTorch supplies device
memory (arenas are uint8 CUDA tensors) and the stream.  There is no CPU fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaxcode_mi355x.so")

MC_F32, MC_BF16 = 0, 1
MC_MAX_TOP_K = 4096
MC_MAX_REWARD = 64
STATUS = {0: "MC_OK", -1: "MC_ERR_INVALID", -2: "MC_ERR_STATE", -3: "MC_ERR_OOM",
          -4: "MC_ERR_DEVICE", -5: "MC_ERR_UNSUPPORTED"}
KERNEL_CLASSES = ["none", "embed", "add_rmsnorm", "linear_qkv", "rope_kv", "attn_decode",
                  "attn_merge", "attn_prefill", "linear_o", "linear_gate_up", "linear_down",
                  "linear_lm_head", "sample", "reward"]


class McError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class mc_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32)]


class mc_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wq", "wk", "wv", "wo",
                                                     "ffn_norm", "w_gate", "w_up", "w_down")] + \
               [("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class mc_arena(C.Structure):
    _fields_ = [("dev_base", C.c_void_p), ("dev_bytes", C.c_size_t), ("hip_stream", C.c_void_p),
                ("device", C.c_int32)]


class mc_session_params(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("max_prefix", "max_cands", "max_suffix", "page_tokens",
                                         "chunk_rows", "pool_pages")]


# name -> (restype, argtypes); must list every symbol include/mc.h declares
_vp, _i32, _f32, _sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
_pi32, _pf32 = C.POINTER(C.c_int32), C.POINTER(C.c_float)
SIGNATURES = {
    "mc_model_bytes": (_sz, [C.POINTER(mc_config)]),
    "mc_model_create": (C.c_int, [C.POINTER(mc_config), C.POINTER(mc_weights), C.POINTER(mc_arena), C.POINTER(_vp)]),
    "mc_model_destroy": (None, [_vp]),
    "mc_session_bytes": (_sz, [C.POINTER(mc_config), C.POINTER(mc_session_params)]),
    "mc_session_create": (C.c_int, [_vp, C.POINTER(mc_arena), C.POINTER(mc_session_params), C.POINTER(_vp)]),
    "mc_session_destroy": (None, [_vp]),
    "mc_session_reset_candidates": (C.c_int, [_vp]),
    "mc_session_sync": (C.c_int, [_vp]),
    "mc_prefill_shared": (C.c_int, [_vp, _vp, _i32]),
    "mc_extend_shared": (C.c_int, [_vp, _vp, _i32]),
    "mc_promote_candidate": (C.c_int, [_vp, _i32]),
    "mc_prefill_suffix": (C.c_int, [_vp, _vp, _i32, _i32]),
    "mc_prefill_suffix_ragged": (C.c_int, [_vp, _vp, _vp, _i32, _i32]),
    "mc_drop_candidates": (C.c_int, [_vp, _vp, _i32]),
    "mc_pause_candidates": (C.c_int, [_vp, _vp, _i32]),
    "mc_resume_candidates": (C.c_int, [_vp, _vp, _i32]),
    "mc_reward_bin": (_i32, [C.c_double, _i32, _vp]),
    "mc_best_so_far": (C.c_int, [_vp, _vp, _i32, C.c_double, _vp]),
    "mc_value_targets": (C.c_int, [_vp, _i32, C.c_double, _vp, _vp]),
    "mc_select_candidate": (_i32, [_vp, _i32]),
    "mc_median_of_max": (C.c_int, [_vp, _vp, _i32, _vp]),
    "mc_average_rank": (C.c_int, [_vp, _i32, _i32, _vp]),
    "mc_decode_step": (C.c_int, [_vp, _vp, _i32]),
    "mc_sample": (C.c_int, [_vp, _i32, _f32, _i32, _vp, _vp, _vp]),
    "mc_score_candidates": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _i32, _f32, _vp, _vp, _vp]),
    "mc_debug_copy_logits": (C.c_int, [_vp, _vp, _i32]),
    "mc_debug_page_table": (C.c_int, [_vp, _vp, _vp, _i32]),
    "mc_debug_set_free_list": (C.c_int, [_vp, _vp, _i32]),
    "mc_debug_pool_pages": (_i32, [_vp]),
    "mc_debug_set_prefix_splits": (C.c_int, [_vp, _i32]),
    "mc_last_error": (C.c_char_p, []),
    "mc_profile_begin": (C.c_int, [_vp, _i32, _i32]),
    "mc_profile_end": (C.c_int, [_vp, _pi32, C.POINTER(C.c_double)]),
    "mc_op_tiled_bytes": (_sz, [_i32, _i32]),
    "mc_op_pack_tiled": (C.c_int, [_vp, _i32, _i32, _vp, _vp]),
    "mc_op_add_rmsnorm": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _i32, _vp, _f32, _vp, _i32]),
    "mc_op_linear": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _i32, _i32]),
    "mc_op_linear_splits": (_i32, [_i32] * 5),
    "mc_op_linear_accumulate": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _vp]),
    "mc_op_linear_qkv_rope": (C.c_int, [_vp] + [_i32] * 6 + [_f32, _i32] + [_vp] * 9),
    "mc_op_linear_swiglu": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _i32]),
    "mc_op_rope_kv_write": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _f32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mc_op_attention_decode_ws": (_sz, [_i32] * 7),
    "mc_op_attention_decode": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _sz, _vp, _i32]),
    "mc_op_attention_decode_static": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _i32]),
    "mc_op_attention_decode_plan": (C.c_int, [_i32] * 8 + [_vp]),
    "mc_op_read_probe": (C.c_int, [_vp, _vp, _sz, _vp]),
    "mc_op_mfma_probe": (C.c_int, [_vp, _vp, _vp, _i32, _i32]),
    "mc_op_attention_prefill": (C.c_int, [_vp, _i32, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32]),
    "mc_op_top_list_bytes": (_sz, [_i32, _i32]),
    "mc_op_lm_head": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp]),
    "mc_op_sample_lists": (C.c_int, [_vp, _i32, _i32, _vp, _sz, _vp, _f32, _i32, _vp, _vp, _vp]),
    "mc_op_sample": (C.c_int, [_vp, _i32, _i32, _vp, _sz, _f32, _i32, _vp, _vp, _vp]),
    "mc_op_reward_score": (C.c_int, [_vp, _i32, _i32, _vp, _vp, _vp, _i32, _f32, _vp, _vp, _vp]),
}

_lib = None


def load_library(path: str = LIB_PATH):
    """Load the shared library and attach signatures.  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  Import it first so that
        # this library binds to the runtime that owns the arenas and streams, not a second copy.
        import torch  # noqa: F401
        lib = C.CDLL(path)
        with open("/proc/self/maps") as f:
            runtimes = {ln.split()[-1] for ln in f if "libamdhip64" in ln}
        if len(runtimes) > 1:
            raise RuntimeError(f"two HIP runtimes in one process: {sorted(runtimes)}")
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(code: int):
    if code != 0:
        raise McError(code, load_library().mc_last_error().decode())


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _dtype_code(name: str) -> int:
    return {"f32": MC_F32, "bf16": MC_BF16}[name]


def make_config(shape) -> mc_config:
    """shape: any object with the fields of synth.Shape."""
    return mc_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                     shape.head_dim, shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_base,
                     _dtype_code(shape.dtype))


def _arena(nbytes: int, device):
    import torch
    buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    assert buf.data_ptr() % 256 == 0
    stream = torch.cuda.current_stream(device).cuda_stream
    return buf, mc_arena(buf.data_ptr(), buf.numel(), stream, buf.device.index or 0)


class Model:
    """Weights on the device.  ``weights``: the dict layout of synth.make_weights (numpy arrays:
    float32, or uint16 bf16 bit patterns)."""

    def __init__(self, shape, weights: Dict[str, object], device="cuda:0"):
        lib = load_library()
        self.shape = shape
        self.cfg = make_config(shape)
        nbytes = lib.mc_model_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise McError(-1, lib.mc_last_error().decode())
        self._buf, arena = _arena(nbytes, device)
        L = shape.n_layers
        want = np.float32 if shape.dtype == "f32" else np.uint16
        keep = []

        def host(a):
            a = np.ascontiguousarray(a)
            assert a.dtype == want, (a.dtype, want)
            keep.append(a)
            return a.ctypes.data

        w = mc_weights()
        w.embed, w.final_norm, w.lm_head = host(weights["embed"]), host(weights["final_norm"]), host(weights["lm_head"])
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            arr = (C.c_void_p * L)(*[host(weights["layers"][l][name]) for l in range(L)])
            keep.append(arr)
            setattr(w, name, arr)
        h = C.c_void_p()
        _check(lib.mc_model_create(C.byref(self.cfg), C.byref(w), C.byref(arena), C.byref(h)))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load_library().mc_model_destroy(self.handle)
            self.handle = None

    __del__ = close


class Session:
    def __init__(self, model: Model, max_prefix: int, max_cands: int, max_suffix: int,
                 page_tokens: int, chunk_rows: int = 0, pool_pages: int = 0):
        lib = load_library()
        self.model = model
        self.params = mc_session_params(max_prefix, max_cands, max_suffix, page_tokens, chunk_rows, pool_pages)
        nbytes = lib.mc_session_bytes(C.byref(model.cfg), C.byref(self.params))
        if nbytes == 0:
            raise McError(-1, lib.mc_last_error().decode())
        self.nbytes = nbytes
        self._buf, arena = _arena(nbytes, model._buf.device)
        h = C.c_void_p()
        _check(lib.mc_session_create(model.handle, C.byref(arena), C.byref(self.params), C.byref(h)))
        self.handle = h
        self.vocab = model.shape.vocab

    def close(self):
        if getattr(self, "handle", None):
            load_library().mc_session_destroy(self.handle)
            self.handle = None

    __del__ = close

    # ---- the four calls
    def prefill_shared(self, tokens: np.ndarray):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        _check(load_library().mc_prefill_shared(self.handle, t.ctypes.data, t.shape[0]))

    def extend_shared(self, tokens: np.ndarray):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        _check(load_library().mc_extend_shared(self.handle, t.ctypes.data, t.shape[0]))

    def promote_candidate(self, cand: int):
        _check(load_library().mc_promote_candidate(self.handle, int(cand)))

    def prefill_suffix(self, suffix_tokens: np.ndarray):
        """suffix_tokens: [n_cands, len] appended to every candidate in one pass."""
        t = np.ascontiguousarray(suffix_tokens, dtype=np.int32)
        _check(load_library().mc_prefill_suffix(self.handle, t.ctypes.data, t.shape[0], t.shape[1]))

    def prefill_suffix_ragged(self, suffix_tokens: np.ndarray, lens):
        """suffix_tokens: [n_cands, max_len]; row r holds lens[r] tokens."""
        t = np.ascontiguousarray(suffix_tokens, dtype=np.int32)
        ln = np.ascontiguousarray(lens, dtype=np.int32)
        assert ln.shape == (t.shape[0],)
        _check(load_library().mc_prefill_suffix_ragged(self.handle, t.ctypes.data, ln.ctypes.data, t.shape[0], t.shape[1]))

    def drop_candidates(self, cands):
        c = np.ascontiguousarray(cands, dtype=np.int32)
        _check(load_library().mc_drop_candidates(self.handle, c.ctypes.data, c.shape[0]))

    def pause_candidates(self, cands):
        c = np.ascontiguousarray(cands, dtype=np.int32)
        _check(load_library().mc_pause_candidates(self.handle, c.ctypes.data, c.shape[0]))

    def resume_candidates(self, cands):
        c = np.ascontiguousarray(cands, dtype=np.int32)
        _check(load_library().mc_resume_candidates(self.handle, c.ctypes.data, c.shape[0]))

    def decode_step(self, tokens: Optional[np.ndarray], n_cands: Optional[int] = None):
        if tokens is None:
            _check(load_library().mc_decode_step(self.handle, None, n_cands))
        else:
            t = np.ascontiguousarray(tokens, dtype=np.int32)
            _check(load_library().mc_decode_step(self.handle, t.ctypes.data, t.shape[0]))

    def sample(self, n_cands: int, temperature: float, top_k: int, uniforms: np.ndarray,
               want_tokens: bool = True, want_topk: bool = False):
        u = np.ascontiguousarray(uniforms, dtype=np.float32)
        assert u.shape == (n_cands,)
        toks = np.empty(n_cands, np.int32) if want_tokens else None
        V = self.vocab
        greedy = temperature <= 0 or top_k == 1
        k = 1 if greedy else (V if (top_k <= 0 or top_k >= V) else top_k)
        topk = np.empty((n_cands, k), np.int32) if want_topk else None
        _check(load_library().mc_sample(self.handle, n_cands, temperature, top_k, u.ctypes.data,
                                        _np_ptr(toks), _np_ptr(topk)))
        return (toks, topk) if want_topk else toks

    def score_candidates(self, suffix_tokens: np.ndarray, suffix_lens: Sequence[int],
                         reward_ids: np.ndarray, reward_values: np.ndarray,
                         score_temperature: float = 1.0):
        st = np.ascontiguousarray(suffix_tokens, dtype=np.int32)
        B, max_len = st.shape
        lens = np.ascontiguousarray(suffix_lens, dtype=np.int32)
        ids = np.ascontiguousarray(reward_ids, dtype=np.int32)
        vals = np.ascontiguousarray(reward_values, dtype=np.float32)
        R = ids.shape[0]
        lp = np.empty((B, R), np.float32)
        sc = np.empty(B, np.float32)
        rk = np.empty(B, np.int32)
        _check(load_library().mc_score_candidates(
            self.handle, st.ctypes.data, lens.ctypes.data, B, max_len, ids.ctypes.data,
            vals.ctypes.data, R, score_temperature, lp.ctypes.data, sc.ctypes.data, rk.ctypes.data))
        return lp, sc, rk

    # ---- housekeeping and hooks
    def reset_candidates(self):
        _check(load_library().mc_session_reset_candidates(self.handle))

    def sync(self):
        _check(load_library().mc_session_sync(self.handle))

    def logits(self, n_rows: int) -> np.ndarray:
        out = np.empty((n_rows, self.vocab), np.float32)
        _check(load_library().mc_debug_copy_logits(self.handle, out.ctypes.data, n_rows))
        return out

    def page_table(self):
        mp = (self.params.max_suffix + self.params.page_tokens - 1) // self.params.page_tokens
        tab = np.empty((self.params.max_cands, mp), np.int32)
        n = np.empty(self.params.max_cands, np.int32)
        _check(load_library().mc_debug_page_table(self.handle, tab.ctypes.data, n.ctypes.data, mp))
        return tab, n

    def pool_pages(self) -> int:
        return load_library().mc_debug_pool_pages(self.handle)

    def set_free_list(self, perm: np.ndarray):
        p = np.ascontiguousarray(perm, dtype=np.int32)
        _check(load_library().mc_debug_set_free_list(self.handle, p.ctypes.data, p.shape[0]))

    def set_prefix_splits(self, n: int):
        _check(load_library().mc_debug_set_prefix_splits(self.handle, n))

    def profile_begin(self, kernel_class: str, stride: int = 1):
        _check(load_library().mc_profile_begin(self.handle, KERNEL_CLASSES.index(kernel_class), stride))

    def profile_end(self):
        n, ms = C.c_int32(), C.c_double()
        _check(load_library().mc_profile_end(self.handle, C.byref(n), C.byref(ms)))
        return n.value, ms.value


# ---- single operations on torch CUDA tensors -------------------------------------------

# ---- host-side bookkeeping of the search loop (argument marshalling only)
MC_SELECT_NONE = -100


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def reward_bin(speedup_percent: float, correct: bool, thresholds) -> int:
    th = _f64(thresholds)
    r = load_library().mc_reward_bin(float(speedup_percent), int(bool(correct)), th.ctypes.data)
    if r < 0:
        _check(r)
    return r


def best_so_far(rewards, depths, gamma: float) -> np.ndarray:
    r = _f64(rewards); d = np.ascontiguousarray(depths, dtype=np.int32)
    out = np.empty(r.shape[0], np.float64)
    _check(load_library().mc_best_so_far(r.ctypes.data, d.ctypes.data, r.shape[0], float(gamma), out.ctypes.data))
    return out


def value_targets(rewards, gamma: float):
    r = _f64(rewards)
    u = np.empty(r.shape[0], np.float64); v = np.empty(r.shape[0], np.float64)
    _check(load_library().mc_value_targets(r.ctypes.data, r.shape[0], float(gamma), u.ctypes.data, v.ctypes.data))
    return u, v


def select_candidate(speedups):
    f = _f64(speedups)
    r = load_library().mc_select_candidate(f.ctypes.data, f.shape[0])
    if r == MC_SELECT_NONE:
        return None
    if r < 0:
        _check(r)
    return r


def median_of_max(speedups_per_problem) -> float:
    counts = np.array([len(g) for g in speedups_per_problem], np.int32)
    flat = _f64(np.concatenate([np.asarray(g, np.float64) for g in speedups_per_problem]))
    out = C.c_double(0.0)
    _check(load_library().mc_median_of_max(flat.ctypes.data, counts.ctypes.data, counts.shape[0], C.addressof(out)))
    return out.value


def average_rank(max_speedup) -> np.ndarray:
    t = _f64(max_speedup)
    out = np.empty(t.shape[0], np.float64)
    _check(load_library().mc_average_rank(t.ctypes.data, t.shape[0], t.shape[1], out.ctypes.data))
    return out


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _code_of(t) -> int:
    import torch
    return {torch.float32: MC_F32, torch.bfloat16: MC_BF16}[t.dtype]


def op_pack_tiled(t):
    """Row-major bf16 [rows, K] -> the tiled layout (a flat bf16 tensor of padded size)."""
    import torch
    rows, K = t.shape
    lib = load_library()
    nbytes = lib.mc_op_tiled_bytes(rows, K)
    if nbytes == 0:
        raise McError(-1, "K must be a positive multiple of 64")
    out = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=t.device)
    _check(lib.mc_op_pack_tiled(_stream(), rows, K, t.contiguous().data_ptr(), out.data_ptr()))
    return out


def tiled_to_rowmajor(flat, rows: int, K: int):
    """Inverse of the tiled layout on the host (numpy/torch indexing only), for checks."""
    rp = (rows + 31) // 32 * 32
    v = flat.reshape(rp // 32, K // 64, 4, 2, 32, 8)          # [rt][u][c][h][row][j]
    return v.permute(0, 4, 1, 3, 2, 5).reshape(rp, K)[:rows]


def kv_page_offsets(page_tokens: int, head_dim: int):
    """Element offsets (k_off[key, d], v_off[key, d]) inside one KV head's region of a page, as
    the library lays pages out: plain ([key][hd] and [hd][key]) unless both sizes are multiples
    of 32, then blocks of 32 keys in the order the 32x32x16 MFMA reads its A operand."""
    pg, hd = page_tokens, head_dim
    key = np.arange(pg, dtype=np.int64)[:, None]
    d = np.arange(hd, dtype=np.int64)[None, :]
    if pg % 32 or hd % 32:
        return key * hd + d, d * pg + key
    blk = (key >> 5) * 32 * hd
    k_off = blk + ((d >> 4) * 64 + (key & 31) + 32 * ((d >> 3) & 1)) * 8 + (d & 7)
    k16, sl = key & 15, (key >> 4) & 1
    v_off = blk + (((d >> 5) * 2 + sl) * 64 + (d & 31) + 32 * ((k16 >> 2) & 1)) * 8 + 4 * (k16 >> 3) + (k16 & 3)
    return k_off, v_off


def kv_pages_pack(k, v):
    """k, v: [n_pages, Hkv, pg, hd] tensors -> (K pool, V pool) in the library's page layout,
    each [n_pages, Hkv, pg * hd] (torch indexing only)."""
    import torch
    n, Hkv, pg, hd = k.shape
    k_off, v_off = kv_page_offsets(pg, hd)
    ko = torch.from_numpy(k_off.reshape(-1)).to(k.device)
    vo = torch.from_numpy(v_off.reshape(-1)).to(k.device)
    kp = torch.empty((n, Hkv, pg * hd), dtype=k.dtype, device=k.device)
    vp = torch.empty_like(kp)
    kp[:, :, ko] = k.reshape(n, Hkv, pg * hd)
    vp[:, :, vo] = v.reshape(n, Hkv, pg * hd)
    return kp, vp


def kv_pages_unpack(kp, vp, page_tokens: int, head_dim: int):
    """Inverse of kv_pages_pack: pools -> (k, v), each [n_pages, Hkv, pg, hd]."""
    import torch
    n, Hkv = kp.shape[0], kp.shape[1]
    k_off, v_off = kv_page_offsets(page_tokens, head_dim)
    ko = torch.from_numpy(k_off.reshape(-1)).to(kp.device)
    vo = torch.from_numpy(v_off.reshape(-1)).to(kp.device)
    k = kp.reshape(n, Hkv, -1)[:, :, ko].reshape(n, Hkv, page_tokens, head_dim)
    v = vp.reshape(n, Hkv, -1)[:, :, vo].reshape(n, Hkv, page_tokens, head_dim)
    return k, v


def op_add_rmsnorm(x, partials, gain, eps: float, tiled: bool = False):
    """x: fp32 [rows, d] (updated in place); partials: fp32 [S, rows, d] or None.  Returns h
    ([rows, d], or the flat tiled buffer when tiled)."""
    import torch
    rows, d = x.shape
    if tiled:
        h = torch.zeros(load_library().mc_op_tiled_bytes(rows, d) // 2, dtype=gain.dtype, device=x.device)
    else:
        h = torch.empty((rows, d), dtype=gain.dtype, device=x.device)
    S = 0 if partials is None else partials.shape[0]
    _check(load_library().mc_op_add_rmsnorm(_stream(), _code_of(gain), rows, d, x.data_ptr(),
                                            None if partials is None else partials.data_ptr(), S,
                                            gain.data_ptr(), eps, h.data_ptr(), int(tiled)))
    return h


def op_linear(a, w, n_splits: int = 1, tiled_shape=None):
    """a: [M, K], w: [N, K] (same dtype).  Returns fp32 [n_splits, M, N] partial sums.
    tiled_shape=(M, N, K): a and w are flat tiled buffers."""
    import torch
    if tiled_shape is None:
        M, K = a.shape
        N = w.shape[0]
    else:
        M, N, K = tiled_shape
    out = torch.empty((n_splits, M, N), dtype=torch.float32, device=a.device)
    _check(load_library().mc_op_linear(_stream(), _code_of(a), M, N, K, a.data_ptr(), w.data_ptr(),
                                       out.data_ptr(), n_splits, int(tiled_shape is not None)))
    return out


def op_linear_accumulate(a, w, x, tiled_shape):
    """x (fp32 [M, N], device) += a w^T on tiled bf16 operands, in place."""
    M, N, K = tiled_shape
    _check(load_library().mc_op_linear_accumulate(_stream(), M, N, K, a.data_ptr(), w.data_ptr(), x.data_ptr()))
    return x


def interleave_qk_rows(wqkv, n_q_heads: int, n_kv_heads: int, head_dim: int):
    """Row order the fused QKV layer expects: in every query / key head, row 2i <- row i and
    row 2i + 1 <- row i + head_dim / 2; value heads unchanged.  wqkv: [(Hq + 2 Hkv) * hd, K]."""
    import torch
    half = head_dim // 2
    inside = torch.stack([torch.arange(half), torch.arange(half) + half], 1).reshape(-1)
    idx = []
    for head in range(n_q_heads + 2 * n_kv_heads):
        idx.append(head * head_dim + (inside if head < n_q_heads + n_kv_heads else torch.arange(head_dim)))
    return wqkv[torch.cat(idx).to(wqkv.device)]


def op_linear_qkv_rope(a, wqkv, rows, K, row_pos, row_page, row_off, n_q_heads, n_kv_heads, head_dim,
                       page_tokens, rope_base, n_pos, k_pages, v_pages):
    """a, wqkv: flat tiled bf16 buffers (wqkv rows interleaved, see interleave_qk_rows).
    Returns q [rows, Hq, hd] bf16; k_pages / v_pages are written in place."""
    import torch
    q = torch.empty((rows, n_q_heads, head_dim), dtype=torch.bfloat16, device=a.device)
    table = torch.empty((n_pos * (head_dim // 2), 2), dtype=torch.float64, device=a.device)
    _check(load_library().mc_op_linear_qkv_rope(
        _stream(), rows, n_q_heads, n_kv_heads, head_dim, page_tokens, K, rope_base, n_pos,
        a.data_ptr(), wqkv.data_ptr(), row_pos.data_ptr(), row_page.data_ptr(), row_off.data_ptr(),
        table.data_ptr(), q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr()))
    return q


def op_linear_splits(dtype: str, M: int, N: int, K: int, tiled: bool) -> int:
    return load_library().mc_op_linear_splits(_dtype_code(dtype), M, N, K, int(tiled))


def op_linear_swiglu(a, w_gate, w_up, tiled_shape=None):
    import torch
    if tiled_shape is None:
        M, K = a.shape
        N = w_gate.shape[0]
        out = torch.empty((M, N), dtype=a.dtype, device=a.device)
    else:
        M, N, K = tiled_shape
        out = torch.zeros(load_library().mc_op_tiled_bytes(M, N) // 2, dtype=a.dtype, device=a.device)
    _check(load_library().mc_op_linear_swiglu(_stream(), _code_of(a), M, N, K, a.data_ptr(),
                                              w_gate.data_ptr(), w_up.data_ptr(), out.data_ptr(),
                                              int(tiled_shape is not None)))
    return out


def op_rope_kv_write(qkv, row_pos, row_page, row_off, n_q_heads, n_kv_heads, head_dim,
                     page_tokens, rope_base, k_pages, v_pages):
    """qkv: fp32 [S, rows, (Hq+2Hkv)*hd]; k_pages/v_pages: model-dtype page pools, written in
    place.  Returns q [rows, Hq, hd] in the pools' dtype."""
    import torch
    S, rows, _ = qkv.shape
    q = torch.empty((rows, n_q_heads, head_dim), dtype=k_pages.dtype, device=qkv.device)
    _check(load_library().mc_op_rope_kv_write(
        _stream(), _code_of(k_pages), rows, n_q_heads, n_kv_heads, head_dim, page_tokens, rope_base,
        qkv.data_ptr(), S, row_pos.data_ptr(), row_page.data_ptr(), row_off.data_ptr(),
        q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr()))
    return q


def op_attention_decode(q, k_prefix, v_prefix, k_suffix, v_suffix, page_table, prefix_len,
                        suffix_len, page_tokens, prefix_splits: int = 0, out_tiled: bool = False,
                        row_len=None, out=None, static_scratch: bool = False):
    """q: [B, Hq, hd]; pools: [n_pages, Hkv, pg * hd] in the page layout (kv_pages_pack);
    page_table: int32 [B, stride]; row_len: optional int32 [B] device tensor of per-candidate
    suffix lengths.  Returns out [B, Hq, hd] (or the flat tiled [B, Hq*hd]); `out` may be passed
    in.  static_scratch: call mc_op_attention_decode_static (the library's own scratch buffer; with
    `out` given the call allocates nothing)."""
    import torch
    lib = load_library()
    B, Hq, hd = q.shape
    Hkv = (k_prefix if k_prefix is not None else k_suffix).shape[1]
    if out is None:
        if out_tiled:
            out = torch.zeros(lib.mc_op_tiled_bytes(B, Hq * hd) // 2, dtype=q.dtype, device=q.device)
        else:
            out = torch.empty_like(q)
    p = lambda t: None if t is None else t.data_ptr()
    if static_scratch:
        _check(lib.mc_op_attention_decode_static(
            _stream(), _code_of(q), B, Hq, Hkv, hd, page_tokens, prefix_len, suffix_len, q.data_ptr(),
            p(k_prefix), p(v_prefix), p(k_suffix), p(v_suffix), p(page_table),
            0 if page_table is None else page_table.shape[1], p(row_len), prefix_splits,
            out.data_ptr(), int(out_tiled)))
        return out
    ws_bytes = lib.mc_op_attention_decode_ws(B, Hq, Hkv, hd, prefix_len, suffix_len, page_tokens)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=q.device)
    _check(lib.mc_op_attention_decode(
        _stream(), _code_of(q), B, Hq, Hkv, hd, page_tokens, prefix_len, suffix_len, q.data_ptr(),
        p(k_prefix), p(v_prefix), p(k_suffix), p(v_suffix), p(page_table),
        0 if page_table is None else page_table.shape[1], p(row_len), prefix_splits, ws.data_ptr(), ws.numel(),
        out.data_ptr(), int(out_tiled)))
    return out


def op_attention_decode_plan(n_cands, n_q_heads, n_kv_heads, head_dim, page_tokens, prefix_len,
                             suffix_len, prefix_splits=0):
    """Host-only: the decode-attention launch plan as a dict (no GPU work)."""
    out = np.zeros(9, np.int32)
    _check(load_library().mc_op_attention_decode_plan(n_cands, n_q_heads, n_kv_heads, head_dim, page_tokens,
                                                      prefix_len, suffix_len, prefix_splits, out.ctypes.data))
    keys = ("prefix_items", "suffix_items", "splits", "blocks_per_split", "suffix_splits", "suffix_bps",
            "n_parts", "prefix_stride", "rb_per_item")
    return dict(zip(keys, (int(v) for v in out)))


def op_read_probe(buf, out_word):
    """One streaming read of the whole uint8 device tensor `buf` (a multiple of 64 MiB)."""
    _check(load_library().mc_op_read_probe(_stream(), buf.data_ptr(), buf.numel() * buf.element_size(), out_word.data_ptr()))


def op_mfma_probe(operands, n_workgroups: int, iters: int):
    """operands: bf16 device tensor of n_workgroups * 256 * 48 elements.  Runs the MFMA-only probe
    kernel once on the current stream; returns the flops it executed."""
    import torch
    assert operands.numel() >= n_workgroups * 256 * 48
    out = torch.empty(n_workgroups * 256, dtype=torch.float32, device=operands.device)
    _check(load_library().mc_op_mfma_probe(_stream(), operands.data_ptr(), out.data_ptr(), n_workgroups, iters))
    return n_workgroups * 4 * iters * 8 * 32768.0


def op_attention_prefill(q, items, k_prefix, v_prefix, k_suffix, v_suffix, page_table, prefix_len,
                         page_tokens, out_tiled: bool = False):
    """q: bf16 [rows, Hq, hd]; items: int32 [n, 4] on device (first row, rows, first position,
    table row or -1).  Returns out [rows, Hq, hd] (or the flat tiled [rows, Hq*hd])."""
    import torch
    lib = load_library()
    rows, Hq, hd = q.shape
    Hkv = k_prefix.shape[1]
    if out_tiled:
        out = torch.zeros(lib.mc_op_tiled_bytes(rows, Hq * hd) // 2, dtype=q.dtype, device=q.device)
    else:
        out = torch.empty_like(q)
    p = lambda t: None if t is None else t.data_ptr()
    _check(lib.mc_op_attention_prefill(
        _stream(), items.shape[0], items.data_ptr(), Hq, Hkv, hd, page_tokens, prefix_len,
        q.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(), p(k_suffix), p(v_suffix),
        p(page_table), 0 if page_table is None else page_table.shape[1], out.data_ptr(),
        int(out_tiled)))
    return out


def op_sample(logits, temperature: float, top_k: int, uniforms, shared_row: bool = False,
              want_topk: bool = False):
    """logits: fp32 [rows, V] on device; uniforms: fp32 [B] on device."""
    import torch
    B = uniforms.shape[0]
    V = logits.shape[1]
    greedy = temperature <= 0 or top_k == 1
    k = 1 if greedy else (V if (top_k <= 0 or top_k >= V) else top_k)
    toks = torch.empty(B, dtype=torch.int32, device=logits.device)
    topk = torch.empty((B, k), dtype=torch.int32, device=logits.device) if want_topk else None
    _check(load_library().mc_op_sample(_stream(), B, V, logits.data_ptr(), 0 if shared_row else V,
                                       temperature, top_k, uniforms.data_ptr(), toks.data_ptr(),
                                       None if topk is None else topk.data_ptr()))
    return (toks, topk) if want_topk else toks


def op_lm_head(a, w, tiled_shape):
    """a, w: flat tiled bf16 buffers.  Returns (logits fp32 [M, N], top lists int32 [M, N / 64, 4, 2]:
    {float bits, id} of the four largest logits of every group of 64 ids)."""
    import torch
    M, N, K = tiled_shape
    lib = load_library()
    logits = torch.empty((M, N), dtype=torch.float32, device=a.device)
    nbytes = lib.mc_op_top_list_bytes(M, N)
    if nbytes == 0:
        raise McError(-1, "N must be a positive multiple of 64")
    lists = torch.zeros((M, N // 64, 4, 2), dtype=torch.int32, device=a.device)
    _check(lib.mc_op_lm_head(_stream(), M, N, K, a.data_ptr(), w.data_ptr(), logits.data_ptr(), lists.data_ptr()))
    return logits, lists


def op_sample_lists(logits, lists, temperature: float, top_k: int, uniforms, shared_row: bool = False,
                    want_topk: bool = False):
    """op_sample reading the LM head's per-group top lists (see op_lm_head) where they suffice."""
    import torch
    B = uniforms.shape[0]
    V = logits.shape[1]
    greedy = temperature <= 0 or top_k == 1
    k = 1 if greedy else (V if (top_k <= 0 or top_k >= V) else top_k)
    toks = torch.empty(B, dtype=torch.int32, device=logits.device)
    topk = torch.empty((B, k), dtype=torch.int32, device=logits.device) if want_topk else None
    _check(load_library().mc_op_sample_lists(_stream(), B, V, logits.data_ptr(), 0 if shared_row else V,
                                             lists.data_ptr(), temperature, top_k, uniforms.data_ptr(),
                                             toks.data_ptr(), None if topk is None else topk.data_ptr()))
    return (toks, topk) if want_topk else toks


def op_reward_score(logits, reward_ids, reward_values, score_temperature: float = 1.0):
    import torch
    B, V = logits.shape
    R = reward_ids.shape[0]
    lp = torch.empty((B, R), dtype=torch.float32, device=logits.device)
    sc = torch.empty(B, dtype=torch.float32, device=logits.device)
    rk = torch.empty(B, dtype=torch.int32, device=logits.device)
    _check(load_library().mc_op_reward_score(_stream(), B, V, logits.data_ptr(), reward_ids.data_ptr(),
                                             reward_values.data_ptr(), R, score_temperature,
                                             lp.data_ptr(), sc.data_ptr(), rk.data_ptr()))
    return lp, sc, rk
