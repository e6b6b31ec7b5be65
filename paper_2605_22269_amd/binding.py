"""ctypes binding of libmukv.so -- argument marshalling only.

The functions carry the names of the C ABI in ``include/mukv.h``.  ``MuKV`` is a
small convenience object that owns a context and passes torch tensors' device
pointers, strides and the current HIP stream through; every step of the method
runs inside the library's kernels.  There is no CPU fallback: if the library
has not been built, loading raises.
"""
from __future__ import annotations

import collections
import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmukv.so")

MUKV_OK, MUKV_ERR_INVALID_ARG, MUKV_ERR_SHAPE, MUKV_ERR_CAPACITY, MUKV_ERR_UNSUPPORTED, MUKV_ERR_HIP = 0, -1, -2, -3, -4, -5
MUKV_BF16, MUKV_F32 = 0, 1
MUKV_SEMI, MUKV_HIER, MUKV_PARALLEL = 0, 1, 2
MUKV_TEMPORAL, MUKV_AS_GIVEN = 0, 1
MUKV_ATT_AUTO, MUKV_ATT_GENERIC, MUKV_ATT_MFMA = 0, 1, 2
MUKV_FREQ_FEATURE, MUKV_FREQ_TOKEN = 0, 1


class mukv_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("tokens_per_frame", C.c_int32), ("frames_per_segment", C.c_int32), ("superpatches_per_frame", C.c_int32),
        ("dtype", C.c_int32), ("keep_ratio", C.c_double), ("alpha", C.c_double), ("causal", C.c_int32),
        ("score_layer", C.c_int32), ("max_frames", C.c_int32), ("max_chunk_frames", C.c_int32),
        ("max_questions", C.c_int32), ("device_id", C.c_int32), ("att_path", C.c_int32), ("batch_chunks", C.c_int32),
        ("refine_margin", C.c_double), ("overlap_copy", C.c_int32), ("freq_axis", C.c_int32),
    ]


class mukv_strides(C.Structure):
    _fields_ = [("layer", C.c_int64), ("head", C.c_int64), ("token", C.c_int64)]


class mukv_signals_out(C.Structure):
    _fields_ = [("att", C.c_void_p), ("fft", C.c_void_p), ("fused", C.c_void_p)]


class mukv_retrieve_params(C.Structure):
    _fields_ = [
        ("mode", C.c_int32), ("k_seg", C.c_int32), ("k_frame", C.c_int32), ("n_global", C.c_int32),
        ("n_visible_frames", C.c_int32), ("reserved0", C.c_int32), ("lambda_frame", C.c_double),
    ]


class mukv_state(C.Structure):
    _fields_ = [
        ("n_frames", C.c_int64), ("n_segments", C.c_int64), ("n_kept_tokens", C.c_int64),
        ("store_token_capacity", C.c_int64), ("kappa", C.c_int32), ("c_kv", C.c_int32),
        ("store_k", C.c_void_p), ("store_v", C.c_void_p), ("kept_idx", C.c_void_p),
        ("rep_frame_k", C.c_void_p), ("rep_frame_v", C.c_void_p), ("rep_patch_k", C.c_void_p),
        ("rep_patch_v", C.c_void_p), ("cnt_patch", C.c_void_p), ("rep_seg_k", C.c_void_p),
        ("rep_seg_v", C.c_void_p), ("margin", C.c_void_p), ("refined", C.c_void_p), ("patch_cap", C.c_int32),
    ]


KERNEL_NAMES = ("att", "freq", "select", "refine", "compact", "poolq", "score", "rerank", "gather", "copy_freq", "chain")


class mukv_profile(C.Structure):
    _fields_ = [("ms", C.c_double * len(KERNEL_NAMES)), ("launches", C.c_int64 * len(KERNEL_NAMES))]


EXPORTS = ("mukv_create", "mukv_destroy", "mukv_reset", "mukv_flush", "mukv_compress_chunk", "mukv_retrieve",
           "mukv_retrieve_patches", "mukv_retrieve_at", "mukv_retrieve_units", "mukv_gather_multi", "mukv_gather_kv", "mukv_gather_patches", "mukv_gather_union",
           "mukv_attend", "mukv_prefill_workspace_size", "mukv_prefill_attend", "mukv_prefill_attend_static",
           "mukv_snapshot_size", "mukv_snapshot_save", "mukv_snapshot_load", "mukv_profile_begin", "mukv_profile_end",
           "mukv_plain_copy", "mukv_get_state", "mukv_strerror")

_lib = None


def load():
    """Loads libmukv.so (built by ``paper_2605_22269_amd.build``); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2605_22269_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.mukv_create.argtypes = [C.POINTER(mukv_config), C.POINTER(vp)]
    lib.mukv_destroy.argtypes = [vp]
    lib.mukv_reset.argtypes = [vp]
    lib.mukv_flush.argtypes = [vp]
    lib.mukv_compress_chunk.argtypes = [vp, vp, vp, C.POINTER(mukv_strides), vp, C.POINTER(mukv_strides), vp, i32, vp,
                                        C.POINTER(mukv_signals_out)]
    lib.mukv_retrieve.argtypes = [vp, vp, vp, i32, C.POINTER(mukv_retrieve_params), vp, vp, vp, vp, vp]
    lib.mukv_gather_kv.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.mukv_retrieve_patches.argtypes = [vp, vp, vp, i32, C.POINTER(mukv_retrieve_params), vp, vp, vp]
    lib.mukv_gather_patches.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.mukv_retrieve_at.argtypes = [vp, vp, vp, vp, i32, C.POINTER(mukv_retrieve_params), i32, vp, vp, vp, vp, vp]
    lib.mukv_gather_union.argtypes = [vp, vp, i32, vp, i32, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.mukv_attend.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp, vp, i32, i32, vp, vp]
    lib.mukv_retrieve_units.argtypes = [vp, vp, vp, i32, i32, C.c_double, i32, vp, i32, vp, vp, vp, vp]
    lib.mukv_gather_multi.argtypes = [C.POINTER(vp), i32, C.POINTER(vp), C.POINTER(i32), C.POINTER(i32), i32, i32, vp, vp,
                                      vp, vp]
    lib.mukv_prefill_workspace_size.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_int64)]
    lib.mukv_prefill_attend.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp, vp, i32, i32, vp, vp, vp, C.c_int64, vp]
    lib.mukv_prefill_attend_static.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.mukv_snapshot_size.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.mukv_snapshot_save.argtypes = [vp, vp, C.c_int64, vp]
    lib.mukv_snapshot_load.argtypes = [vp, vp, C.c_int64, vp]
    lib.mukv_get_state.argtypes = [vp, C.POINTER(mukv_state)]
    lib.mukv_plain_copy.argtypes = [vp, vp, C.c_int64, vp]
    lib.mukv_profile_begin.argtypes = [vp]
    lib.mukv_profile_end.argtypes = [vp, C.POINTER(mukv_profile)]
    lib.mukv_strerror.argtypes = [i32]
    lib.mukv_strerror.restype = C.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def gather_multi(stores, idx_list, units_per_step, rows_cap):
    """One decode context from several MuKV stores: idx_list[i] int32 [B][k_i] device tensors of chosen units.
    Returns (k_out, v_out, n_tokens) with k_out, v_out [B][L][Hkv][rows_cap][D]."""
    s0 = stores[0]
    B = idx_list[0].shape[0]
    dev = idx_list[0].device
    shape = (B, s0.cfg.n_layers, s0.cfg.n_kv_heads, rows_cap, s0.cfg.head_dim)
    ko = torch.empty(shape, dtype=s0.dtype, device=dev)
    vo = torch.empty(shape, dtype=s0.dtype, device=dev)
    nt = torch.empty(B, dtype=torch.int32, device=dev)
    mukv_gather_multi([s.h for s in stores], [_ptr(i) for i in idx_list], [int(i.shape[1]) for i in idx_list],
                      list(units_per_step), B, rows_cap, _ptr(ko), _ptr(vo), _ptr(nt), _stream())
    for s in stores:
        s._held.clear()
    return ko, vo, nt


class MuKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {load().mukv_strerror(status).decode()} ({status})")


def _check(status: int, where: str):
    if status != MUKV_OK:
        raise MuKVError(status, where)


# ---- functions named after the C ABI -------------------------------------------------------
def mukv_create(cfg: mukv_config) -> C.c_void_p:
    h = C.c_void_p()
    _check(load().mukv_create(C.byref(cfg), C.byref(h)), "mukv_create")
    return h


def mukv_destroy(h):
    _check(load().mukv_destroy(h), "mukv_destroy")


def mukv_reset(h):
    _check(load().mukv_reset(h), "mukv_reset")


def mukv_flush(h):
    _check(load().mukv_flush(h), "mukv_flush")


def mukv_compress_chunk(h, k_ptr, v_ptr, kv_strides, q_ptr, q_strides, att_ptr, n_frames, stream, sig=None):
    _check(load().mukv_compress_chunk(h, k_ptr, v_ptr, C.byref(kv_strides), q_ptr,
                                      C.byref(q_strides) if q_strides is not None else None, att_ptr, n_frames,
                                      stream, C.byref(sig) if sig is not None else None), "mukv_compress_chunk")


def mukv_retrieve(h, q_ptr, off_ptr, B, params, seg_idx, seg_score, frm_idx, frm_score, stream):
    _check(load().mukv_retrieve(h, q_ptr, off_ptr, B, C.byref(params), seg_idx, seg_score, frm_idx, frm_score, stream),
           "mukv_retrieve")


def mukv_gather_kv(h, idx_ptr, B, k_frame, order, k_out, v_out, n_tok, stream):
    _check(load().mukv_gather_kv(h, idx_ptr, B, k_frame, order, k_out, v_out, n_tok, stream), "mukv_gather_kv")


def mukv_retrieve_patches(h, q_ptr, off_ptr, B, params, patch_idx, patch_score, stream):
    _check(load().mukv_retrieve_patches(h, q_ptr, off_ptr, B, C.byref(params), patch_idx, patch_score, stream),
           "mukv_retrieve_patches")


def mukv_retrieve_at(h, q_ptr, off_ptr, nv_ptr, B, params, level, seg_idx, seg_score, fine_idx, fine_score, stream):
    _check(load().mukv_retrieve_at(h, q_ptr, off_ptr, nv_ptr, B, C.byref(params), level, seg_idx, seg_score, fine_idx,
                                   fine_score, stream), "mukv_retrieve_at")


def mukv_gather_patches(h, idx_ptr, B, k_patch, order, k_out, v_out, n_tok, stream):
    _check(load().mukv_gather_patches(h, idx_ptr, B, k_patch, order, k_out, v_out, n_tok, stream), "mukv_gather_patches")


def mukv_gather_union(h, seg_ptr, k_seg, frm_ptr, k_frame, pat_ptr, k_patch, B, rows_cap, k_out, v_out, n_tok, stream):
    _check(load().mukv_gather_union(h, seg_ptr, k_seg, frm_ptr, k_frame, pat_ptr, k_patch, B, rows_cap, k_out, v_out, n_tok,
                                    stream), "mukv_gather_union")


def mukv_attend(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B, causal_local, out_ptr, stream):
    _check(load().mukv_attend(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B, causal_local, out_ptr,
                              stream), "mukv_attend")


def mukv_retrieve_units(h, q_ptr, off_ptr, B, k, lambda_g, n_visible, g_in_ptr, n_global, g_out_ptr, idx_ptr, score_ptr,
                        stream):
    _check(load().mukv_retrieve_units(h, q_ptr, off_ptr, B, k, lambda_g, n_visible, g_in_ptr, n_global, g_out_ptr,
                                      idx_ptr, score_ptr, stream), "mukv_retrieve_units")


def mukv_gather_multi(handles, idx_ptrs, ks, units_per_step, B, rows_cap, k_out_ptr, v_out_ptr, n_tok_ptr, stream):
    n = len(handles)
    raw = lambda p: p.value if isinstance(p, C.c_void_p) else p
    hs = (C.c_void_p * n)(*[raw(h) for h in handles])
    ips = (C.c_void_p * n)(*[raw(p) for p in idx_ptrs])
    kk = (C.c_int32 * n)(*ks)
    ups = (C.c_int32 * n)(*units_per_step)
    _check(load().mukv_gather_multi(hs, n, ips, kk, ups, B, rows_cap, k_out_ptr, v_out_ptr, n_tok_ptr, stream),
           "mukv_gather_multi")


def mukv_prefill_workspace_size(h, n_q, k_frame, B):
    n = C.c_int64(0)
    _check(load().mukv_prefill_workspace_size(h, n_q, k_frame, B, C.byref(n)), "mukv_prefill_workspace_size")
    return n.value


def mukv_prefill_attend(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B, causal_local, out_ptr, sig_ptr,
                        ws_ptr, ws_bytes, stream):
    _check(load().mukv_prefill_attend(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B, causal_local,
                                      out_ptr, sig_ptr, ws_ptr, ws_bytes, stream), "mukv_prefill_attend")


MUKV_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def mukv_prefill_attend_static(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B, causal_local, out_ptr,
                               sig_ptr, stream):
    _check(load().mukv_prefill_attend_static(h, layer, q_ptr, n_q, idx_ptr, k_frame, kl_ptr, vl_ptr, loff_ptr, B,
                                             causal_local, out_ptr, sig_ptr, stream), "mukv_prefill_attend_static")


def mukv_snapshot_size(h) -> int:
    n = C.c_int64()
    _check(load().mukv_snapshot_size(h, C.byref(n)), "mukv_snapshot_size")
    return n.value


def mukv_snapshot_save(h, host_ptr, n_bytes, stream):
    _check(load().mukv_snapshot_save(h, host_ptr, n_bytes, stream), "mukv_snapshot_save")


def mukv_snapshot_load(h, host_ptr, n_bytes, stream):
    _check(load().mukv_snapshot_load(h, host_ptr, n_bytes, stream), "mukv_snapshot_load")


def mukv_profile_begin(h):
    _check(load().mukv_profile_begin(h), "mukv_profile_begin")


def mukv_profile_end(h) -> dict:
    p = mukv_profile()
    _check(load().mukv_profile_end(h, C.byref(p)), "mukv_profile_end")
    return {n: {"ms": p.ms[i], "launches": p.launches[i]} for i, n in enumerate(KERNEL_NAMES)}


def mukv_plain_copy(dst_ptr, src_ptr, n_bytes, stream):
    _check(load().mukv_plain_copy(dst_ptr, src_ptr, n_bytes, stream), "mukv_plain_copy")


def mukv_get_state(h) -> mukv_state:
    s = mukv_state()
    _check(load().mukv_get_state(h, C.byref(s)), "mukv_get_state")
    return s


# ---- convenience object ----------------------------------------------------------------------
_hip = None


def _hip_rt():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMemcpyAsync.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        _hip.hipMemcpyAsync.restype = C.c_int
    return _hip


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class MuKV:
    """Owns one mukv_ctx.  All tensors must live on the context's device."""

    def __init__(self, *, n_layers, n_q_heads, n_kv_heads, head_dim, tokens_per_frame, frames_per_segment,
                 superpatches_per_frame=4, dtype=torch.bfloat16, keep_ratio=0.25, alpha=0.7, causal=True,
                 score_layer=-1, max_frames=4096, max_chunk_frames=8, max_questions=1, device_id=0,
                 att_path=MUKV_ATT_AUTO, refine_margin=-1.0, batch_chunks=1, overlap_copy=0,
                 freq_axis=MUKV_FREQ_FEATURE):
        self.cfg = mukv_config(n_layers, n_q_heads, n_kv_heads, head_dim, tokens_per_frame, frames_per_segment,
                               superpatches_per_frame, MUKV_BF16 if dtype == torch.bfloat16 else MUKV_F32,
                               keep_ratio, alpha, int(causal), score_layer, max_frames, max_chunk_frames,
                               max_questions, device_id, att_path, batch_chunks, refine_margin, overlap_copy, freq_axis)
        self.dtype = dtype
        self.device = torch.device("cuda", device_id)
        self.h = mukv_create(self.cfg)
        st = mukv_get_state(self.h)
        self.kappa, self.c_kv, self.patch_cap = st.kappa, st.c_kv, st.patch_cap
        # references to the buffers of the chunks the library may still read: the batch being
        # gathered, the two before it (overlap_copy) and one spare
        self._held = collections.deque(maxlen=4 * max(1, batch_chunks) + 1)

    def close(self):
        if self.h is not None:
            mukv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        mukv_reset(self.h)
        self._held.clear()

    def flush(self):
        mukv_flush(self.h)
        self._held.clear()   # everything that reads them is enqueued on the stream

    @property
    def n_frames(self):
        return mukv_get_state(self.h).n_frames

    def snapshot(self):
        """The cache's content as a host uint8 tensor (mukv_snapshot_save)."""
        buf = torch.empty(mukv_snapshot_size(self.h), dtype=torch.uint8)
        mukv_snapshot_save(self.h, C.c_void_p(buf.data_ptr()), buf.numel(), _stream())
        self._held.clear()
        return buf

    def restore(self, buf):
        """Replaces the content by a snapshot taken from a context of the same configuration."""
        assert buf.device.type == "cpu" and buf.dtype == torch.uint8 and buf.is_contiguous()
        mukv_snapshot_load(self.h, C.c_void_p(buf.data_ptr()), buf.numel(), _stream())
        self._held.clear()

    def compress_chunk(self, k, v, q_last=None, att_signal=None, want_signals=False):
        """k, v: [L][Hkv][n*P][D] (any layer/head/token strides, D contiguous);
        q_last: [Hq][n*P][D]; att_signal: float32 [n][P]."""
        P = self.cfg.tokens_per_frame
        assert k.dim() == 4 and k.shape == v.shape and k.stride() == v.stride() and k.stride(3) == 1
        assert k.dtype == self.dtype and k.shape[2] % P == 0
        n = k.shape[2] // P
        kvs = mukv_strides(k.stride(0), k.stride(1), k.stride(2))
        qs = None
        if q_last is not None:
            assert q_last.dim() == 3 and q_last.stride(2) == 1 and q_last.dtype == self.dtype
            assert q_last.shape[1] == k.shape[2]
            qs = mukv_strides(0, q_last.stride(0), q_last.stride(1))
        sig, outs = None, None
        if want_signals:
            outs = {n_: torch.zeros(n, P, dtype=torch.float32, device=k.device) for n_ in ("att", "fft", "fused")}
            sig = mukv_signals_out(outs["att"].data_ptr(), outs["fft"].data_ptr(), outs["fused"].data_ptr())
        if att_signal is not None:
            assert att_signal.dtype == torch.float32 and att_signal.is_contiguous() and att_signal.shape == (n, P)
        mukv_compress_chunk(self.h, _ptr(k), _ptr(v), kvs, _ptr(q_last), qs, _ptr(att_signal), n, _stream(), sig)
        # The library reads these buffers (and writes the signal outputs) when the gathered batch is
        # launched, with overlap_copy one batch later still: hold references that long.
        self._held.append((k, v, q_last, att_signal, outs))
        return outs

    def retrieve(self, q_tokens, q_offsets, *, mode=MUKV_SEMI, k_seg=8, k_frame=32, lambda_frame=0.3, n_global=0,
                 n_visible_frames=-1, out=None):
        """q_tokens: [sum Nq][Hq][D] contiguous; q_offsets: int32 [B+1] on the device."""
        assert q_tokens.is_contiguous() and q_tokens.dtype == self.dtype
        assert q_offsets.dtype == torch.int32 and q_offsets.is_cuda
        B = q_offsets.numel() - 1
        prm = mukv_retrieve_params(mode, k_seg, k_frame, n_global, n_visible_frames, 0, lambda_frame)
        if out is None:
            dev = q_tokens.device
            out = {
                "seg_idx": torch.empty(B, k_seg, dtype=torch.int32, device=dev),
                "seg_score": torch.empty(B, k_seg, dtype=torch.float32, device=dev),
                "frame_idx": torch.empty(B, k_frame, dtype=torch.int32, device=dev),
                "frame_score": torch.empty(B, k_frame, dtype=torch.float32, device=dev),
            }
        mukv_retrieve(self.h, _ptr(q_tokens), _ptr(q_offsets), B, prm, _ptr(out["seg_idx"]), _ptr(out["seg_score"]),
                      _ptr(out["frame_idx"]), _ptr(out["frame_score"]), _stream())
        self._held.clear()   # the call has enqueued everything that reads them
        return out

    def retrieve_patches(self, q_tokens, q_offsets, *, mode=MUKV_SEMI, k_seg=8, k_patch=20, lambda_patch=0.3, n_global=0,
                         n_visible_frames=-1, out=None):
        """The search of retrieve() with super-patches as the fine level; a patch is frame * S + s."""
        assert q_tokens.is_contiguous() and q_tokens.dtype == self.dtype
        assert q_offsets.dtype == torch.int32 and q_offsets.is_cuda
        B = q_offsets.numel() - 1
        prm = mukv_retrieve_params(mode, k_seg, k_patch, n_global, n_visible_frames, 0, lambda_patch)
        if out is None:
            dev = q_tokens.device
            out = {"patch_idx": torch.empty(B, k_patch, dtype=torch.int32, device=dev),
                   "patch_score": torch.empty(B, k_patch, dtype=torch.float32, device=dev)}
        mukv_retrieve_patches(self.h, _ptr(q_tokens), _ptr(q_offsets), B, prm, _ptr(out["patch_idx"]),
                              _ptr(out["patch_score"]), _stream())
        self._held.clear()
        return out

    def retrieve_at(self, q_tokens, q_offsets, n_visible, *, level="frame", mode=MUKV_SEMI, k_seg=8, k_fine=32,
                    lambda_fine=0.3, n_global=0):
        """retrieve() / retrieve_patches() for questions asked at different times: n_visible is an
        int32 tensor [B] on the device, question b sees frames < n_visible[b]."""
        assert q_tokens.is_contiguous() and q_tokens.dtype == self.dtype
        assert q_offsets.dtype == torch.int32 and q_offsets.is_cuda
        assert n_visible.dtype == torch.int32 and n_visible.is_cuda and n_visible.is_contiguous()
        B = q_offsets.numel() - 1
        assert n_visible.numel() == B
        prm = mukv_retrieve_params(mode, k_seg, k_fine, n_global, -1, 0, lambda_fine)
        dev = q_tokens.device
        out = {"seg_idx": torch.empty(B, k_seg, dtype=torch.int32, device=dev),
               "seg_score": torch.empty(B, k_seg, dtype=torch.float32, device=dev),
               "fine_idx": torch.empty(B, k_fine, dtype=torch.int32, device=dev),
               "fine_score": torch.empty(B, k_fine, dtype=torch.float32, device=dev)}
        mukv_retrieve_at(self.h, _ptr(q_tokens), _ptr(q_offsets), _ptr(n_visible), B, prm, 1 if level == "patch" else 0,
                         _ptr(out["seg_idx"]), _ptr(out["seg_score"]), _ptr(out["fine_idx"]), _ptr(out["fine_score"]),
                         _stream())
        self._held.clear()
        return out

    def gather_patches(self, patch_idx, order=MUKV_TEMPORAL, out=None):
        """patch_idx: int32 [B][k_patch] on the device.  Returns (k_out, v_out, n_tokens) with
        k_out, v_out [B][L][Hkv][k_patch*patch_cap][D]."""
        assert patch_idx.dtype == torch.int32 and patch_idx.is_contiguous() and patch_idx.dim() == 2
        B, kp = patch_idx.shape
        c = self.cfg
        if out is None:
            shape = (B, c.n_layers, c.n_kv_heads, kp * self.patch_cap, c.head_dim)
            out = (torch.empty(shape, dtype=self.dtype, device=patch_idx.device),
                   torch.empty(shape, dtype=self.dtype, device=patch_idx.device),
                   torch.empty(B, dtype=torch.int32, device=patch_idx.device))
        mukv_gather_patches(self.h, _ptr(patch_idx), B, kp, order, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _stream())
        self._held.clear()
        return out

    def gather_union(self, seg_idx=None, frame_idx=None, patch_idx=None, rows_cap=None, out=None):
        """Kept rows of the chosen segments' frames, the chosen frames and the chosen super-patches,
        each once, in temporal order.  Index tensors int32 [B][k] on the device (or None).  Returns
        (k_out, v_out, n_tokens) with k_out, v_out [B][L][Hkv][rows_cap][D]."""
        lists = [t for t in (seg_idx, frame_idx, patch_idx) if t is not None]
        assert lists and all(t.dtype == torch.int32 and t.is_contiguous() and t.dim() == 2 for t in lists)
        B = lists[0].shape[0]
        c = self.cfg
        ks = 0 if seg_idx is None else seg_idx.shape[1]
        kf = 0 if frame_idx is None else frame_idx.shape[1]
        kp = 0 if patch_idx is None else patch_idx.shape[1]
        if rows_cap is None:  # room for everything that could be chosen
            rows_cap = (ks * c.frames_per_segment + kf) * self.kappa + kp * self.patch_cap
        if out is None:
            shape = (B, c.n_layers, c.n_kv_heads, rows_cap, c.head_dim)
            dev = lists[0].device
            out = (torch.empty(shape, dtype=self.dtype, device=dev), torch.empty(shape, dtype=self.dtype, device=dev),
                   torch.empty(B, dtype=torch.int32, device=dev))
        mukv_gather_union(self.h, _ptr(seg_idx), ks, _ptr(frame_idx), kf, _ptr(patch_idx), kp, B, rows_cap,
                          _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _stream())
        self._held.clear()
        return out

    def attend(self, layer, q, frame_idx=None, k_local=None, v_local=None, local_offsets=None, causal_local=True,
               out=None):
        """q [B][n_q][Hq][D]; frame_idx [B][k] int32 or None; local rows [n][Hkv][D] with offsets [B+1]."""
        B, n_q = q.shape[0], q.shape[1]
        k_frame = 0 if frame_idx is None else frame_idx.shape[1]
        if out is None:
            out = torch.empty_like(q)
        mukv_attend(self.h, layer, _ptr(q), n_q, _ptr(frame_idx), k_frame, _ptr(k_local), _ptr(v_local),
                    _ptr(local_offsets), B, int(causal_local), _ptr(out), _stream())
        self._held.clear()
        return out

    def prefill_attend(self, layer, q, frame_idx, k_local, v_local, local_offsets, causal_local=True, out=None,
                       signal=None, workspace=None):
        """As attend(), for many new tokens (the last n_q local rows of each question); also returns the
        attention each new token receives, float32 [B][n_q].  workspace: a uint8 device tensor to reuse."""
        B, n_q = q.shape[0], q.shape[1]
        k_frame = 0 if frame_idx is None else frame_idx.shape[1]
        need = mukv_prefill_workspace_size(self.h, n_q, k_frame, B)
        if workspace is None or workspace.numel() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if out is None:
            out = torch.empty_like(q)
        if signal is None:
            signal = torch.empty(B, n_q, dtype=torch.float32, device=q.device)
        mukv_prefill_attend(self.h, layer, _ptr(q), n_q, _ptr(frame_idx), k_frame, _ptr(k_local), _ptr(v_local),
                            _ptr(local_offsets), B, int(causal_local), _ptr(out), _ptr(signal), _ptr(workspace),
                            workspace.numel(), _stream())
        self._held.clear()
        return out, signal

    def prefill_attend_static(self, layer, q, frame_idx, k_local, v_local, local_offsets, causal_local, out, signal):
        """prefill_attend() on the library's fixed per-GPU scratch: allocates nothing, so `out` (like q) and
        `signal` (float32 [B][n_q]) are the caller's."""
        B, n_q = q.shape[0], q.shape[1]
        k_frame = 0 if frame_idx is None else frame_idx.shape[1]
        mukv_prefill_attend_static(self.h, layer, _ptr(q), n_q, _ptr(frame_idx), k_frame, _ptr(k_local), _ptr(v_local),
                                   _ptr(local_offsets), B, int(causal_local), _ptr(out), _ptr(signal), _stream())
        self._held.clear()
        return out, signal

    def retrieve_units(self, q_tokens, q_offsets, k, lambda_g=0.0, g_in=None, n_global=0, want_g=False, n_visible=-1):
        """This context's units as the blocks of one of several stores.  g_in None: the k best by the stage-1
        score (want_g: also the global query, float64 [B][C]); g_in given: stage 1, Eq. 8 with it, the k best.
        Returns dict(idx int32 [B][k], score float32 [B][k], g)."""
        B = q_offsets.numel() - 1
        dev = q_tokens.device
        idx = torch.empty(B, k, dtype=torch.int32, device=dev)
        score = torch.empty(B, k, dtype=torch.float32, device=dev)
        g_out = torch.empty(B, self.cfg.n_kv_heads * self.cfg.head_dim, dtype=torch.float64, device=dev) if want_g else None
        mukv_retrieve_units(self.h, _ptr(q_tokens), _ptr(q_offsets), B, k, float(lambda_g), n_visible, _ptr(g_in),
                            n_global, _ptr(g_out), _ptr(idx), _ptr(score), _stream())
        self._held.clear()
        return {"idx": idx, "score": score, "g": g_out}

    def gather_kv(self, frame_idx, order=MUKV_TEMPORAL, out=None):
        """frame_idx: int32 [B][k_frame] on the device.  Returns (k_out, v_out,
        n_tokens) with k_out, v_out [B][L][Hkv][k_frame*kappa][D]."""
        assert frame_idx.dtype == torch.int32 and frame_idx.is_contiguous() and frame_idx.dim() == 2
        B, kf = frame_idx.shape
        c = self.cfg
        if out is None:
            shape = (B, c.n_layers, c.n_kv_heads, kf * self.kappa, c.head_dim)
            out = (torch.empty(shape, dtype=self.dtype, device=frame_idx.device),
                   torch.empty(shape, dtype=self.dtype, device=frame_idx.device),
                   torch.empty(B, dtype=torch.int32, device=frame_idx.device))
        mukv_gather_kv(self.h, _ptr(frame_idx), B, kf, order, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _stream())
        self._held.clear()
        return out

    # -- read-only copies of the context's tables (tests, inspection) ----------------------
    def _copy(self, ptr, shape, dtype):
        t = torch.empty(shape, dtype=dtype, device=self.device)
        if t.numel():
            rc = _hip_rt().hipMemcpyAsync(t.data_ptr(), ptr, t.numel() * t.element_size(), 3, _stream())
            if rc != 0:
                raise RuntimeError(f"hipMemcpyAsync failed ({rc})")
        return t

    def state(self):
        """Copies of the tables for the frames ingested so far (device tensors)."""
        mukv_flush(self.h)
        s = mukv_get_state(self.h)
        c = self.cfg
        n, S, Ckv, kap = s.n_frames, c.superpatches_per_frame, s.c_kv, s.kappa
        out = {
            "n_frames": n, "n_segments": s.n_segments, "kappa": kap,
            "kept_idx": self._copy(s.kept_idx, (n, kap), torch.int32),
            "rep_frame_k": self._copy(s.rep_frame_k, (n, Ckv), torch.float32),
            "rep_frame_v": self._copy(s.rep_frame_v, (n, Ckv), torch.float32),
            "rep_patch_k": self._copy(s.rep_patch_k, (n * S, Ckv), torch.float32),
            "rep_patch_v": self._copy(s.rep_patch_v, (n * S, Ckv), torch.float32),
            "cnt_patch": self._copy(s.cnt_patch, (n * S,), torch.int32),
            "rep_seg_k": self._copy(s.rep_seg_k, (s.n_segments, Ckv), torch.float32),
            "rep_seg_v": self._copy(s.rep_seg_v, (s.n_segments, Ckv), torch.float32),
            "margin": self._copy(s.margin, (n,), torch.float32),
            "refined": self._copy(s.refined, (n,), torch.int32),
        }
        return out

    def store_rows(self, row0, row1):
        """Copy of store rows [row0, row1) of every (layer, head): (K, V), each
        [L][Hkv][row1-row0][D]."""
        mukv_flush(self.h)
        s = mukv_get_state(self.h)
        c = self.cfg
        esz = 2 if self.dtype == torch.bfloat16 else 4
        row_b = c.head_dim * esz
        n = row1 - row0
        k = torch.empty(c.n_layers, c.n_kv_heads, n, c.head_dim, dtype=self.dtype, device=self.device)
        v = torch.empty_like(k)
        for dst, base in ((k, s.store_k), (v, s.store_v)):
            for l in range(c.n_layers):
                for g in range(c.n_kv_heads):
                    off = ((l * c.n_kv_heads + g) * s.store_token_capacity + row0) * row_b
                    rc = _hip_rt().hipMemcpyAsync(dst[l, g].data_ptr(), base + off, n * row_b, 3, _stream())
                    if rc != 0:
                        raise RuntimeError(f"hipMemcpyAsync failed ({rc})")
        return k, v
