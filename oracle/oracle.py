"""MuKV CPU oracle (Python side) -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Composes the plain fp64 loops of ``mukv_oracle.c`` into the two halves of the
method in the order the paper gives them:

* offline, per chunk of frames (Sec. 3.3): attention indicator (Eq. 1),
  frequency indicator (Eq. 2-3), min-max fusion (Eq. 4), per-frame keep of the
  kappa best tokens, storage of the kept K/V rows of every layer, and the
  block keys of Eq. 5 at super-patch, frame and segment level;
* online, per question (Sec. 3.4): Eq. 6 question pooling, Eq. 7 cosine
  scoring, stage-1 candidates, the global query and Eq. 8 rerank, final
  selection, and the concatenation of the selected blocks' KV (Sec. 3.5);
* the attention of new tokens over that context (Sec. 3.5, Eq. 9), one layer
  at a time.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It imports nothing from the HIP package.
bfloat16 data is carried as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mukv_oracle.c")
_LIB = os.path.join(_HERE, "libmukv_oracle.so")

BF16, F32 = 0, 1
SEMI, HIER, PARALLEL = 0, 1, 2
TEMPORAL, AS_GIVEN = 0, 1


_LIB_SAN = os.path.join(_HERE, "libmukv_oracle_san.so")
_DRIVER = os.path.join(_HERE, "sanitize_driver.c")
# MUKV_ORACLE_SANITIZE=1 in the environment makes every test that uses the oracle run its C half from a
# build instrumented with UndefinedBehaviorSanitizer (any report aborts the process)
_SANITIZE = os.environ.get("MUKV_ORACLE_SANITIZE", "0") not in ("", "0")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the C half with gcc (-O2, OpenMP on the outer loops only).  sanitize: a second library
    built -O1 -g with -fsanitize=undefined,bounds,float-divide-by-zero and no recovery, for CPU test
    runs (host code only; AddressSanitizer needs its runtime first in the process and so runs from an
    executable of its own: sanitizer_selftest)."""
    out = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=undefined,bounds,float-divide-by-zero", "-fno-sanitize-recover=all"]
                 if sanitize else ["-O2"])
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", out, _SRC, "-lm"])
    return out


def sanitizer_selftest() -> str:
    """Builds sanitize_driver.c + mukv_oracle.c with AddressSanitizer and UndefinedBehaviorSanitizer
    (runtime linked statically into the executable) and runs it: every function of the C half on heap
    blocks of exactly the documented sizes.  Returns the driver's output; raises if it reports anything."""
    exe = os.path.join(_HERE, "sanitize_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-Wall", "-o", exe, _DRIVER, _SRC, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    if r.returncode != 0:
        raise RuntimeError(f"sanitizer run failed ({r.returncode}):\n{r.stdout}\n{r.stderr}")
    return r.stdout


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(sanitize=_SANITIZE))
        _lib.orc_cos.restype = ctypes.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"oracle takes uint16 (bf16 bits) or float32, got {a.dtype}")


def _c(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a)


def values_f64(a: np.ndarray) -> np.ndarray:
    """Payload (bf16 bit patterns or float32) as float64 values."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def kappa_of(keep_ratio: float, unit: int) -> int:
    """kappa = floor(rho * |unit|) (Sec. 3.3); 1e-9 guards ratios such as 0.29*100."""
    return int(math.floor(keep_ratio * unit + 1e-9))


def superpatch_bounds(P: int, S: int):
    """Index-contiguous super-patches of length floor(P/S) (Sec. 3.2); the last
    one takes the remainder so the S groups partition the frame."""
    n = P // S
    return [(s * n, (s + 1) * n if s < S - 1 else P) for s in range(S)]


# ----------------------------------------------------------------------------
# thin typed wrappers over the C loops
# ----------------------------------------------------------------------------
def att_signal(q, k, n_frames, P, causal=True):
    q, k = _c(q), _c(k)
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    assert T == n_frames * P and k.shape == (Hkv, T, D)
    out = np.empty((n_frames, P), np.float64)
    rc = lib().orc_att_signal(_p(q), _p(k), _dtype_code(k), n_frames, Hq, Hkv, P, D, int(causal), _p(out))
    assert rc == 0
    return out


FEATURE_AXIS, TOKEN_AXIS = 0, 1


def fft_signal(k, n_frames, P, axis=FEATURE_AXIS):
    """Eq. 2-3.  axis: the transform runs along each token's features (the reading
    taken by default) or along the frame's tokens, feature by feature."""
    k = _c(k)
    Hkv, T, D = k.shape
    assert T == n_frames * P
    out = np.empty((n_frames, P), np.float64)
    fn = lib().orc_fft_signal if axis == FEATURE_AXIS else lib().orc_fft_signal_token
    rc = fn(_p(k), _dtype_code(k), n_frames, Hkv, P, D, _p(out))
    assert rc == 0
    return out


def fuse(att, fft, alpha):
    ref = att if att is not None else fft
    n_frames, P = ref.shape
    out = np.empty((n_frames, P), np.float64)
    a = None if att is None else _c(att.astype(np.float64))
    b = None if fft is None else _c(fft.astype(np.float64))
    rc = lib().orc_fuse(_p(a), _p(b), n_frames, P, ctypes.c_double(alpha), _p(out))
    assert rc == 0
    return out


def topk(scores, k, mask=None):
    s = _c(np.asarray(scores, np.float64))
    m = None if mask is None else _c(np.asarray(mask, np.uint8))
    idx = np.empty(max(k, 1), np.int32)
    found = lib().orc_topk(_p(s), _p(m), s.shape[0], k, _p(idx))
    return idx[:k], found


def keep(fused, kappa):
    fused = _c(np.asarray(fused, np.float64))
    n_frames, P = fused.shape
    kept = np.empty((n_frames, kappa), np.int32)
    rc = lib().orc_keep(_p(fused), n_frames, P, kappa, _p(kept))
    assert rc == 0
    return kept


def compact(src, n_frames, P, kept):
    src = _c(src)
    L, Hkv, T, D = src.shape
    assert T == n_frames * P
    kappa = kept.shape[1]
    kept = _c(kept.astype(np.int32))
    dst = np.empty((L, Hkv, n_frames * kappa, D), src.dtype)
    rc = lib().orc_compact(_p(src), src.dtype.itemsize, L, Hkv, n_frames, P, D, _p(kept), kappa, _p(dst))
    assert rc == 0
    return dst


def pool_rows(x, rows):
    x = _c(x)
    Hkv, T, D = x.shape
    rows = _c(np.asarray(rows, np.int64))
    out = np.empty(Hkv * D, np.float64)
    rc = lib().orc_pool_rows(_p(x), _dtype_code(x), Hkv, ctypes.c_int64(T), D, _p(rows), rows.shape[0], _p(out))
    assert rc == 0
    return out


def pool_question(q_tokens):
    q_tokens = _c(q_tokens)
    Nq, Hq, D = q_tokens.shape
    out = np.empty(Hq * D, np.float64)
    rc = lib().orc_pool_question(_p(q_tokens), _dtype_code(q_tokens), Nq, Hq, D, _p(out))
    assert rc == 0
    return out


def score_blocks(q, reps32, Hq, Hkv, D):
    q = _c(np.asarray(q, np.float64))
    reps32 = _c(np.asarray(reps32, np.float32))
    N = reps32.shape[0]
    out = np.empty(N, np.float64)
    if N:
        rc = lib().orc_score_blocks(_p(q), _p(reps32), N, Hq, Hkv, D, _p(out))
        assert rc == 0
    return out


def consistency(g_vec, reps32, cand):
    g_vec = _c(np.asarray(g_vec, np.float64))
    reps32 = _c(np.asarray(reps32, np.float32))
    cand = _c(np.asarray(cand, np.int32))
    out = np.empty(cand.shape[0], np.float64)
    if cand.shape[0]:
        rc = lib().orc_consistency(_p(g_vec), _p(reps32), ctypes.c_int64(reps32.shape[1]), _p(cand), cand.shape[0], _p(out))
        assert rc == 0
    return out


# ----------------------------------------------------------------------------
# the method, step by step
# ----------------------------------------------------------------------------
@dataclass
class OracleConfig:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    tokens_per_frame: int
    frames_per_segment: int
    superpatches_per_frame: int = 4
    keep_ratio: float = 0.25
    alpha: float = 0.7
    causal: bool = True
    score_layer: int = -1
    freq_axis: int = FEATURE_AXIS


@dataclass
class RetrieveParams:
    mode: int = SEMI
    k_seg: int = 8
    k_frame: int = 32
    lambda_frame: float = 0.3
    n_global: int = 0          # 0 -> k_seg
    n_visible_frames: int = -1  # -1 -> every ingested frame


class OracleMuKV:
    """Streaming state of the method on the host: the compact store, the kept
    positions (timestamps are the frame numbers) and the Eq. 5 block keys."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.kappa = kappa_of(cfg.keep_ratio, cfg.tokens_per_frame)
        assert 1 <= self.kappa <= cfg.tokens_per_frame
        self.ls = cfg.score_layer if cfg.score_layer >= 0 else cfg.n_layers - 1
        self.n_frames = 0
        self._store_k, self._store_v = [], []
        self.kept = np.empty((0, self.kappa), np.int32)
        C = cfg.n_kv_heads * cfg.head_dim
        self.rep_frame_k = np.empty((0, C), np.float64)
        self.rep_frame_v = np.empty((0, C), np.float64)
        self.rep_patch_k = np.empty((0, C), np.float64)
        self.rep_patch_v = np.empty((0, C), np.float64)
        self.cnt_patch = np.empty((0,), np.int32)

    # -- offline ------------------------------------------------------------
    def compress_chunk(self, k, v, q_last=None, att=None):
        """k, v: [L][Hkv][n*P][D]; q_last: [Hq][n*P][D] of the scoring layer, or
        att: [n][P] attention received, handed over by the caller's prefill."""
        c = self.cfg
        P, S = c.tokens_per_frame, c.superpatches_per_frame
        n = k.shape[2] // P
        assert k.shape == v.shape == (c.n_layers, c.n_kv_heads, n * P, c.head_dim)
        k_s, v_s = k[self.ls], v[self.ls]
        a = None
        if c.alpha != 0.0:
            a = att if att is not None else att_signal(q_last, k_s, n, P, c.causal)
        fq = fft_signal(k_s, n, P, c.freq_axis) if c.alpha != 1.0 else None
        fused = fuse(a, fq, c.alpha)
        kept = keep(fused, self.kappa)
        self._store_k.append(compact(k, n, P, kept))
        self._store_v.append(compact(v, n, P, kept))
        C = c.n_kv_heads * c.head_dim
        rfk, rfv = np.empty((n, C)), np.empty((n, C))
        rpk, rpv = np.empty((n * S, C)), np.empty((n * S, C))
        cnt = np.empty(n * S, np.int32)
        bounds = superpatch_bounds(P, S)
        for f in range(n):
            rows = f * P + kept[f].astype(np.int64)
            rfk[f], rfv[f] = pool_rows(k_s, rows), pool_rows(v_s, rows)
            for s, (lo, hi) in enumerate(bounds):
                sel = rows[(kept[f] >= lo) & (kept[f] < hi)]
                rpk[f * S + s], rpv[f * S + s] = pool_rows(k_s, sel), pool_rows(v_s, sel)
                cnt[f * S + s] = sel.shape[0]
        self.kept = np.concatenate([self.kept, kept])
        self.rep_frame_k = np.concatenate([self.rep_frame_k, rfk])
        self.rep_frame_v = np.concatenate([self.rep_frame_v, rfv])
        self.rep_patch_k = np.concatenate([self.rep_patch_k, rpk])
        self.rep_patch_v = np.concatenate([self.rep_patch_v, rpv])
        self.cnt_patch = np.concatenate([self.cnt_patch, cnt])
        self.n_frames += n
        return {"att": a, "fft": fq, "fused": fused, "kept": kept}

    def store(self):
        """Compact store so far: (K, V), each [L][Hkv][n_frames*kappa][D]."""
        if len(self._store_k) > 1:
            self._store_k = [np.concatenate(self._store_k, axis=2)]
            self._store_v = [np.concatenate(self._store_v, axis=2)]
        return self._store_k[0], self._store_v[0]

    def n_segments(self, n_visible=None):
        nv = self.n_frames if n_visible is None else n_visible
        F = self.cfg.frames_per_segment
        return (nv + F - 1) // F

    def seg_reps(self, n_visible=None, which="k"):
        """Eq. 5 at segment level: mean over the kept tokens of the segment's
        visible frames, scoring layer.  [n_segments][Hkv*D] float64."""
        nv = self.n_frames if n_visible is None else n_visible
        F, kap = self.cfg.frames_per_segment, self.kappa
        sk, sv = self.store()
        x = (sk if which == "k" else sv)[self.ls]
        out = np.empty((self.n_segments(nv), x.shape[0] * x.shape[2]), np.float64)
        for s in range(out.shape[0]):
            f0, f1 = s * F, min((s + 1) * F, nv)
            out[s] = pool_rows(x, np.arange(f0 * kap, f1 * kap, dtype=np.int64))
        return out

    # -- online -------------------------------------------------------------
    def retrieve(self, q_tokens, prm: RetrieveParams, level="frame"):
        """q_tokens: [Nq][Hq][D] scoring-layer query states of one question.

        level="frame": Sec. 3.4 with frames as the fine level.  level="patch": the
        same with the super-patches as the fine level (block f*S + s; k_frame and
        lambda_frame are then k_g and lambda_g of the patch level; super-patches
        without a kept token cannot be chosen; the results come back under the
        "frame_*" names)."""
        c = self.cfg
        Hq, Hkv, D = c.n_q_heads, c.n_kv_heads, c.head_dim
        nv = self.n_frames if prm.n_visible_frames < 0 else min(prm.n_visible_frames, self.n_frames)
        F = c.frames_per_segment
        if level == "patch":
            return self._retrieve_fine(q_tokens, prm, nv, self.rep_patch_k[:nv * c.superpatches_per_frame].astype(np.float32),
                                       F * c.superpatches_per_frame,
                                       (self.cnt_patch[:nv * c.superpatches_per_frame] > 0).astype(np.uint8))
        return self._retrieve_fine(q_tokens, prm, nv, self.rep_frame_k[:nv].astype(np.float32), F, None)

    def _retrieve_fine(self, q_tokens, prm, nv, frm32, F, allowed):
        """Sec. 3.4 over the segment keys and one table of finer block keys: frm32
        [n_fine][C] float32, F fine blocks per segment, allowed = optional 0/1 mask
        of the fine blocks that may be chosen."""
        c = self.cfg
        Hq, Hkv, D = c.n_q_heads, c.n_kv_heads, c.head_dim
        nf = frm32.shape[0]
        base = np.ones(nf, np.uint8) if allowed is None else allowed
        seg32 = self.seg_reps(nv).astype(np.float32) if nv > 0 else np.empty((0, Hkv * D), np.float32)
        q = pool_question(q_tokens)                               # Eq. 6
        s_seg = score_blocks(q, seg32, Hq, Hkv, D)                # Eq. 7
        s_frm = score_blocks(q, frm32, Hq, Hkv, D)
        ks, kf = prm.k_seg, prm.k_frame
        res = {"s_seg": s_seg, "s_frm": s_frm}
        if prm.mode == PARALLEL:
            seg_idx, ns = topk(s_seg, ks)
            frm_idx, nfound = topk(s_frm, kf, base)
            frm_score = s_frm
        elif prm.mode == HIER:
            seg_idx, ns = topk(s_seg, ks)
            mask = np.zeros(nf, np.uint8)
            for s in seg_idx[:ns]:
                mask[s * F:min((s + 1) * F, nf)] = 1
            frm_idx, nfound = topk(s_frm, kf, mask & base)
            frm_score = s_frm
        else:
            cand_seg, ncs = topk(s_seg, 2 * ks)                   # stage 1
            cand_frm, ncf = topk(s_frm, 2 * kf, base)
            n_glob = min(prm.n_global if prm.n_global > 0 else ks, ncs)
            g_vec = seg32[cand_seg[:n_glob]].astype(np.float64).mean(axis=0) if n_glob else np.zeros(Hkv * D)
            gamma = consistency(g_vec, frm32, cand_frm[:ncf])     # stage 2
            s_tilde = np.full(nf, -np.inf)
            s_tilde[cand_frm[:ncf]] = (1.0 - prm.lambda_frame) * s_frm[cand_frm[:ncf]] + prm.lambda_frame * gamma  # Eq. 8
            mask = np.zeros(nf, np.uint8)
            mask[cand_frm[:ncf]] = 1
            frm_idx, nfound = topk(s_tilde, kf, mask)
            seg_idx, ns = cand_seg[:ks].copy(), min(ks, ncs)      # lambda = 0 for segments
            frm_score = s_tilde
            res.update({"cand_seg": cand_seg, "cand_frm": cand_frm, "g": g_vec, "gamma": gamma})
        seg_score = np.zeros(ks)
        seg_score[:ns] = s_seg[seg_idx[:ns]]
        frame_score = np.zeros(kf)
        frame_score[:nfound] = frm_score[frm_idx[:nfound]]
        res.update({"seg_idx": seg_idx, "seg_score": seg_score, "frame_idx": frm_idx, "frame_score": frame_score})
        return res

    def gather_union(self, seg_idx=(), frame_idx=(), patch_idx=(), rows_cap=None):
        """Combined gather over the three granularities (Sec. 3.4): the kept rows
        of every frame of the chosen segments, of the chosen frames and of the
        chosen super-patches, each row once, ascending (frame, position).
        Returns (K, V, n_rows); K, V [L][Hkv][rows_cap][D], tail zero; when the
        union holds more than rows_cap rows only the first rows_cap are copied."""
        sk, sv = self.store()
        c = self.cfg
        kap, S, P, F = self.kappa, c.superpatches_per_frame, c.tokens_per_frame, c.frames_per_segment
        rows = set()
        for s in seg_idx:
            if s >= 0:
                for f in range(int(s) * F, min((int(s) + 1) * F, self.n_frames)):
                    rows.update(range(f * kap, (f + 1) * kap))
        for f in frame_idx:
            if 0 <= f < self.n_frames:
                rows.update(range(int(f) * kap, (int(f) + 1) * kap))
        bounds = superpatch_bounds(P, S)
        for pid in patch_idx:
            if 0 <= pid < self.n_frames * S:
                f, sp = divmod(int(pid), S)
                lo, hi = bounds[sp]
                rows.update(f * kap + r for r in range(kap) if lo <= self.kept[f, r] < hi)
        rows = sorted(rows)
        if rows_cap is None:
            rows_cap = max(len(rows), 1)
        L, Hkv, _, D = sk.shape
        ko = np.zeros((L, Hkv, rows_cap, D), sk.dtype)
        vo = np.zeros_like(ko)
        n = min(len(rows), rows_cap)
        ko[:, :, :n] = sk[:, :, rows[:n]]
        vo[:, :, :n] = sv[:, :, rows[:n]]
        return ko, vo, len(rows)

    def gather_patches(self, patch_idx, order=TEMPORAL):
        """Concatenate the stored K,V of the selected super-patches: for patch
        f*S + s the kept rows of frame f whose position lies in super-patch s.
        Returns (K, V, n_tokens), K and V [L][Hkv][len(patch_idx)*patch_cap][D]
        with the unused tail zero.  Entries equal to -1 are skipped."""
        sk, sv = self.store()
        kap, S, P = self.kappa, self.cfg.superpatches_per_frame, self.cfg.tokens_per_frame
        cap = min(kap, P - (S - 1) * (P // S))
        sel = [int(x) for x in patch_idx if 0 <= x < self.n_frames * S]
        if order == TEMPORAL:
            sel = sorted(sel)
        L, Hkv, _, D = sk.shape
        ko = np.zeros((L, Hkv, len(patch_idx) * cap, D), sk.dtype)
        vo = np.zeros_like(ko)
        n = 0
        for pid in sel:
            f, sp = divmod(pid, S)
            lo, hi = superpatch_bounds(P, S)[sp]
            rows = [f * kap + r for r in range(kap) if lo <= self.kept[f, r] < hi]
            ko[:, :, n:n + len(rows)] = sk[:, :, rows]
            vo[:, :, n:n + len(rows)] = sv[:, :, rows]
            n += len(rows)
        return ko, vo, n

    def attend(self, layer, q, frame_idx, k_local=None, v_local=None, causal_local=True):
        """Attention of new tokens over the retrieved context at one layer
        (Sec. 3.5, Eq. 9): query token i, head h attends to the keys
        [R_k, W_K X] = kept rows of the listed frames (entries that name no
        frame of the cache, such as the -1 padding, are skipped)
        followed by the caller's own ("local") rows, with values [R_v, W_V X];
        scores q.k / sqrt(D), softmax over all visible keys, KV head h // G.
        The query tokens are the last n_q local rows: with causal_local, token
        i sees local row j only if j <= n_l - n_q + i.  Every retrieved row is
        visible.  q [n_q][Hq][D]; k_local, v_local [n_l][Hkv][D] or None.
        Returns float64 [n_q][Hq][D]; all zero for a token that sees no key."""
        return self._attend(layer, q, frame_idx, k_local, v_local, causal_local)[0]

    def prefill_attend(self, layer, q, frame_idx, k_local, v_local, causal_local=True):
        """The prefill of new tokens at one layer (Sec. 3.2: the new tokens attend
        to the past cache and to themselves), which also yields the attention
        each new token RECEIVES (Sec. 3.3, Eq. 1) with no second pass: the same
        attention as attend(); the signal of new token j (local row n_l - n_q + j)
        is the mean over the heads and over the n_q query rows of the softmax
        weight put on it, the softmax being normalised over everything the query
        sees, past rows included.  Returns (out [n_q][Hq][D], signal [n_q])."""
        out, w_local = self._attend(layer, q, frame_idx, k_local, v_local, causal_local)
        n_q = out.shape[0]
        return out, w_local[w_local.shape[0] - n_q:] / (self.cfg.n_q_heads * n_q)

    def _attend(self, layer, q, frame_idx, k_local, v_local, causal_local):
        """Eq. 9 as described in attend(); also returns, per local row, the softmax
        weight it receives summed over heads and query tokens."""
        c = self.cfg
        sk, sv = self.store() if self.n_frames else (None, None)
        kap, G, D = self.kappa, c.n_q_heads // c.n_kv_heads, c.head_dim
        qf = values_f64(np.asarray(q))
        n_q = qf.shape[0]
        n_l = 0 if k_local is None else k_local.shape[0]
        rows = [r for f in frame_idx if 0 <= f < self.n_frames for r in range(int(f) * kap, (int(f) + 1) * kap)]
        out = np.zeros((n_q, c.n_q_heads, D))
        received = np.zeros(n_l)
        for h in range(c.n_q_heads):
            g = h // G
            parts_k, parts_v = [], []
            if rows:
                parts_k.append(values_f64(sk[layer, g][rows]))
                parts_v.append(values_f64(sv[layer, g][rows]))
            if n_l:
                parts_k.append(values_f64(np.asarray(k_local)[:, g]))
                parts_v.append(values_f64(np.asarray(v_local)[:, g]))
            if not parts_k:
                continue
            kk, vv = np.concatenate(parts_k), np.concatenate(parts_v)
            for i in range(n_q):
                s = kk @ qf[i, h] / math.sqrt(D)
                if causal_local and n_l:
                    j = np.arange(n_l)
                    s[len(rows):][j > n_l - n_q + i] = -np.inf
                if not np.isfinite(s).any():
                    continue
                w = np.exp(s - s[np.isfinite(s)].max())
                w = w / w.sum()
                out[i, h] = w @ vv
                received += w[len(rows):]
        return out, received

    def gather(self, frame_idx, order=TEMPORAL):
        """Concatenate the stored K,V of the selected frames (Sec. 3.5): returns
        (K, V, n_tokens), K and V [L][Hkv][len(frame_idx)*kappa][D] with the
        unused tail zero.  Entries that name no frame of the cache (the -1 padding,
        numbers >= n_frames) are skipped."""
        sk, sv = self.store()
        kap = self.kappa
        sel = [int(f) for f in frame_idx if 0 <= f < self.n_frames]
        if order == TEMPORAL:
            sel = sorted(sel)
        L, Hkv, _, D = sk.shape
        ko = np.zeros((L, Hkv, len(frame_idx) * kap, D), sk.dtype)
        vo = np.zeros_like(ko)
        for slot, f in enumerate(sel):
            ko[:, :, slot * kap:(slot + 1) * kap] = sk[:, :, f * kap:(f + 1) * kap]
            vo[:, :, slot * kap:(slot + 1) * kap] = sv[:, :, f * kap:(f + 1) * kap]
        return ko, vo, len(sel) * kap


# ----------------------------------------------------------------------------
# three independently compressed stores searched together (Sec. 3.3 last two
# paragraphs, Sec. 3.4 stage 2, Sec. 4.1 hyper-parameters)
# ----------------------------------------------------------------------------
def retrieve_units(store: OracleMuKV, q_tokens, k, lam=0.0, g_in=None, n_global=0, n_visible=-1):
    """Sec. 3.4 over the blocks of ONE store, a block being a unit of that store's
    compression (its Eq. 5 key = mean of the unit's kept scoring-layer keys, held
    as float32): Eq. 6-7 scores s of the visible units against the question.
      g_in is None (the coarsest store, lambda_g = 0): the top-k units by s; also
        returns the global query g = mean of the keys of the first n_global
        (0 -> k) of them, which stage 2 applies to the finer stores.
      g_in given: stage 1 keeps the top-2k units by s, stage 2 gives each candidate
        gamma = cos(its key, g_in) and s~ = (1 - lam) s + lam gamma (Eq. 8), and the
        top-k by s~ are returned (equal s~: the lower unit number).
    Returns dict(idx [k] int32 padded with -1, score [k], s, g)."""
    c = store.cfg
    n_all = store.n_frames
    nv = n_all if n_visible < 0 else min(n_visible, n_all)
    keys32 = store.rep_frame_k[:nv].astype(np.float32)
    q = pool_question(q_tokens)                                    # Eq. 6
    s = score_blocks(q, keys32, c.n_q_heads, c.n_kv_heads, c.head_dim)  # Eq. 7
    score = np.zeros(k)
    if g_in is None:
        idx, n = topk(s, k)
        n_glob = min(n_global if n_global > 0 else k, n)
        g = keys32[idx[:n_glob]].astype(np.float64).mean(axis=0) if n_glob else np.zeros(keys32.shape[1])
        score[:n] = s[idx[:n]]
        return {"idx": idx, "score": score, "s": s, "g": g}
    cand, nc = topk(s, 2 * k)                                      # stage 1
    gamma = consistency(np.asarray(g_in, np.float64), keys32, cand[:nc])  # stage 2
    s_tilde = np.full(nv, -np.inf)
    s_tilde[cand[:nc]] = (1.0 - lam) * s[cand[:nc]] + lam * gamma  # Eq. 8
    mask = np.zeros(nv, np.uint8)
    mask[cand[:nc]] = 1
    idx, n = topk(s_tilde, k, mask)
    score[:n] = s_tilde[idx[:n]]
    return {"idx": idx, "score": score, "s": s, "g": np.asarray(g_in, np.float64), "cand": cand, "gamma": gamma}


def retrieve_multi(stores, q_tokens, ks, lams, n_global=0):
    """The question against several stores, coarsest first: stores[0] (segment units)
    is ranked by its stage-1 scores and supplies the global query; every other store
    is reranked with it (Eq. 8 with its own lambda_g) -- the paper's patch / frame /
    segment stores with k_g = 20 / 32 / 12 and lambda_g = 0.3 / 0.3 / 0 are
    stores = [segment, frame, patch], ks = [12, 32, 20], lams = [0, 0.3, 0.3].
    Returns the list of retrieve_units results."""
    out = [retrieve_units(stores[0], q_tokens, ks[0], n_global=n_global)]
    for st, k, lam in zip(stores[1:], ks[1:], lams[1:]):
        out.append(retrieve_units(st, q_tokens, k, lam, g_in=out[0]["g"]))
    return out


def gather_multi(stores, idx_lists, units_per_step, rows_cap=None):
    """The decode context of Sec. 3.5 from several stores: the kept rows of the chosen
    units of every store, in temporal order -- ascending time step (unit u of store i
    belongs to step u // units_per_step[i]), within a step the stores in the order
    given (coarse to fine) and a store's units ascending; a unit listed twice is
    copied once, entries that name no unit are skipped.  All stores share L, Hkv, D.
    Returns (K, V, n_rows), K and V [L][Hkv][rows_cap][D] with the unused tail zero;
    when the context holds more than rows_cap rows only the first rows_cap are copied."""
    entries = set()
    for i, (st, idx) in enumerate(zip(stores, idx_lists)):
        for u in idx:
            if 0 <= u < st.n_frames:
                entries.add((int(u) // units_per_step[i], i, int(u)))
    ks, vs = [], []
    for _, i, u in sorted(entries):
        sk, sv = stores[i].store()
        kap = stores[i].kappa
        ks.append(sk[:, :, u * kap:(u + 1) * kap])
        vs.append(sv[:, :, u * kap:(u + 1) * kap])
    sk0, _ = stores[0].store()
    L, Hkv, _, D = sk0.shape
    n_rows = sum(x.shape[2] for x in ks)
    if rows_cap is None:
        rows_cap = max(n_rows, 1)
    ko = np.zeros((L, Hkv, rows_cap, D), sk0.dtype)
    vo = np.zeros_like(ko)
    if ks:
        kc, vc = np.concatenate(ks, axis=2), np.concatenate(vs, axis=2)
        n = min(n_rows, rows_cap)
        ko[:, :, :n], vo[:, :, :n] = kc[:, :, :n], vc[:, :, :n]
    return ko, vo, n_rows

