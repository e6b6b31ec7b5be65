"""Shared helpers of the GPU parity tests: run the same seeded stream through the
HIP library (via the C ABI binding) and through the CPU oracle, and compare."""
from __future__ import annotations

import numpy as np
import torch

from oracle import oracle as orc
from paper_2605_22269_amd import binding as mk
from paper_2605_22269_amd import synth

# max-abs-error bars of the build's target: bf16 payloads 2e-2, fp32 payloads 1e-5
TOL = {"bf16": 2e-2, "f32": 1e-5}


def oracle_config(w: synth.Workload, **kw) -> orc.OracleConfig:
    base = dict(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                tokens_per_frame=w.tokens_per_frame, frames_per_segment=w.frames_per_segment,
                superpatches_per_frame=w.superpatches_per_frame, keep_ratio=w.keep_ratio, alpha=w.alpha,
                causal=True, score_layer=-1)
    base.update(kw)
    return orc.OracleConfig(**base)


def gpu_context(w: synth.Workload, max_frames=None, max_chunk_frames=None, max_questions=None, **kw) -> mk.MuKV:
    base = dict(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                tokens_per_frame=w.tokens_per_frame, frames_per_segment=w.frames_per_segment,
                superpatches_per_frame=w.superpatches_per_frame, dtype=w.torch_dtype, keep_ratio=w.keep_ratio,
                alpha=w.alpha, causal=True, max_frames=max_frames or w.n_frames,
                max_chunk_frames=max_chunk_frames or w.chunk_frames, max_questions=max_questions or w.n_questions)
    base.update(kw)
    return mk.MuKV(**base)


def np_view(t):
    return synth.as_numpy(t)


def out_err(got, want):
    """Largest error of an attention output, each element measured against max(1, |its expected value|): the
    output is rounded to the payload type, and a bf16 value of magnitude x sits up to x / 512 from what was
    rounded, so a plain 2e-2 is out of reach from |x| = 4 on whatever the arithmetic does.  Below 1 the bar
    is the plain one."""
    return float((np.abs(got - want) / np.maximum(1.0, np.abs(want))).max())


def to_f64(a):
    """numpy payload (uint16 bf16 bits or float32) -> float64 values"""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


class Pair:
    """One stream through both implementations."""

    def __init__(self, w: synth.Workload, seed=0, chunk=None, with_q=True, gpu_kw=None, orc_kw=None, frames=None):
        self.w = w
        self.chunk = chunk or w.chunk_frames
        self.n = frames or w.n_frames
        self.gpu = gpu_context(w, max_frames=self.n, max_chunk_frames=self.chunk, **(gpu_kw or {}))
        margin = (gpu_kw or {}).get("refine_margin", -1.0)
        self.refine_margin = 1e-5 if margin < 0 else margin   # the library's default threshold
        self.orc = orc.OracleMuKV(oracle_config(w, **(orc_kw or {})))
        self.stream = synth.SynthStream(w, seed, device="cpu", with_q=with_q)
        self.sig_gpu, self.sig_orc = [], []
        self.keep_alive = []  # device inputs must outlive a gathered batch

    def ingest(self, n_frames=None, att_from_oracle=False, att_seed=None):
        """Feeds the next n_frames (default: all remaining) in chunks to both sides.  The attention
        signal is computed by each side from the queries, or handed to both: the oracle's own
        (att_from_oracle) or a seeded stand-in (att_seed)."""
        todo = self.n - self.orc.n_frames if n_frames is None else n_frames
        while todo > 0:
            n = min(self.chunk, todo)
            k, v, q = self.stream.next_chunk(n)
            kn, vn, qn = np_view(k), np_view(v), (np_view(q) if q is not None else None)
            att_np = att_t = None
            if att_from_oracle or att_seed is not None:
                if att_seed is not None:
                    att_np = synth.handed_over_attention(n, self.w.tokens_per_frame, att_seed + self.orc.n_frames).numpy()
                else:
                    att_np = orc.att_signal(qn, kn[self.orc.ls], n, self.w.tokens_per_frame, self.orc.cfg.causal)
                    att_np = att_np.astype(np.float32)
                att_t = torch.from_numpy(att_np).cuda()
                kd, vd = k.cuda(), v.cuda()
                self.keep_alive += [kd, vd, att_t]
                self.sig_orc.append(self.orc.compress_chunk(kn, vn, att=att_np.astype(np.float64)))
                self.sig_gpu.append(self.gpu.compress_chunk(kd, vd, att_signal=att_t, want_signals=True))
            else:
                kd, vd, qd = k.cuda(), v.cuda(), (q.cuda() if q is not None else None)
                self.keep_alive += [kd, vd, qd]
                self.sig_orc.append(self.orc.compress_chunk(kn, vn, q_last=qn))
                self.sig_gpu.append(self.gpu.compress_chunk(kd, vd, qd, want_signals=True))
            torch.cuda.synchronize()
            todo -= n

    # ---- comparisons -----------------------------------------------------------------
    def check_compress(self, exact_reps=True, raw_signals=True):
        w, tol = self.w, TOL[self.w.dtype]
        alpha = self.orc.cfg.alpha
        self.gpu.flush()
        torch.cuda.synchronize()
        for so, sg in zip(self.sig_orc, self.sig_gpu):
            if alpha != 0.0 and raw_signals:
                assert np.abs(sg["att"].cpu().numpy() - so["att"]).max() <= tol
            if alpha != 1.0 and raw_signals:  # the raw Eq. 3 signal scales with the keys: absolute bar only for O(1) inputs
                assert np.abs(sg["fft"].cpu().numpy() - so["fft"]).max() <= tol
            assert np.abs(sg["fused"].cpu().numpy() - so["fused"]).max() <= tol
        st = self.gpu.state()
        torch.cuda.synchronize()
        assert st["n_frames"] == self.orc.n_frames
        np.testing.assert_array_equal(st["kept_idx"].cpu().numpy(), self.orc.kept)       # bit-exact indices
        n, kap = self.orc.n_frames, self.orc.kappa
        # the selection in isolation: the oracle's keep applied to the GPU's OWN fused scores gives the GPU's
        # indices for every frame decided in fp32; a frame decided by the fp64 pass had its boundary gap
        # below the threshold (which is why it was re-scored)
        refined = st["refined"].cpu().numpy().astype(bool)
        gpu_kept = st["kept_idx"].cpu().numpy()
        f0 = 0
        for sg in self.sig_gpu:
            fused = sg["fused"].cpu().numpy().astype(np.float64)
            own = orc.keep(fused, kap)
            for i in range(fused.shape[0]):
                if not refined[f0 + i]:
                    np.testing.assert_array_equal(own[i], gpu_kept[f0 + i], err_msg=f"frame {f0 + i}")
                elif kap < fused.shape[1] <= 256 and self.refine_margin < 1.0:   # (units above 256 tokens all go to the fp64 pass)
                    srt = np.sort(fused[i])[::-1]
                    assert srt[kap - 1] - srt[kap] <= self.refine_margin + 1e-6, f"frame {f0 + i}"
            f0 += fused.shape[0]
        gk, gv = self.gpu.store_rows(0, n * kap)
        ok, ov = self.orc.store()
        np.testing.assert_array_equal(np_view(gk), ok)                                    # byte copy
        np.testing.assert_array_equal(np_view(gv), ov)
        F = w.frames_per_segment
        pairs = [("rep_frame_k", self.orc.rep_frame_k), ("rep_frame_v", self.orc.rep_frame_v),
                 ("rep_patch_k", self.orc.rep_patch_k), ("rep_patch_v", self.orc.rep_patch_v),
                 ("rep_seg_k", self.orc.seg_reps(which="k")), ("rep_seg_v", self.orc.seg_reps(which="v"))]
        for name, want in pairs:
            got = st[name].cpu().numpy()
            assert got.shape == want.shape, name
            assert np.abs(got - want).max() <= tol * max(1.0, float(np.abs(want).max())), name
            if exact_reps:  # fp64 sums of the payload are exact, so the float32 tables agree to the bit
                np.testing.assert_array_equal(got, want.astype(np.float32), err_msg=name)
        np.testing.assert_array_equal(st["cnt_patch"].cpu().numpy(), self.orc.cnt_patch)
        assert st["n_segments"] == (n + F - 1) // F
        return st

    def check_retrieve(self, questions, mode, k_seg, k_frame, lambda_frame=0.3, n_visible=-1, n_global=0):
        """questions: list of torch tensors [Nq][Hq][D] (cpu)."""
        tol = TOL[self.w.dtype]
        offs = np.zeros(len(questions) + 1, np.int32)
        offs[1:] = np.cumsum([q.shape[0] for q in questions])
        qt = torch.cat(questions).cuda().contiguous()
        out = self.gpu.retrieve(qt, torch.from_numpy(offs).cuda(), mode=mode, k_seg=k_seg, k_frame=k_frame,
                                lambda_frame=lambda_frame, n_visible_frames=n_visible, n_global=n_global)
        kg, vg, ntok = self.gpu.gather_kv(out["frame_idx"])
        torch.cuda.synchronize()
        res = []
        for b, q in enumerate(questions):
            r = self.orc.retrieve(np_view(q), orc.RetrieveParams(mode, k_seg, k_frame, lambda_frame, n_global, n_visible))
            np.testing.assert_array_equal(out["seg_idx"][b].cpu().numpy(), r["seg_idx"])
            np.testing.assert_array_equal(out["frame_idx"][b].cpu().numpy(), r["frame_idx"])
            assert np.abs(out["seg_score"][b].cpu().numpy() - r["seg_score"]).max() <= min(tol, 1e-5)
            assert np.abs(out["frame_score"][b].cpu().numpy() - r["frame_score"]).max() <= min(tol, 1e-5)
            ko, vo, n_tok = self.orc.gather(r["frame_idx"])
            assert int(ntok[b]) == n_tok
            np.testing.assert_array_equal(np_view(kg[b]), ko)
            np.testing.assert_array_equal(np_view(vg[b]), vo)
            res.append(r)
        return out, res

    def check_retrieve_patches(self, questions, mode, k_seg, k_patch, lambda_patch=0.3, n_visible=-1, n_global=0):
        """The super-patch level: indices and gathered bytes exact, scores within tolerance."""
        tol = TOL[self.w.dtype]
        offs = np.zeros(len(questions) + 1, np.int32)
        offs[1:] = np.cumsum([q.shape[0] for q in questions])
        qt = torch.cat(questions).cuda().contiguous()
        out = self.gpu.retrieve_patches(qt, torch.from_numpy(offs).cuda(), mode=mode, k_seg=k_seg, k_patch=k_patch,
                                        lambda_patch=lambda_patch, n_visible_frames=n_visible, n_global=n_global)
        res = []
        for order, oorder in ((mk.MUKV_TEMPORAL, orc.TEMPORAL), (mk.MUKV_AS_GIVEN, orc.AS_GIVEN)):
            kg, vg, ntok = self.gpu.gather_patches(out["patch_idx"], order)
            torch.cuda.synchronize()
            for b, q in enumerate(questions):
                r = self.orc.retrieve(np_view(q), orc.RetrieveParams(mode, k_seg, k_patch, lambda_patch, n_global, n_visible),
                                      level="patch")
                np.testing.assert_array_equal(out["patch_idx"][b].cpu().numpy(), r["frame_idx"])
                assert np.abs(out["patch_score"][b].cpu().numpy() - r["frame_score"]).max() <= min(tol, 1e-5)
                ko, vo, n_tok = self.orc.gather_patches(r["frame_idx"], oorder)
                assert int(ntok[b]) == n_tok
                np.testing.assert_array_equal(np_view(kg[b]), ko)
                np.testing.assert_array_equal(np_view(vg[b]), vo)
                res.append(r)
        return out, res

    def check_retrieve_at(self, questions, n_visible, level, mode, k_seg, k_fine, lambda_fine=0.3):
        """Questions with their own timestamps in one call against one oracle call per question."""
        tol = TOL[self.w.dtype]
        offs = np.zeros(len(questions) + 1, np.int32)
        offs[1:] = np.cumsum([q.shape[0] for q in questions])
        qt = torch.cat(questions).cuda().contiguous()
        nv = torch.tensor(n_visible, dtype=torch.int32, device="cuda")
        out = self.gpu.retrieve_at(qt, torch.from_numpy(offs).cuda(), nv, level=level, mode=mode, k_seg=k_seg, k_fine=k_fine,
                                   lambda_fine=lambda_fine)
        torch.cuda.synchronize()
        for b, q in enumerate(questions):
            r = self.orc.retrieve(np_view(q), orc.RetrieveParams(mode, k_seg, k_fine, lambda_fine, 0, n_visible[b]), level=level)
            np.testing.assert_array_equal(out["seg_idx"][b].cpu().numpy(), r["seg_idx"], err_msg=f"question {b}")
            np.testing.assert_array_equal(out["fine_idx"][b].cpu().numpy(), r["frame_idx"], err_msg=f"question {b}")
            assert np.abs(out["seg_score"][b].cpu().numpy() - r["seg_score"]).max() <= min(tol, 1e-5)
            assert np.abs(out["fine_score"][b].cpu().numpy() - r["frame_score"]).max() <= min(tol, 1e-5)
        return out

    def check_gather_union(self, seg_idx, frame_idx, patch_idx, rows_cap=None):
        """Lists of per-question index lists (or None).  Bytes and counts exact."""
        def dev(x):
            return None if x is None else torch.tensor(x, dtype=torch.int32, device="cuda")
        kg, vg, nt = self.gpu.gather_union(dev(seg_idx), dev(frame_idx), dev(patch_idx), rows_cap)
        torch.cuda.synchronize()
        B = kg.shape[0]
        for b in range(B):
            ko, vo, n = self.orc.gather_union(() if seg_idx is None else seg_idx[b], () if frame_idx is None else frame_idx[b],
                                              () if patch_idx is None else patch_idx[b], rows_cap=kg.shape[3])
            assert int(nt[b]) == n
            np.testing.assert_array_equal(np_view(kg[b]), ko)
            np.testing.assert_array_equal(np_view(vg[b]), vo)

    def check_attend(self, layer, n_q, frame_idx, local_lens=None, causal=True, seed=0):
        """Attention of n_q new tokens per question over [kept rows of frame_idx[b], local rows of b]
        (Eq. 9) against the oracle, question by question.  frame_idx: list of lists (or None);
        local_lens: local rows per question (or None).  Returns the largest error (absolute, or
        relative to the largest output where that exceeds one)."""
        w, tol = self.w, TOL[self.w.dtype]
        B = len(frame_idx) if frame_idx is not None else len(local_lens)
        g = torch.Generator().manual_seed(seed)
        q = torch.randn(B, n_q, w.n_q_heads, w.head_dim, generator=g).to(w.torch_dtype)
        fi = None if frame_idx is None else torch.tensor(frame_idx, dtype=torch.int32, device="cuda")
        kl = vl = lo = None
        if local_lens is not None:
            offs = np.zeros(B + 1, np.int32)
            offs[1:] = np.cumsum(local_lens)
            kl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
            vl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
            lo = torch.from_numpy(offs).cuda()
        out = self.gpu.attend(layer, q.cuda(), fi, None if kl is None else kl.cuda(), None if vl is None else vl.cuda(),
                              lo, causal)
        torch.cuda.synchronize()
        got = to_f64(np_view(out.cpu()))
        worst = 0.0
        for b in range(B):
            kb = vb = None
            if local_lens is not None:
                kb, vb = np_view(kl[offs[b]:offs[b + 1]]), np_view(vl[offs[b]:offs[b + 1]])
            want = self.orc.attend(layer, np_view(q[b]), [] if frame_idx is None else frame_idx[b], kb, vb, causal)
            err = out_err(got[b], want)
            assert err <= tol, (b, err)
            worst = max(worst, err)
        return worst

    def check_prefill(self, layer, n_q, frame_idx, old_lens, causal=True, seed=0):
        """Prefill of n_q new tokens per question behind old_lens[b] older local rows, over the kept rows
        of frame_idx[b]: output and received-attention signal against the oracle.  Returns the GPU's
        (out, signal) and the largest errors."""
        w, tol = self.w, TOL[self.w.dtype]
        B = len(old_lens)
        g = torch.Generator().manual_seed(seed)
        q = torch.randn(B, n_q, w.n_q_heads, w.head_dim, generator=g).to(w.torch_dtype)
        fi = None if frame_idx is None else torch.tensor(frame_idx, dtype=torch.int32, device="cuda")
        offs = np.zeros(B + 1, np.int32)
        offs[1:] = np.cumsum([n + n_q for n in old_lens])
        kl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
        vl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
        out, sig = self.gpu.prefill_attend(layer, q.cuda(), fi, kl.cuda(), vl.cuda(), torch.from_numpy(offs).cuda(), causal)
        torch.cuda.synchronize()
        got, got_sig = to_f64(np_view(out.cpu())), sig.cpu().numpy().astype(np.float64)
        worst = worst_sig = 0.0
        for b in range(B):
            kb, vb = np_view(kl[offs[b]:offs[b + 1]]), np_view(vl[offs[b]:offs[b + 1]])
            want, want_sig = self.orc.prefill_attend(layer, np_view(q[b]), [] if frame_idx is None else frame_idx[b], kb, vb,
                                                     causal)
            err = out_err(got[b], want)
            assert err <= tol, (b, err)
            # the signal is fp32 arithmetic on the same payload values on both sides
            err_sig = float(np.abs(got_sig[b] - want_sig).max())
            assert err_sig <= 1e-6, (b, err_sig)
            worst, worst_sig = max(worst, err), max(worst_sig, err_sig)
        return out, sig, worst, worst_sig

    def close(self):
        self.gpu.close()
