"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- closed forms, invariants, numpy library routines used as
textbook special cases, brute force, and the token counts the paper prints.
None of these tests touches the HIP path."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2605_22269_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(20260522)


def bf16_bits(x):
    """float array -> bf16 bit patterns (round to nearest even), via torch."""
    return synth.as_numpy(torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16))


def bf16_value(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- Eq. 2-3 ----
class TestFrequencySignal:
    D = 64

    def _one(self, vec):
        k = np.asarray(vec, np.float32).reshape(1, 1, -1)
        return orc.fft_signal(k, 1, 1)[0, 0]

    def test_constant_key_has_only_dc(self):
        # k = c*1 -> Z[0] = D*c, all other bins 0 -> mean |Z| = |c|
        assert self._one(np.full(self.D, -2.5)) == pytest.approx(2.5, abs=1e-12)

    def test_delta_key_has_flat_spectrum(self):
        v = np.zeros(self.D)
        v[5] = 3.0
        assert self._one(v) == pytest.approx(3.0, abs=1e-12)

    def test_cosine_key_has_two_bins(self):
        d = np.arange(self.D)
        v = 1.75 * np.cos(2 * np.pi * 7 * d / self.D)  # bins 7 and D-7, each D*A/2
        got = orc.fft_signal(v.astype(np.float64).astype(np.float32).reshape(1, 1, -1), 1, 1)[0, 0]
        exact = np.abs(np.fft.fft(v.astype(np.float32).astype(np.float64))).mean()
        assert got == pytest.approx(exact, abs=1e-12)
        assert got == pytest.approx(1.75, abs=1e-6)

    def test_sine_key_sign_and_parseval(self):
        # Parseval: sum |Z|^2 = D * sum k^2 -- checked through a 2-bin signal
        d = np.arange(self.D)
        v = (0.5 * np.sin(2 * np.pi * 3 * d / self.D)).astype(np.float32)
        assert self._one(v) == pytest.approx(0.5, abs=1e-6)

    @pytest.mark.parametrize("dtype", ["f32", "bf16"])
    def test_matches_numpy_fft_along_feature_axis(self, dtype):
        Hkv, n, P, D = 3, 2, 5, 32
        x = rng.standard_normal((Hkv, n * P, D)).astype(np.float32)
        if dtype == "bf16":
            bits = bf16_bits(x)
            val = bf16_value(bits)
            got = orc.fft_signal(bits, n, P)
        else:
            val = x.astype(np.float64)
            got = orc.fft_signal(x, n, P)
        want = np.abs(np.fft.fft(val, axis=-1)).mean(axis=(0, 2)).reshape(n, P)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
        # a transform along the token axis would give something else entirely
        wrong = np.abs(np.fft.fft(val.reshape(Hkv, n, P, D), axis=2)).mean(axis=(0, 3))
        assert np.abs(wrong - want).max() > 1e-2

    def test_heads_are_averaged(self):
        D = 16
        k = np.zeros((2, 1, D), np.float32)
        k[0, 0, :] = 4.0       # constant -> 4
        k[1, 0, 3] = -1.0      # delta -> 1
        assert orc.fft_signal(k, 1, 1)[0, 0] == pytest.approx(2.5, abs=1e-12)


class TestFrequencySignalAlongTokens:
    """The other reading of Eq. 2: the transform runs over the frame's tokens, feature by feature."""

    def _frame(self, cols):
        """cols: [P][D] values of one KV head of one frame."""
        k = np.asarray(cols, np.float32)[None]
        return orc.fft_signal(k, 1, k.shape[1], orc.TOKEN_AXIS)[0]

    def test_static_frame_has_only_dc(self):
        # every token the same vector c: Z[0][d] = P c_d, all other rows 0
        P, D = 12, 8
        c = rng.standard_normal(D).astype(np.float32)
        got = self._frame(np.tile(c, (P, 1)))
        assert got[0] == pytest.approx(P * np.abs(c.astype(np.float64)).mean(), abs=1e-12)
        assert np.abs(got[1:]).max() < 1e-12

    def test_one_token_lights_every_frequency_equally(self):
        P, D = 9, 4
        x = np.zeros((P, D), np.float32)
        x[5] = [1.0, -2.0, 0.5, 4.0]
        np.testing.assert_allclose(self._frame(x), np.full(P, 7.5 / 4), atol=1e-12)

    def test_cosine_over_the_tokens_has_two_rows(self):
        P, D = 14, 3
        j = np.arange(P)[:, None]
        amp = np.array([1.0, 2.0, 0.25])
        x = (amp * np.cos(2 * np.pi * 3 * j / P)).astype(np.float32)
        got = self._frame(x)
        want = np.zeros(P)
        want[3] = want[P - 3] = P / 2 * amp.mean()
        np.testing.assert_allclose(got, want, atol=1e-5)

    @pytest.mark.parametrize("dtype", ["f32", "bf16"])
    def test_matches_numpy_fft_along_token_axis(self, dtype):
        Hkv, n, P, D = 3, 2, 7, 16                      # P not a power of two
        x = rng.standard_normal((Hkv, n * P, D)).astype(np.float32)
        if dtype == "bf16":
            bits = bf16_bits(x)
            val = bf16_value(bits)
            got = orc.fft_signal(bits, n, P, orc.TOKEN_AXIS)
        else:
            val = x.astype(np.float64)
            got = orc.fft_signal(x, n, P, orc.TOKEN_AXIS)
        want = np.abs(np.fft.fft(val.reshape(Hkv, n, P, D), axis=2)).mean(axis=(0, 3))
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
        # rows m and P - m of a real signal carry the same magnitude: the oracle makes the tie exact
        np.testing.assert_array_equal(got[:, 1:], got[:, 1:][:, ::-1])
        # and it is not the feature-axis signal
        assert np.abs(got - orc.fft_signal(bits if dtype == "bf16" else x, n, P)).max() > 1e-2

    def test_the_stream_keeps_what_this_signal_ranks_first(self):
        # alpha = 0: the keep is the top-kappa of the token-axis signal alone
        cfg = tiny_cfg(alpha=0.0, freq_axis=orc.TOKEN_AXIS)
        k, v, q = tiny_stream(cfg, 6, seed=12)
        o = run_stream(cfg, k, v, q, 3)
        sig = orc.fft_signal(k[-1], 6, cfg.tokens_per_frame, orc.TOKEN_AXIS)
        for f in range(6):
            want = np.sort(np.argsort(-sig[f], kind="stable")[:o.kappa])
            np.testing.assert_array_equal(o.kept[f], want)


# ------------------------------------------------------------------ Eq. 1 ----
def numpy_att(q, k, n, P, causal):
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    G = Hq // Hkv
    out = np.zeros((n, P))
    for f in range(n):
        for h in range(Hq):
            qq = q[h, f * P:(f + 1) * P].astype(np.float64)
            kk = k[h // G, f * P:(f + 1) * P].astype(np.float64)
            s = qq @ kk.T / math.sqrt(D)
            if causal:
                s = np.where(np.tril(np.ones((P, P), bool)), s, -np.inf)
            a = np.exp(s - s.max(axis=1, keepdims=True))
            a /= a.sum(axis=1, keepdims=True)
            out[f] += a.sum(axis=0)
    return out / (Hq * P)


class TestAttentionSignal:
    def test_two_token_closed_form(self):
        # P=2, H=1, D=1, causal: row 0 = [1, 0]; row 1 = softmax(q1*k0, q1*k1)
        q = np.array([[[0.3], [1.7]]], np.float32)
        k = np.array([[[0.9], [-0.4]]], np.float32)
        sig = 1.0 / (1.0 + math.exp(-float(q[0, 1, 0]) * (float(k[0, 0, 0]) - float(k[0, 1, 0]))))
        got = orc.att_signal(q, k, 1, 2, causal=True)[0]
        np.testing.assert_allclose(got, [(1 + sig) / 2, (1 - sig) / 2], atol=1e-14)

    def test_scale_is_inverse_sqrt_head_dim(self):
        D = 4
        q = np.zeros((1, 2, D), np.float32)
        k = np.zeros((1, 2, D), np.float32)
        q[0, 1] = [1, 2, 0, -1]
        k[0, 0] = [0.5, 0.5, 3, 0]
        k[0, 1] = [-1, 0.25, 1, 2]
        dot = float(q[0, 1] @ (k[0, 0] - k[0, 1])) / math.sqrt(D)
        sig = 1 / (1 + math.exp(-dot))
        got = orc.att_signal(q, k, 1, 2, causal=True)[0]
        np.testing.assert_allclose(got, [(1 + sig) / 2, (1 - sig) / 2], atol=1e-14)

    def test_identical_keys_non_causal_is_uniform(self):
        P, D = 7, 8
        q = rng.standard_normal((2, P, D)).astype(np.float32)
        k = np.tile(rng.standard_normal((1, 1, D)).astype(np.float32), (1, P, 1))
        np.testing.assert_allclose(orc.att_signal(q, k, 1, P, causal=False)[0], 1.0 / P, atol=1e-15)

    def test_zero_keys_causal_gives_harmonic_tail(self):
        P, D = 9, 4
        q = rng.standard_normal((3, P, D)).astype(np.float32)
        k = np.zeros((1, P, D), np.float32)
        want = [sum(1.0 / (i + 1) for i in range(j, P)) / P for j in range(P)]
        got = orc.att_signal(q, k, 1, P, causal=True)[0]
        np.testing.assert_allclose(got, want, atol=1e-15)
        assert np.all(np.diff(got) < 0)  # earlier tokens receive more attention

    @pytest.mark.parametrize("causal", [True, False])
    @pytest.mark.parametrize("dtype", ["f32", "bf16"])
    def test_matches_numpy_softmax_with_grouped_heads(self, causal, dtype):
        Hq, Hkv, n, P, D = 6, 3, 3, 11, 16
        q = rng.standard_normal((Hq, n * P, D)).astype(np.float32) * 2
        k = rng.standard_normal((Hkv, n * P, D)).astype(np.float32) * 2
        if dtype == "bf16":
            qb, kb = bf16_bits(q), bf16_bits(k)
            got = orc.att_signal(qb, kb, n, P, causal)
            want = numpy_att(bf16_value(qb), bf16_value(kb), n, P, causal)
        else:
            got = orc.att_signal(q, k, n, P, causal)
            want = numpy_att(q, k, n, P, causal)
        np.testing.assert_allclose(got, want, atol=1e-13)
        np.testing.assert_allclose(got.sum(axis=1), 1.0, atol=1e-13)  # rows of A sum to 1


# ------------------------------------------------------------------ Eq. 4 ----
class TestFusion:
    def test_hand_worked(self):
        att = np.array([[1.0, 2.0, 3.0]])
        fft = np.array([[30.0, 10.0, 20.0]])
        np.testing.assert_allclose(orc.fuse(att, fft, 0.7), [[0.3, 0.35, 0.85]], atol=1e-15)

    def test_positive_affine_invariance_and_range(self):
        att, fft = rng.random((4, 13)), rng.random((4, 13)) * 9 + 2
        base = orc.fuse(att, fft, 0.6)
        np.testing.assert_allclose(orc.fuse(att * 7 + 3, fft * 0.01 - 5, 0.6), base, atol=1e-12)
        assert base.min() >= 0 and base.max() <= 1
        a1 = orc.fuse(att, fft, 1.0)
        assert np.all(a1.min(axis=1) == 0) and np.all(a1.max(axis=1) == 1)

    def test_single_signal_modes_and_constant_signal(self):
        att, fft = rng.random((2, 9)), rng.random((2, 9))
        np.testing.assert_array_equal(orc.fuse(att, None, 1.0), orc.fuse(att, fft, 1.0))
        np.testing.assert_array_equal(orc.fuse(None, fft, 0.0), orc.fuse(att, fft, 0.0))
        lo, hi = fft.min(axis=1, keepdims=True), fft.max(axis=1, keepdims=True)
        np.testing.assert_allclose(orc.fuse(None, fft, 0.0), (fft - lo) / (hi - lo), atol=1e-15)
        const = np.full((1, 9), 3.3)
        np.testing.assert_array_equal(orc.fuse(const, fft[:1], 0.5), 0.5 * orc.fuse(None, fft[:1], 0.0))


# ---------------------------------------------------------- top-k and keep ---
class TestSelection:
    def test_brute_force_with_ties(self):
        for _ in range(50):
            n = int(rng.integers(1, 40))
            k = int(rng.integers(0, n + 3))
            s = rng.integers(0, 6, n).astype(np.float64)  # many exact ties
            idx, found = orc.topk(s, k)
            order = sorted(range(n), key=lambda i: (-s[i], i))[:k]
            assert found == min(k, n)
            assert list(idx[:found]) == order
            assert np.all(idx[found:] == -1)

    def test_all_equal_keeps_first(self):
        idx, found = orc.topk(np.zeros(10), 4)
        assert list(idx) == [0, 1, 2, 3] and found == 4

    def test_mask(self):
        s = np.array([5.0, 9.0, 7.0, 9.0, 1.0])
        idx, found = orc.topk(s, 3, mask=[1, 0, 1, 1, 0])
        assert list(idx) == [3, 2, 0] and found == 3

    def test_keep_is_ascending_topk_and_identity_at_ratio_one(self):
        fused = rng.random((5, 21))
        kept = orc.keep(fused, 6)
        for f in range(5):
            want = sorted(sorted(range(21), key=lambda i: (-fused[f, i], i))[:6])
            assert list(kept[f]) == want
        np.testing.assert_array_equal(orc.keep(fused, 21), np.tile(np.arange(21), (5, 1)))

    def test_kappa_floor_against_paper_token_counts(self):
        g = json.load(open(os.path.join(GOLDEN, "paper_token_counts.json")))
        hp = g["hyper_parameters"]
        P, F, S = hp["P"], hp["F"], hp["S"]
        unit = {"segment": P * F, "frame": P, "patch": P // S}
        kap = {n: orc.kappa_of(hp["rho"][n], unit[n]) for n in unit}
        assert kap == {"segment": 627, "frame": 19, "patch": 4}
        inf = sum(hp["k_g"][n] * kap[n] for n in unit)
        assert inf == 8212
        assert abs(inf / 1000 - g["inference_tokens"]["mukv_printed_K"]) / 8.3 < 0.02
        assert g["inference_tokens"]["rekv_blocks"] * P == 12544  # printed as 12.5K
        # memory per 300 frames: each granularity covers 196*300 tokens before pruning
        per_gran = P * 300
        assert round(3 * per_gran / 1000) in (176, 177)
        assert sum(hp["rho"].values()) * per_gran == pytest.approx(58800)  # printed as 59K
        assert orc.kappa_of(0.25, 49) == 12 and orc.kappa_of(0.125, 196) == 24
        assert orc.kappa_of(0.29, 100) == 29 and orc.kappa_of(1.0, 196) == 196

    def test_store_size_is_linear_in_kept_fraction(self):
        g = json.load(open(os.path.join(GOLDEN, "paper_token_counts.json")))["cache_size_G_per_hour"]
        for name, frac in (("ratio_1_2", 1 / 2), ("ratio_2_3", 1 / 3), ("ratio_3_4", 1 / 4)):
            assert g["ratio_0"] * frac == pytest.approx(g[name], abs=0.025)


# --------------------------------------------- compaction, pooling, whole path
def tiny_cfg(**kw):
    base = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=16, tokens_per_frame=13,
                frames_per_segment=3, superpatches_per_frame=4, keep_ratio=0.4, alpha=0.7)
    base.update(kw)
    return orc.OracleConfig(**base)


def tiny_stream(cfg, n_frames, dtype="f32", seed=1):
    w = synth.Workload("t", cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dtype, n_frames,
                       cfg.tokens_per_frame, cfg.frames_per_segment, spike_prob=0.1)
    k, v, q = synth.SynthStream(w, seed).next_chunk(n_frames)
    return synth.as_numpy(k), synth.as_numpy(v), synth.as_numpy(q)


def run_stream(cfg, k, v, q, chunk):
    o = orc.OracleMuKV(cfg)
    P = cfg.tokens_per_frame
    n = k.shape[2] // P
    for f0 in range(0, n, chunk):
        f1 = min(f0 + chunk, n)
        o.compress_chunk(k[:, :, f0 * P:f1 * P], v[:, :, f0 * P:f1 * P], q[:, f0 * P:f1 * P])
    return o


class TestCompactionAndPooling:
    @pytest.mark.parametrize("dtype", ["f32", "bf16"])
    def test_store_equals_fancy_index(self, dtype):
        cfg = tiny_cfg()
        k, v, q = tiny_stream(cfg, 7, dtype)
        o = run_stream(cfg, k, v, q, 3)
        P, kap = cfg.tokens_per_frame, o.kappa
        assert kap == 5
        rows = (np.arange(7)[:, None] * P + o.kept).reshape(-1)
        sk, sv = o.store()
        assert sk.shape == (2, 2, 7 * kap, 16) and sk.dtype == k.dtype
        np.testing.assert_array_equal(sk, k[:, :, rows])
        np.testing.assert_array_equal(sv, v[:, :, rows])

    def test_keep_ratio_one_is_identity(self):
        cfg = tiny_cfg(keep_ratio=1.0)
        k, v, q = tiny_stream(cfg, 4)
        o = run_stream(cfg, k, v, q, 2)
        sk, sv = o.store()
        np.testing.assert_array_equal(sk, k)
        np.testing.assert_array_equal(sv, v)
        # mean over all tokens of a frame
        want = k[-1].astype(np.float64).reshape(2, 4, 13, 16).mean(axis=2).transpose(1, 0, 2).reshape(4, -1)
        np.testing.assert_allclose(o.rep_frame_k, want, atol=1e-14)

    def test_mean_of_identical_tokens_is_the_token(self):
        x = np.tile(rng.standard_normal((2, 1, 8)).astype(np.float32), (1, 6, 1))
        np.testing.assert_array_equal(orc.pool_rows(x, [1, 3, 4]), x[:, 0].reshape(-1).astype(np.float64))
        np.testing.assert_array_equal(orc.pool_rows(x, []), np.zeros(16))

    def test_pool_rows_matches_numpy_mean_bf16(self):
        x = bf16_bits(rng.standard_normal((3, 10, 8)))
        rows = [7, 0, 2, 9]
        want = bf16_value(x)[:, rows].mean(axis=1).reshape(-1)
        np.testing.assert_allclose(orc.pool_rows(x, rows), want, atol=1e-15)

    def test_block_hierarchy_consistency(self):
        cfg = tiny_cfg()
        k, v, q = tiny_stream(cfg, 8)
        o = run_stream(cfg, k, v, q, 8)
        S, F, kap = 4, 3, o.kappa
        # frame key = count-weighted mean of its super-patch keys
        cnt = o.cnt_patch.reshape(8, S)
        assert np.all(cnt.sum(axis=1) == kap)
        recon = (o.rep_patch_k.reshape(8, S, -1) * cnt[:, :, None]).sum(axis=1) / kap
        np.testing.assert_allclose(recon, o.rep_frame_k, atol=1e-14)
        # super-patch membership follows the index-contiguous partition 3,3,3,4
        assert orc.superpatch_bounds(13, 4) == [(0, 3), (3, 6), (6, 9), (9, 13)]
        assert orc.superpatch_bounds(49, 4) == [(0, 12), (12, 24), (24, 36), (36, 49)]
        # segment key = mean of its frame keys (kappa is the same for every frame)
        seg = o.seg_reps()
        assert seg.shape[0] == 3  # 3 + 3 + 2 frames
        for s in range(3):
            np.testing.assert_allclose(seg[s], o.rep_frame_k[s * F:min((s + 1) * F, 8)].mean(axis=0), atol=1e-14)
        segv = o.seg_reps(which="v")
        np.testing.assert_allclose(segv[2], o.rep_frame_v[6:8].mean(axis=0), atol=1e-14)
        # a question asked before the end of the stream sees only earlier frames
        np.testing.assert_allclose(o.seg_reps(n_visible=5)[1], o.rep_frame_k[3:5].mean(axis=0), atol=1e-14)

    def test_chunking_invariance(self):
        cfg = tiny_cfg()
        k, v, q = tiny_stream(cfg, 9)
        ref = run_stream(cfg, k, v, q, 9)
        for chunk in (1, 2, 4):
            o = run_stream(cfg, k, v, q, chunk)
            np.testing.assert_array_equal(o.kept, ref.kept)
            np.testing.assert_array_equal(o.store()[0], ref.store()[0])
            np.testing.assert_allclose(o.rep_frame_k, ref.rep_frame_k, atol=1e-14)
            np.testing.assert_allclose(o.seg_reps(), ref.seg_reps(), atol=1e-14)

    def test_attention_handed_over_equals_attention_recomputed(self):
        cfg = tiny_cfg()
        k, v, q = tiny_stream(cfg, 3)
        a = orc.att_signal(q, k[-1], 3, 13, True)
        o1 = orc.OracleMuKV(cfg)
        r1 = o1.compress_chunk(k, v, q_last=q)
        o2 = orc.OracleMuKV(cfg)
        r2 = o2.compress_chunk(k, v, att=a)
        np.testing.assert_array_equal(r1["kept"], r2["kept"])

    def test_spiked_tokens_are_kept_by_the_frequency_signal(self):
        # |Z| scales with the key, so a token whose key is 3x larger must win
        cfg = tiny_cfg(alpha=0.0, keep_ratio=0.1)
        k, v, q = tiny_stream(cfg, 2)
        k = k.copy()
        k[:, :, 4] *= 25
        k[:, :, 13 + 9] *= 25
        o = orc.OracleMuKV(cfg)
        r = o.compress_chunk(k, v, None)
        assert o.kappa == 1 and list(r["kept"][:, 0]) == [4, 9]


class TestSegmentAsUnit:
    """Sec. 3.3 with a whole segment as the unit of Eq. 4 (the coarsest granularity keeps a
    fraction of the segment's tokens, wherever they lie): the unit is F_u frames of p tokens,
    its attention signal is handed over, its super-patches are its frames."""

    def cfg(self, **kw):
        base = dict(tokens_per_frame=6 * 49, superpatches_per_frame=6, frames_per_segment=1, keep_ratio=0.8, alpha=0.8)
        base.update(kw)
        return tiny_cfg(**base)

    def test_ramp_of_attention_over_equal_keys_keeps_the_top_of_the_ramp(self):
        cfg = self.cfg()
        P, kap = cfg.tokens_per_frame, int(0.8 * 6 * 49 + 1e-9)
        k = np.ones((2, 2, 2 * P, 16), np.float32)  # equal keys: the frequency indicator is flat and drops out
        v = rng.standard_normal(k.shape).astype(np.float32)
        ramp = np.stack([np.arange(P, dtype=np.float64), np.arange(P, 0, -1, dtype=np.float64)])
        o = orc.OracleMuKV(cfg)
        r = o.compress_chunk(k, v, att=ramp)
        assert o.kappa == kap == 235
        np.testing.assert_array_equal(r["kept"][0], np.arange(P - kap, P))  # rising ramp: the last kappa tokens
        np.testing.assert_array_equal(r["kept"][1], np.arange(kap))         # falling ramp: the first kappa
        # the unit's frames are its super-patches: 59 tokens go, the first frame and 10 of the second
        assert list(o.cnt_patch.reshape(2, 6)[0]) == [0, 39, 49, 49, 49, 49]
        assert list(o.cnt_patch.reshape(2, 6)[1]) == [49, 49, 49, 49, 39, 0]

    def test_tokens_are_ranked_over_the_unit_not_per_frame(self):
        # all of the attention mass in one frame of the unit: that frame is kept whole and the
        # other frames share what is left, which a per-frame ratio could not do
        cfg = self.cfg(alpha=1.0, keep_ratio=0.25)
        P = cfg.tokens_per_frame
        k, v, _ = tiny_stream(cfg, 1)
        att = np.zeros((1, P))
        att[0, 3 * 49:4 * 49] = 1.0 + rng.random(49)
        o = orc.OracleMuKV(cfg)
        r = o.compress_chunk(k, v, att=att)
        kap = o.kappa
        assert kap == 73
        kept = r["kept"][0]
        assert set(range(3 * 49, 4 * 49)) <= set(kept)
        # the remaining 24 slots go to equal (zero) scores: the earliest positions
        np.testing.assert_array_equal(kept[:kap - 49], np.arange(kap - 49))
        assert list(o.cnt_patch.reshape(1, 6)[0]) == [kap - 49, 0, 0, 49, 0, 0]

    def test_block_keys_of_the_unit_are_means_of_its_kept_rows(self):
        cfg = self.cfg()
        P = cfg.tokens_per_frame
        k, v, _ = tiny_stream(cfg, 3, "bf16")
        att = rng.random((3, P))
        o = orc.OracleMuKV(cfg)
        r = o.compress_chunk(k, v, att=att)
        kv = bf16_value(k[-1])  # scoring layer, [Hkv][3P][D]
        for u in range(3):
            kept = r["kept"][u]
            rows = kv[:, u * P + kept]                                  # [Hkv][kappa][D]
            np.testing.assert_allclose(o.rep_frame_k[u], rows.mean(axis=1).reshape(-1), atol=1e-14)
            for s in range(6):
                inside = kept[(kept >= s * 49) & (kept < (s + 1) * 49)]
                want = kv[:, u * P + inside].mean(axis=1).reshape(-1) if len(inside) else np.zeros(32)
                np.testing.assert_allclose(o.rep_patch_k[u * 6 + s], want, atol=1e-14)
        # a segment of one unit has the unit's key
        np.testing.assert_allclose(o.seg_reps(), o.rep_frame_k, atol=1e-14)


# ------------------------------------------------------------- Eq. 6, 7, 8 ---
class TestRetrieval:
    def test_question_pooling_is_token_mean(self):
        qt = rng.standard_normal((5, 3, 4)).astype(np.float32)
        np.testing.assert_allclose(orc.pool_question(qt), qt.astype(np.float64).mean(axis=0).reshape(-1), atol=1e-15)

    def test_cosine_against_closed_form_and_numpy(self):
        Hq, Hkv, D, N = 6, 2, 8, 9
        G = Hq // Hkv
        q = rng.standard_normal(Hq * D)
        reps = rng.standard_normal((N, Hkv * D)).astype(np.float32)
        got = orc.score_blocks(q, reps, Hq, Hkv, D)
        # closed form: group-sum of q against the un-expanded key
        qg = q.reshape(Hkv, G, D).sum(axis=1).reshape(-1)
        r64 = reps.astype(np.float64)
        want = (r64 @ qg) / (np.linalg.norm(q) * math.sqrt(G) * np.linalg.norm(r64, axis=1))
        np.testing.assert_allclose(got, want, atol=1e-14)
        assert np.all(np.abs(got) <= 1 + 1e-15)
        # invariant to positive scaling of either side
        np.testing.assert_allclose(orc.score_blocks(q * 3.5, reps * np.float32(0.25), Hq, Hkv, D), got, atol=1e-14)
        # no grouping: plain cosine
        q2 = rng.standard_normal(Hkv * D)
        plain = (r64 @ q2) / (np.linalg.norm(q2) * np.linalg.norm(r64, axis=1))
        np.testing.assert_allclose(orc.score_blocks(q2, reps, Hkv, Hkv, D), plain, atol=1e-14)
        # head h must read KV head h // G, not h % Hkv
        wrong = r64.reshape(N, Hkv, 1, D).repeat(G, axis=2).transpose(0, 2, 1, 3).reshape(N, -1)
        wrong = (wrong @ q) / (np.linalg.norm(q) * np.linalg.norm(wrong, axis=1))
        assert np.abs(wrong - got).max() > 1e-3

    def test_zero_key_scores_zero(self):
        reps = np.zeros((1, 8), np.float32)
        assert orc.score_blocks(np.ones(16), reps, 4, 2, 4)[0] == 0.0

    def test_consistency_is_one_for_the_global_query_itself(self):
        reps = rng.standard_normal((4, 12)).astype(np.float32)
        g = reps[2].astype(np.float64) * 5
        got = orc.consistency(g, reps, [2, 0])
        assert got[0] == pytest.approx(1.0, abs=1e-15)
        want = reps[0].astype(np.float64) @ g / np.linalg.norm(reps[0].astype(np.float64)) / np.linalg.norm(g)
        assert got[1] == pytest.approx(want, abs=1e-15)

    def _state(self, n_frames=24, **kw):
        cfg = tiny_cfg(frames_per_segment=4, **kw)
        k, v, q = tiny_stream(cfg, n_frames, seed=3)
        return cfg, run_stream(cfg, k, v, q, 8)

    def test_lambda_zero_semi_equals_parallel(self):
        cfg, o = self._state()
        qt = rng.standard_normal((6, 4, 16)).astype(np.float32)
        a = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 2, 5, lambda_frame=0.0))
        b = o.retrieve(qt, orc.RetrieveParams(orc.PARALLEL, 2, 5))
        np.testing.assert_array_equal(a["frame_idx"], b["frame_idx"])
        np.testing.assert_array_equal(a["seg_idx"], b["seg_idx"])
        np.testing.assert_allclose(a["frame_score"], b["frame_score"], atol=1e-15)

    def test_semi_rerank_by_hand(self):
        cfg, o = self._state()
        qt = rng.standard_normal((6, 4, 16)).astype(np.float32)
        prm = orc.RetrieveParams(orc.SEMI, 2, 3, lambda_frame=0.3)
        r = o.retrieve(qt, prm)
        # segments keep their stage-1 order
        par = o.retrieve(qt, orc.RetrieveParams(orc.PARALLEL, 2, 3))
        np.testing.assert_array_equal(r["seg_idx"], par["seg_idx"])
        # redo stage 2 with numpy on the stage-1 candidates
        s = r["s_frm"]
        cand = sorted(range(24), key=lambda i: (-s[i], i))[:6]
        assert list(r["cand_frm"]) == cand
        sseg = r["s_seg"]
        top_seg = sorted(range(6), key=lambda i: (-sseg[i], i))[:2]
        g = o.seg_reps().astype(np.float32).astype(np.float64)[top_seg].mean(axis=0)
        reps = o.rep_frame_k.astype(np.float32).astype(np.float64)
        gam = [reps[j] @ g / np.linalg.norm(reps[j]) / np.linalg.norm(g) for j in cand]
        st = [0.7 * s[j] + 0.3 * gm for j, gm in zip(cand, gam)]
        order = sorted(range(6), key=lambda c: (-st[c], cand[c]))[:3]
        assert list(r["frame_idx"]) == [cand[c] for c in order]
        np.testing.assert_allclose(r["frame_score"], [st[c] for c in order], atol=1e-14)

    def test_hier_frames_lie_in_chosen_segments(self):
        cfg, o = self._state()
        qt = rng.standard_normal((6, 4, 16)).astype(np.float32)
        r = o.retrieve(qt, orc.RetrieveParams(orc.HIER, 2, 5))
        segs = set(int(s) for s in r["seg_idx"])
        assert all(int(f) // 4 in segs for f in r["frame_idx"])
        s = r["s_frm"]
        allowed = [i for i in range(24) if i // 4 in segs]
        assert list(r["frame_idx"]) == sorted(allowed, key=lambda i: (-s[i], i))[:5]

    def test_k_larger_than_available_pads_with_minus_one(self):
        cfg, o = self._state(n_frames=6)
        qt = rng.standard_normal((2, 4, 16)).astype(np.float32)
        for mode in (orc.SEMI, orc.HIER, orc.PARALLEL):
            r = o.retrieve(qt, orc.RetrieveParams(mode, 3, 8))
            assert list(r["seg_idx"][2:]) == [-1] and sorted(r["seg_idx"][:2]) == [0, 1]
            assert list(r["frame_idx"][6:]) == [-1, -1] and sorted(r["frame_idx"][:6]) == list(range(6))

    def test_timestamp_constraint(self):
        cfg, o = self._state()
        qt = rng.standard_normal((3, 4, 16)).astype(np.float32)
        r = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 2, 4, n_visible_frames=10))
        assert all(0 <= f < 10 for f in r["frame_idx"]) and all(0 <= s < 3 for s in r["seg_idx"])
        assert r["s_seg"].shape == (3,) and r["s_frm"].shape == (10,)

    def test_planted_targets_are_retrieved(self):
        cfg, o = self._state(n_frames=40)
        w = synth.Workload("t", 2, 4, 2, 16, "f32", 40, 13, 4)
        targets = [5, 17, 33]
        qt = synth.as_numpy(synth.planted_question(w, torch.from_numpy(o.rep_frame_k[targets]), 12, seed=9, cosine=0.8))
        r = o.retrieve(qt, orc.RetrieveParams(orc.PARALLEL, 3, 3))
        assert sorted(int(f) for f in r["frame_idx"]) == targets

    def test_gather_is_temporal_concatenation(self):
        cfg, o = self._state()
        sk, sv = o.store()
        kap = o.kappa
        ko, vo, n = o.gather(np.array([9, 2, -1, 4], np.int32))
        assert n == 3 * kap
        rows = np.concatenate([np.arange(f * kap, (f + 1) * kap) for f in (2, 4, 9)])
        np.testing.assert_array_equal(ko[:, :, :n], sk[:, :, rows])
        np.testing.assert_array_equal(vo[:, :, :n], sv[:, :, rows])
        assert not ko[:, :, n:].any()
        ko2, _, _ = o.gather(np.array([9, 2, -1, 4], np.int32), order=orc.AS_GIVEN)
        rows2 = np.concatenate([np.arange(f * kap, (f + 1) * kap) for f in (9, 2, 4)])
        np.testing.assert_array_equal(ko2[:, :, :n], sk[:, :, rows2])


class TestRetrievalLooseEnds:
    """Branches of the retrieval and of the gathers that the pins above leave out."""

    def _state(self, n_frames=24):
        cfg = tiny_cfg(frames_per_segment=4)
        k, v, q = tiny_stream(cfg, n_frames, seed=3)
        return cfg, run_stream(cfg, k, v, q, 8)

    def test_global_query_of_the_first_n_segments_by_hand(self):
        # n_global = 1: the global query is the single best segment's key, not the mean of the top k_seg
        cfg, o = self._state()
        qt = rng.standard_normal((5, 4, 16)).astype(np.float32)
        r1 = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 3, 4, lambda_frame=0.6, n_global=1))
        r3 = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 3, 4, lambda_frame=0.6, n_global=0))
        sseg, s = r1["s_seg"], r1["s_frm"]
        best = sorted(range(6), key=lambda i: (-sseg[i], i))
        seg32 = o.seg_reps().astype(np.float32).astype(np.float64)
        np.testing.assert_allclose(r1["g"], seg32[best[0]], atol=0)
        np.testing.assert_allclose(r3["g"], seg32[best[:3]].mean(axis=0), atol=1e-15)
        reps = o.rep_frame_k.astype(np.float32).astype(np.float64)
        cand = sorted(range(24), key=lambda i: (-s[i], i))[:8]
        for r, g in ((r1, seg32[best[0]]), (r3, seg32[best[:3]].mean(axis=0))):
            st = [0.4 * s[j] + 0.6 * (reps[j] @ g) / np.linalg.norm(reps[j]) / np.linalg.norm(g) for j in cand]
            order = sorted(range(8), key=lambda c: (-st[c], cand[c]))[:4]
            assert list(r["frame_idx"]) == [cand[c] for c in order]
        # the two global queries differ, and with lambda = 0.6 so do the reranked scores
        assert np.abs(r1["frame_score"] - r3["frame_score"]).max() > 1e-6
        # n_global beyond the stage-1 segment candidates is clamped to them
        r9 = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 3, 4, lambda_frame=0.6, n_global=99))
        np.testing.assert_allclose(r9["g"], seg32[best[:6]].mean(axis=0), atol=1e-15)

    def test_gather_skips_numbers_that_name_no_frame(self):
        cfg, o = self._state(n_frames=10)
        sk, sv = o.store()
        kap = o.kappa
        ko, vo, n = o.gather(np.array([7, 10, -1, 3, 4096, -5], np.int32))
        assert n == 2 * kap
        rows = np.concatenate([np.arange(f * kap, (f + 1) * kap) for f in (3, 7)])
        np.testing.assert_array_equal(ko[:, :, :n], sk[:, :, rows])
        np.testing.assert_array_equal(vo[:, :, :n], sv[:, :, rows])
        assert ko.shape[2] == 6 * kap and not ko[:, :, n:].any() and not vo[:, :, n:].any()

    def test_attend_skips_numbers_that_name_no_frame(self):
        cfg, o = self._state(n_frames=10)
        q = rng.standard_normal((2, 4, 16)).astype(np.float32)
        a = o.attend(1, q, [7, 3])
        b = o.attend(1, q, [10, 7, -1, 3, 4096])
        np.testing.assert_array_equal(a, b)
        assert np.abs(a).max() > 0


class TestThreeStores:
    """Sec. 3.3 (granularity-adaptive compression) and Sec. 3.4 stage 2 with the paper's three
    independently compressed caches: a segment store (units of O = F*P tokens), a frame store
    (the middle frame of every segment, P tokens) and a patch store (the S super-patches of
    that frame, floor(P/S) tokens each)."""

    def _stores(self, T, P=12, F=2, S=3, rhos=(0.8, 0.25, 0.5), alphas=(0.8, 0.7, 0.5), seed=41, dtype="f32"):
        """T time steps; one K/V stream of T*F frames; store i is fed its own view of it."""
        base = tiny_cfg(tokens_per_frame=P, frames_per_segment=F)
        k, v, _ = tiny_stream(base, T * F, dtype=dtype, seed=seed)
        mid = F // 2
        tok_seg = np.arange(T * F * P)
        tok_frm = np.concatenate([(t * F + mid) * P + np.arange(P) for t in range(T)])
        units = (P * F, P, P // S)
        stores = []
        for i, (toks, u) in enumerate(zip((tok_seg, tok_frm, tok_frm), units)):
            if i == 2:   # the S super-patches of the middle frame, floor(P/S) tokens each (Sec. 3.2)
                toks = np.concatenate([(t * F + mid) * P + np.arange(S * u) for t in range(T)])
            cfg = tiny_cfg(tokens_per_frame=u, frames_per_segment=1, superpatches_per_frame=1, keep_ratio=rhos[i],
                           alpha=alphas[i])
            o = orc.OracleMuKV(cfg)
            n_units = toks.shape[0] // u
            att = np.random.default_rng(seed + i).random((n_units, u))
            o.compress_chunk(np.ascontiguousarray(k[:, :, toks]), np.ascontiguousarray(v[:, :, toks]), att=att)
            stores.append(o)
        return stores, k, v, (tok_seg, tok_frm)

    def test_paper_default_run_gathers_the_printed_token_count(self):
        # Sec. 4.1: P = 196, F = 4, S = 4, rho = 0.8 / 0.1 / 0.1 and k_g = 12 / 32 / 20 for segment / frame /
        # patch; Table 1 prints 8.3K inference tokens for it: 12 * 627 + 32 * 19 + 20 * 4 = 8212
        gold = json.load(open(os.path.join(GOLDEN, "paper_token_counts.json")))
        hp = gold["hyper_parameters"]
        P, F, S = hp["P"], hp["F"], hp["S"]
        rho, kg = hp["rho"], hp["k_g"]
        T = 36  # time steps: more than 32 frames, 12 segments and 20 of the 4 T super-patches
        base = orc.OracleConfig(1, 2, 1, 16, P, F)
        w = synth.Workload("t", 1, 2, 1, 16, "bf16", T * F, P, F)
        kt, vt, _ = synth.SynthStream(w, 77).next_chunk(T * F)
        k, v = synth.as_numpy(kt), synth.as_numpy(vt)
        mid = F // 2
        tok_frm = np.concatenate([(t * F + mid) * P + np.arange(P) for t in range(T)])
        tok_pat = np.concatenate([(t * F + mid) * P + np.arange(S * (P // S)) for t in range(T)])
        views = ((np.arange(T * F * P), P * F, rho["segment"], 0.8), (tok_frm, P, rho["frame"], 0.7),
                 (tok_pat, P // S, rho["patch"], 0.5))
        stores = []
        for i, (toks, u, r, al) in enumerate(views):
            o = orc.OracleMuKV(orc.OracleConfig(1, 2, 1, 16, u, 1, 1, r, al))
            att = np.random.default_rng(500 + i).random((toks.shape[0] // u, u))
            o.compress_chunk(np.ascontiguousarray(k[:, :, toks]), np.ascontiguousarray(v[:, :, toks]), att=att)
            stores.append(o)
        assert [o.kappa for o in stores] == [627, 19, 4]
        assert [o.n_frames for o in stores] == [T, T, S * T]
        qt = rng.standard_normal((9, 2, 16)).astype(np.float32)
        res = orc.retrieve_multi(stores, qt, [kg["segment"], kg["frame"], kg["patch"]], [0.0, 0.3, 0.3])
        assert all((r["idx"] >= 0).all() for r in res)
        ko, vo, n = orc.gather_multi(stores, [r["idx"] for r in res], [1, 1, S])
        assert n == 12 * 627 + 32 * 19 + 20 * 4 == 8212
        assert abs(n / 1000 - gold["inference_tokens"]["mukv_printed_K"]) <= 0.1    # 8.2K against the printed 8.3K
        assert ko.shape == (1, 1, 8212, 16)

    def test_rerank_of_the_finer_stores_by_hand(self):
        stores, k, v, _ = self._stores(T=9)
        qt = rng.standard_normal((4, 4, 16)).astype(np.float32)
        ks, lams = [2, 3, 4], [0.0, 0.3, 0.6]
        res = orc.retrieve_multi(stores, qt, ks, lams, n_global=2)
        # the literal definitions with numpy: the query expanded over the grouped heads, plain cosines
        q = qt.astype(np.float64).mean(axis=0).reshape(-1)                       # [Hq*D]

        def cosines(o):
            keys = o.rep_frame_k.astype(np.float32).astype(np.float64)           # [n][Hkv*D]
            wide = np.repeat(keys.reshape(len(keys), 2, 16), 2, axis=1).reshape(len(keys), -1)   # each KV head twice
            return keys, wide @ q / np.linalg.norm(wide, axis=1) / np.linalg.norm(q)
        keys0, s0 = cosines(stores[0])
        top0 = sorted(range(len(s0)), key=lambda i: (-s0[i], i))
        assert list(res[0]["idx"]) == top0[:2]
        g = keys0[top0[:2]].mean(axis=0)
        np.testing.assert_allclose(res[0]["g"], g, atol=1e-15)
        for i in (1, 2):
            keys, s = cosines(stores[i])
            cand = sorted(range(len(s)), key=lambda j: (-s[j], j))[:2 * ks[i]]
            gam = [keys[j] @ g / np.linalg.norm(keys[j]) / np.linalg.norm(g) for j in cand]
            st = [(1 - lams[i]) * s[j] + lams[i] * gm for j, gm in zip(cand, gam)]
            order = sorted(range(len(cand)), key=lambda c: (-st[c], cand[c]))[:ks[i]]
            assert list(res[i]["idx"]) == [cand[c] for c in order]
            np.testing.assert_allclose(res[i]["score"], [st[c] for c in order], atol=1e-14)

    def test_without_the_consistency_term_every_store_keeps_its_stage_one_ranking(self):
        stores, *_ = self._stores(T=8)
        qt = rng.standard_normal((3, 4, 16)).astype(np.float32)
        res = orc.retrieve_multi(stores, qt, [3, 3, 5], [0.0, 0.0, 0.0])
        for o, r, kk in zip(stores, res, [3, 3, 5]):
            s = r["s"]
            assert list(r["idx"]) == sorted(range(len(s)), key=lambda j: (-s[j], j))[:kk]

    def test_a_unit_whose_key_is_the_global_query_is_fully_consistent(self):
        stores, *_ = self._stores(T=6)
        qt = rng.standard_normal((3, 4, 16)).astype(np.float32)
        g = stores[1].rep_frame_k[4].astype(np.float32).astype(np.float64)
        r = orc.retrieve_units(stores[1], qt, 6, lam=1.0, g_in=g)             # lambda = 1: the ranking is gamma alone
        assert r["idx"][0] == 4 and r["score"][0] == pytest.approx(1.0, abs=1e-12)

    def test_more_units_asked_for_than_exist(self):
        stores, *_ = self._stores(T=3)
        qt = rng.standard_normal((3, 4, 16)).astype(np.float32)
        res = orc.retrieve_multi(stores, qt, [5, 5, 12], [0.0, 0.3, 0.3])
        assert sorted(res[0]["idx"][:3]) == [0, 1, 2] and list(res[0]["idx"][3:]) == [-1, -1]
        assert sorted(res[2]["idx"][:9]) == list(range(9)) and list(res[2]["idx"][9:]) == [-1, -1, -1]

    def test_the_context_is_the_kept_rows_in_temporal_order(self):
        T, P, F, S = 7, 12, 2, 3
        stores, k, v, (tok_seg, tok_frm) = self._stores(T=T, P=P, F=F, S=S, dtype="bf16")
        seg, frm, pat = [5, 1, -1], [6, 1, 1, 3], [3 * S + 2, 1 * S + 0, 99, 5 * S + 1]
        ko, vo, n = orc.gather_multi(stores, [seg, frm, pat], [1, 1, S])
        # straight from the inputs: per time step the segment's kept tokens, the middle frame's, the super-patches'
        mid, u = F // 2, P // S
        want = []
        for t in range(T):
            if t in seg:
                want += [t * F * P + j for j in stores[0].kept[t]]
            if t in frm:
                want += [(t * F + mid) * P + j for j in stores[1].kept[t]]
            for sp in range(S):
                if t * S + sp in pat:
                    want += [(t * F + mid) * P + sp * u + j for j in stores[2].kept[t * S + sp]]
        assert n == len(want) == 2 * stores[0].kappa + 3 * stores[1].kappa + 3 * stores[2].kappa
        np.testing.assert_array_equal(ko[:, :, :n], k[:, :, want])
        np.testing.assert_array_equal(vo[:, :, :n], v[:, :, want])
        # a cap below the context cuts it; above, the tail stays zero
        kc, _, n2 = orc.gather_multi(stores, [seg, frm, pat], [1, 1, S], rows_cap=10)
        assert n2 == n and kc.shape[2] == 10
        np.testing.assert_array_equal(kc, ko[:, :, :10])
        kz, vz, _ = orc.gather_multi(stores, [seg, frm, pat], [1, 1, S], rows_cap=n + 5)
        assert not kz[:, :, n:].any() and not vz[:, :, n:].any()


class TestPatchLevel:
    """Super-patches as the fine level of the search and of the gather (Sec. 3.2, 3.4)."""

    def _state(self, n_frames=24, **kw):
        cfg = tiny_cfg(frames_per_segment=4, **kw)
        k, v, q = tiny_stream(cfg, n_frames, seed=5)
        return cfg, run_stream(cfg, k, v, q, 8), (k, v)

    @pytest.mark.parametrize("mode", [orc.SEMI, orc.HIER, orc.PARALLEL])
    def test_one_super_patch_per_frame_is_the_frame_level(self, mode):
        cfg, o, _ = self._state(superpatches_per_frame=1)
        qt = rng.standard_normal((5, 4, 16)).astype(np.float32)
        prm = orc.RetrieveParams(mode, 2, 5, lambda_frame=0.4)
        a, b = o.retrieve(qt, prm), o.retrieve(qt, prm, level="patch")
        np.testing.assert_array_equal(a["frame_idx"], b["frame_idx"])
        np.testing.assert_array_equal(a["frame_score"], b["frame_score"])
        ka, va, na = o.gather(a["frame_idx"])
        kb, vb, nb = o.gather_patches(b["frame_idx"])
        assert na == nb
        np.testing.assert_array_equal(ka, kb)
        np.testing.assert_array_equal(va, vb)

    def test_parallel_mode_is_a_masked_argsort_of_literal_cosines(self):
        cfg, o, _ = self._state(keep_ratio=0.2)            # kappa = 2 of 13: at least two empty super-patches per frame
        assert (o.cnt_patch == 0).any()
        qt = rng.standard_normal((7, 4, 16)).astype(np.float32)
        r = o.retrieve(qt, orc.RetrieveParams(orc.PARALLEL, 2, 9), level="patch")
        q = qt.astype(np.float64).mean(axis=0).reshape(-1)                       # Eq. 6, heads concatenated
        reps = o.rep_patch_k.astype(np.float32).astype(np.float64)
        G = cfg.n_q_heads // cfg.n_kv_heads
        full = np.repeat(reps.reshape(len(reps), cfg.n_kv_heads, 1, cfg.head_dim), G, axis=2).reshape(len(reps), -1)
        with np.errstate(invalid="ignore", divide="ignore"):
            cos = full @ q / (np.linalg.norm(full, axis=1) * np.linalg.norm(q))
        cos[o.cnt_patch.reshape(-1) == 0] = -np.inf
        want = np.argsort(-cos, kind="stable")[:9]
        np.testing.assert_array_equal(r["frame_idx"], want)
        assert all(o.cnt_patch.reshape(-1)[p] > 0 for p in r["frame_idx"])

    def test_lambda_zero_semi_equals_parallel_and_hier_stays_inside(self):
        cfg, o, _ = self._state()
        qt = rng.standard_normal((6, 4, 16)).astype(np.float32)
        a = o.retrieve(qt, orc.RetrieveParams(orc.SEMI, 2, 7, lambda_frame=0.0), level="patch")
        b = o.retrieve(qt, orc.RetrieveParams(orc.PARALLEL, 2, 7), level="patch")
        np.testing.assert_array_equal(a["frame_idx"], b["frame_idx"])
        h = o.retrieve(qt, orc.RetrieveParams(orc.HIER, 2, 7), level="patch")
        per_seg = cfg.frames_per_segment * cfg.superpatches_per_frame
        assert all(p // per_seg in set(int(s) for s in h["seg_idx"]) for p in h["frame_idx"] if p >= 0)

    def test_planted_super_patches_are_retrieved(self):
        cfg, o, _ = self._state(n_frames=40)
        w = synth.Workload("t", 2, 4, 2, 16, "f32", 40, 13, 4)
        full = [p for p in range(160) if o.cnt_patch.reshape(-1)[p] > 0]
        for i, target in enumerate((full[3], full[40], full[77])):       # one target per question: keys of 32
            key = torch.from_numpy(o.rep_patch_k.reshape(-1, 32)[[target]])  # channels are too noisy for a mean of several
            qt = synth.as_numpy(synth.planted_question(w, key, 12, seed=9 + i, cosine=0.95))
            for mode in (orc.PARALLEL, orc.SEMI):
                r = o.retrieve(qt, orc.RetrieveParams(mode, 3, 2, lambda_frame=0.2), level="patch")
                assert int(r["frame_idx"][0]) == target

    def test_gather_is_the_kept_rows_inside_each_super_patch(self):
        cfg, o, (k, v) = self._state()
        P, S, kap = cfg.tokens_per_frame, cfg.superpatches_per_frame, o.kappa
        cap = min(kap, P - (S - 1) * (P // S))
        sel = np.array([4 * 7 + 3, -1, 4 * 2 + 1, 4 * 7 + 0, 4 * 20 + 2], np.int32)
        ko, vo, n = o.gather_patches(sel)
        tok = []
        for pid in sorted(int(x) for x in sel if x >= 0):                       # straight from the inputs
            f, sp = divmod(pid, S)
            lo, hi = orc.superpatch_bounds(P, S)[sp]
            tok += [f * P + j for j in o.kept[f] if lo <= j < hi]
        assert n == len(tok) and ko.shape[2] == len(sel) * cap
        np.testing.assert_array_equal(ko[:, :, :n], k[:, :, tok])
        np.testing.assert_array_equal(vo[:, :, :n], v[:, :, tok])
        assert not ko[:, :, n:].any() and not vo[:, :, n:].any()
        # all S super-patches of a frame, in order, are the frame
        kf, vf, nf = o.gather(np.array([7], np.int32))
        kp, vp, npat = o.gather_patches(np.arange(4 * 7, 4 * 8, dtype=np.int32))
        assert nf == npat == kap
        np.testing.assert_array_equal(kf[:, :, :kap], kp[:, :, :kap])
        np.testing.assert_array_equal(vf[:, :, :kap], vp[:, :, :kap])
        # list order
        k2, _, n2 = o.gather_patches(sel, order=orc.AS_GIVEN)
        tok2 = []
        for pid in (int(x) for x in sel if x >= 0):
            f, sp = divmod(pid, S)
            lo, hi = orc.superpatch_bounds(P, S)[sp]
            tok2 += [f * P + j for j in o.kept[f] if lo <= j < hi]
        assert n2 == n
        np.testing.assert_array_equal(k2[:, :, :n], k[:, :, tok2])

    def test_combined_gather_is_the_union_of_the_three_levels(self):
        cfg, o, (k, v) = self._state()
        P, S, kap, F = cfg.tokens_per_frame, cfg.superpatches_per_frame, o.kappa, cfg.frames_per_segment
        # one level at a time it is that level's gather (temporal order, distinct entries)
        frames = np.array([9, 2, 4], np.int32)
        ka, va, na = o.gather(frames)
        kb, vb, nb = o.gather_union(frame_idx=frames, rows_cap=ka.shape[2])
        assert na == nb
        np.testing.assert_array_equal(ka, kb)
        np.testing.assert_array_equal(va, vb)
        pats = np.array([4 * 7 + 3, 4 * 2 + 1, 4 * 7 + 0], np.int32)
        ka, va, na = o.gather_patches(pats)
        kb, vb, nb = o.gather_union(patch_idx=pats, rows_cap=ka.shape[2])
        assert na == nb
        np.testing.assert_array_equal(ka, kb)
        ka, _, na = o.gather(np.arange(2 * F, 3 * F, dtype=np.int32))          # a segment is its frames
        kb, _, nb = o.gather_union(seg_idx=[2], rows_cap=ka.shape[2])
        assert na == nb == F * kap
        np.testing.assert_array_equal(ka, kb)
        # together: every row once, straight from the inputs, in (frame, position) order
        ku, vu, n = o.gather_union(seg_idx=[1, -1], frame_idx=[5, 17, 99], patch_idx=[4 * 5 + 1, 4 * 20 + 2, 4 * 17 + 3, -1])
        want = set()
        for f in list(range(F, 2 * F)) + [5, 17]:
            want.update(f * P + int(j) for j in o.kept[f])
        lo, hi = orc.superpatch_bounds(P, S)[2]
        want.update(20 * P + int(j) for j in o.kept[20] if lo <= j < hi)
        tok = sorted(want)
        assert n == len(tok) == ku.shape[2]
        np.testing.assert_array_equal(ku, k[:, :, tok])
        np.testing.assert_array_equal(vu, v[:, :, tok])
        # a smaller output holds the first rows only, the count still reports the union
        k3, _, n3 = o.gather_union(seg_idx=[1], frame_idx=[5, 17], rows_cap=7)
        assert n3 == (F + 1) * kap and k3.shape[2] == 7                    # frame 5 lies inside segment 1: counted once


# ------------------------------------------------------------ Sec. 3.5, Eq. 9 ----
class TestAttend:
    """Attention of new tokens over [retrieved rows, local rows] at one layer."""

    def _state(self, n_frames=12, const_values=False, dtype="f32"):
        cfg = tiny_cfg(frames_per_segment=4)
        k, v, q = tiny_stream(cfg, n_frames, dtype=dtype, seed=6)
        if const_values:   # every value vector of (layer l, KV head g) is the constant 10 (l + 1) + g + 1
            for l in range(cfg.n_layers):
                for g in range(cfg.n_kv_heads):
                    v[l, g] = 10.0 * (l + 1) + g + 1
        return cfg, run_stream(cfg, k, v, q, 4)

    def test_a_single_visible_key_returns_its_value(self):
        cfg, o = self._state()
        q = rng.standard_normal((1, 4, 16)).astype(np.float32)
        kl = rng.standard_normal((1, 2, 16)).astype(np.float32)
        vl = rng.standard_normal((1, 2, 16)).astype(np.float32)
        out = o.attend(0, q, [-1, -1], kl, vl)
        for h in range(4):
            np.testing.assert_allclose(out[0, h], vl[0, h // 2].astype(np.float64), rtol=0, atol=1e-15)

    def test_no_visible_key_gives_zero(self):
        cfg, o = self._state()
        q = rng.standard_normal((2, 4, 16)).astype(np.float32)
        assert not o.attend(1, q, [-1]).any()

    def test_equal_keys_average_the_values(self):
        cfg, o = self._state()
        q = rng.standard_normal((1, 4, 16)).astype(np.float32)
        kl = np.repeat(rng.standard_normal((1, 2, 16)).astype(np.float32), 5, axis=0)
        vl = rng.standard_normal((5, 2, 16)).astype(np.float32)
        out = o.attend(0, q, [], kl, vl, causal_local=False)
        for h in range(4):
            np.testing.assert_allclose(out[0, h], vl[:, h // 2].astype(np.float64).mean(axis=0), atol=1e-14)

    def test_two_keys_mix_with_the_logistic_of_the_scaled_score_gap(self):
        cfg, o = self._state()
        D = 16
        q = np.zeros((1, 4, D), np.float32)
        q[0, :, 3] = 2.0
        kl = np.zeros((2, 2, D), np.float32)
        kl[0, :, 3], kl[1, :, 3] = 1.5, -0.5           # scores 3/sqrt(D) and -1/sqrt(D)
        vl = np.zeros((2, 2, D), np.float32)
        vl[0, :, 0], vl[1, :, 0] = 1.0, 0.0
        out = o.attend(0, q, [], kl, vl, causal_local=False)
        want = 1.0 / (1.0 + math.exp(-(3.0 - (-1.0)) / math.sqrt(D)))    # 1/sqrt(D) scale: gap 4/4 = 1
        np.testing.assert_allclose(out[0, :, 0], want, atol=1e-15)

    def test_layer_and_grouped_head_of_the_retrieved_rows(self):
        # constant values per (layer, KV head): whatever the weights, the output names the slab read
        cfg, o = self._state(const_values=True)
        q = rng.standard_normal((3, 4, 16)).astype(np.float32)
        for layer in (0, 1):
            out = o.attend(layer, q, [7, 2, -1, 9])
            for h in range(4):
                np.testing.assert_allclose(out[:, h], 10.0 * (layer + 1) + h // 2 + 1, rtol=1e-14)

    def test_matches_library_softmax_over_the_gathered_rows(self):
        import scipy.special
        cfg, o = self._state(dtype="bf16")
        sel = [5, 0, 11, -1, 3]
        ko, vo, n = o.gather(sel, orc.AS_GIVEN)                  # gather is pinned on its own
        q = bf16_bits(rng.standard_normal((2, 4, 16)))
        kl, vl = bf16_bits(rng.standard_normal((3, 2, 16))), bf16_bits(rng.standard_normal((3, 2, 16)))
        out = o.attend(1, q, sel, kl, vl, causal_local=False)
        for h in range(4):
            K = np.concatenate([bf16_value(ko[1, h // 2, :n]), bf16_value(kl[:, h // 2])])
            V = np.concatenate([bf16_value(vo[1, h // 2, :n]), bf16_value(vl[:, h // 2])])
            w = scipy.special.softmax(bf16_value(q[:, h]) @ K.T / 4.0, axis=1)
            np.testing.assert_allclose(out[:, h], w @ V, atol=1e-13)

    def test_order_of_the_retrieved_frames_does_not_matter(self):
        cfg, o = self._state()
        q = rng.standard_normal((2, 4, 16)).astype(np.float32)
        a = o.attend(0, q, [1, 8, 4, -1])
        b = o.attend(0, q, [-1, 4, 1, 8])
        np.testing.assert_allclose(a, b, atol=1e-13)

    def test_causal_mask_over_the_local_rows(self):
        cfg, o = self._state()
        n = 5
        q = rng.standard_normal((n, 4, 16)).astype(np.float32)
        kl = rng.standard_normal((n, 2, 16)).astype(np.float32)
        vl = rng.standard_normal((n, 2, 16)).astype(np.float32)
        out = o.attend(0, q, [], kl, vl)                      # pure self-attention of the local rows
        for h in range(4):                                     # token 0 sees only row 0
            np.testing.assert_allclose(out[0, h], vl[0, h // 2].astype(np.float64), atol=1e-15)
        kl2, vl2 = kl.copy(), vl.copy()
        kl2[3:], vl2[3:] = 7.0, -3.0                           # rows 3, 4 changed: tokens 0..2 must not notice
        out2 = o.attend(0, q, [], kl2, vl2)
        np.testing.assert_array_equal(out[:3], out2[:3])
        assert np.abs(out[3:] - out2[3:]).max() > 1e-3
        free = o.attend(0, q, [], kl2, vl2, causal_local=False)
        assert np.abs(free[:3] - out2[:3]).max() > 1e-3
        # fewer query tokens than local rows: the queries are the LAST rows
        tail = o.attend(0, q[3:], [], kl, vl)
        np.testing.assert_allclose(tail, out[3:], atol=1e-14)

    def test_retrieved_rows_are_visible_to_every_token_and_scores_shift_freely(self):
        cfg, o = self._state()
        q = rng.standard_normal((1, 4, 16)).astype(np.float32)
        kl = rng.standard_normal((1, 2, 16)).astype(np.float32)
        vl = rng.standard_normal((1, 2, 16)).astype(np.float32)
        with_ctx = o.attend(1, q, [2, 6], kl, vl)
        ctx_only = o.attend(1, q, [2, 6])
        # a local key far below every other score drops out: the retrieved part alone remains
        far = kl.copy()
        for g in range(2):
            far[0, g] = -1e4 * q[0, 2 * g] / np.linalg.norm(q[0, 2 * g])
        drop = o.attend(1, q[:, [0, 0, 2, 2]], [2, 6], far, vl)
        np.testing.assert_allclose(drop, o.attend(1, q[:, [0, 0, 2, 2]], [2, 6]), atol=1e-12)
        assert np.abs(with_ctx - ctx_only).max() > 1e-6


class TestPrefillAttend:
    """The prefill of new tokens over [past cache, themselves] that also yields Eq. 1."""

    def _state(self, n_frames=8):
        cfg = tiny_cfg(frames_per_segment=4)
        k, v, q = tiny_stream(cfg, n_frames, seed=9)
        return cfg, run_stream(cfg, k, v, q, 4)

    def test_without_a_past_it_is_the_attention_signal_of_the_frame(self):
        # no retrieved rows, the local rows are exactly the new tokens: Eq. 1 of one frame, which has its own pins
        cfg, o = self._state()
        P = cfg.tokens_per_frame
        k, v, q = tiny_stream(cfg, 1, seed=31)
        ql = np.ascontiguousarray(q.transpose(1, 0, 2))                 # [P][Hq][D]
        kl = np.ascontiguousarray(k[-1].transpose(1, 0, 2))             # [P][Hkv][D]
        vl = np.ascontiguousarray(v[-1].transpose(1, 0, 2))
        for causal in (True, False):
            out, sig = o.prefill_attend(1, ql, [], kl, vl, causal)
            np.testing.assert_allclose(sig, orc.att_signal(q, k[-1], 1, P, causal)[0], rtol=0, atol=1e-14)
            np.testing.assert_array_equal(out, o.attend(1, ql, [], kl, vl, causal))

    def test_equal_keys_closed_form_with_a_past(self):
        # every key the same (retrieved rows replaced by copies would need the store; use older local rows as the
        # past): query i sees n_old + i + 1 equal keys, so new token j receives sum_{i >= j} 1 / (n_old + i + 1)
        cfg, o = self._state()
        n_old, n_q = 5, 4
        q = rng.standard_normal((n_q, 4, 16)).astype(np.float32)
        kl = np.repeat(rng.standard_normal((1, 2, 16)).astype(np.float32), n_old + n_q, axis=0)
        vl = rng.standard_normal((n_old + n_q, 2, 16)).astype(np.float32)
        _, sig = o.prefill_attend(0, q, [], kl, vl, True)
        want = [sum(1.0 / (n_old + i + 1) for i in range(j, n_q)) / n_q for j in range(n_q)]
        np.testing.assert_allclose(sig, want, rtol=0, atol=1e-14)

    def test_what_the_past_absorbs_is_missing_from_the_signal(self):
        cfg, o = self._state()
        n_q = 6
        q = rng.standard_normal((n_q, 4, 16)).astype(np.float32)
        kl = rng.standard_normal((n_q, 2, 16)).astype(np.float32)
        vl = rng.standard_normal((n_q, 2, 16)).astype(np.float32)
        _, alone = o.prefill_attend(1, q, [], kl, vl, True)
        assert alone.sum() == pytest.approx(1.0, abs=1e-14)            # all of every query's mass lies on new tokens
        _, with_past = o.prefill_attend(1, q, [2, 5], kl, vl, True)
        assert 0.0 < with_past.sum() < 1.0 and np.all(with_past <= alone + 1e-15)
        # the mass on the retrieved rows, recomputed with scipy over the gathered rows
        from scipy.special import softmax
        sk, _ = o.store()
        kap = o.kappa
        rows = np.r_[2 * kap:3 * kap, 5 * kap:6 * kap]
        on_new = 0.0
        for h in range(4):
            kk = np.concatenate([sk[1, h // 2][rows].astype(np.float64), kl[:, h // 2].astype(np.float64)])
            for i in range(n_q):
                s = kk[:len(rows) + i + 1] @ q[i, h].astype(np.float64) / 4.0
                on_new += softmax(s)[len(rows):].sum()
        assert with_past.sum() == pytest.approx(on_new / (4 * n_q), abs=1e-13)

    def test_a_new_token_nobody_can_see_receives_nothing_but_its_own_glance(self):
        # causal: the last new token is seen only by itself
        cfg, o = self._state()
        n_q = 3
        q = np.zeros((n_q, 4, 16), np.float32)                         # zero queries: uniform weights
        kl = rng.standard_normal((n_q, 2, 16)).astype(np.float32)
        vl = rng.standard_normal((n_q, 2, 16)).astype(np.float32)
        _, sig = o.prefill_attend(0, q, [], kl, vl, True)
        np.testing.assert_allclose(sig, [(1 + 1 / 2 + 1 / 3) / 3, (1 / 2 + 1 / 3) / 3, (1 / 3) / 3], atol=1e-15)


def test_c_half_runs_clean_under_address_and_undefined_behaviour_sanitizers():
    # every function of mukv_oracle.c on heap blocks of exactly the documented sizes, in an executable
    # instrumented with ASan + UBSan; MUKV_ORACLE_SANITIZE=1 runs all of these pins on a UBSan build too
    assert "ok" in orc.sanitizer_selftest()
