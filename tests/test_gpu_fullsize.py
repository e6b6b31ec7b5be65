"""GPU parity at the full sizes of the five benchmark configurations, in the launch
configuration bench.py times (same chunking, same kernels, same retrieval
parameters).  The oracle is fast enough on the machine's host cores to redo every
frame, so nothing is sampled: every kept index, every stored byte, every block
key, and the retrieval + gather of every question is compared."""
import time

import numpy as np
import pytest
import torch

from mukv_testlib import TOL, gpu_context, np_view, oracle_config, out_err
from oracle import oracle as orc
from paper_2605_22269_amd import binding as mk
from paper_2605_22269_amd import synth

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


BENCH_LAUNCH = dict(batch_chunks=64, overlap_copy=1)   # bench.py's defaults


def run_full(w: synth.Workload, seed: int, oracle_chunk: int = 64, max_questions: int = 1):
    """Streams the workload through the GPU library in w.chunk_frames chunks, gathered and
    overlapped as bench.py does, and through the oracle in oracle_chunk chunks (its results
    do not depend on the chunking).  Inputs of the last two batches are kept alive, as the
    overlapped mode asks."""
    assert oracle_chunk % w.chunk_frames == 0
    gpu = gpu_context(w, max_frames=w.n_frames, max_chunk_frames=w.chunk_frames, max_questions=max_questions,
                      **BENCH_LAUNCH)
    alive = []
    keep_big = 2 * (BENCH_LAUNCH["batch_chunks"] * w.chunk_frames + oracle_chunk - 1) // oracle_chunk + 1
    ref = orc.OracleMuKV(oracle_config(w))
    stream = synth.SynthStream(w, seed, device="cuda")
    P, tol = w.tokens_per_frame, TOL[w.dtype]
    worst = 0.0
    t_orc = 0.0
    done = 0
    while done < w.n_frames:
        n_big = min(oracle_chunk, w.n_frames - done)
        k, v, q = stream.next_chunk(n_big)
        fused_gpu = []
        for f0 in range(0, n_big, w.chunk_frames):
            n = min(w.chunk_frames, n_big - f0)
            sl = slice(f0 * P, (f0 + n) * P)
            # the whole dict is kept: all three signal buffers are written when the batch is launched
            fused_gpu.append(gpu.compress_chunk(k[:, :, sl], v[:, :, sl], q[:, sl], want_signals=True))
        t0 = time.perf_counter()
        so = ref.compress_chunk(np_view(k), np_view(v), q_last=np_view(q))
        t_orc += time.perf_counter() - t0
        alive.append((k, v, q, fused_gpu, so["fused"]))
        done += n_big
        del k, v, q
        if len(alive) > keep_big:       # its batch was flushed at least one batch ago
            _, _, _, fg, fo = alive.pop(0)
            torch.cuda.synchronize()
            worst = max(worst, float(np.abs(torch.cat([x["fused"] for x in fg]).cpu().numpy() - fo).max()))
    gpu.flush()
    torch.cuda.synchronize()
    for _, _, _, fg, fo in alive:
        worst = max(worst, float(np.abs(torch.cat([x["fused"] for x in fg]).cpu().numpy() - fo).max()))
    alive.clear()
    assert worst <= tol, f"fused score error {worst}"
    st = gpu.state()
    torch.cuda.synchronize()
    mism = np.nonzero((st["kept_idx"].cpu().numpy() != ref.kept).any(axis=1))[0]
    assert mism.size == 0, f"kept indices differ in frames {mism[:10]} (margins {st['margin'].cpu().numpy()[mism[:10]]})"
    for name, want in (("rep_frame_k", ref.rep_frame_k), ("rep_frame_v", ref.rep_frame_v),
                       ("rep_patch_k", ref.rep_patch_k), ("rep_patch_v", ref.rep_patch_v),
                       ("rep_seg_k", ref.seg_reps(which="k")), ("rep_seg_v", ref.seg_reps(which="v"))):
        got = st[name].cpu().numpy()
        assert np.abs(got - want).max() <= tol, name
        np.testing.assert_array_equal(got, want.astype(np.float32), err_msg=name)
    np.testing.assert_array_equal(st["cnt_patch"].cpu().numpy(), ref.cnt_patch)
    ok, ov = ref.store()
    kap = ref.kappa
    step = 256 * kap                                    # compare the store in slices of 256 frames
    for r0 in range(0, w.n_frames * kap, step):
        r1 = min(r0 + step, w.n_frames * kap)
        gk, gv = gpu.store_rows(r0, r1)
        np.testing.assert_array_equal(np_view(gk), ok[:, :, r0:r1])
        np.testing.assert_array_equal(np_view(gv), ov[:, :, r0:r1])
    info = {"refined": int(st["refined"].sum()), "min_margin": float(st["margin"].min()), "max_fused_err": worst,
            "oracle_s": t_orc}
    return gpu, ref, info


def check_questions(w, gpu, ref, questions, mode=mk.MUKV_SEMI):
    offs = np.zeros(len(questions) + 1, np.int32)
    offs[1:] = np.cumsum([q.shape[0] for q in questions])
    qt = torch.cat(questions).cuda().contiguous()
    out = gpu.retrieve(qt, torch.from_numpy(offs).cuda(), mode=mode, k_seg=w.k_seg, k_frame=w.k_frame,
                       lambda_frame=w.lambda_frame)
    kg, vg, nt = gpu.gather_kv(out["frame_idx"])
    torch.cuda.synchronize()
    hits = []
    for b, q in enumerate(questions):
        r = ref.retrieve(np_view(q.cpu()), orc.RetrieveParams(mode, w.k_seg, w.k_frame, w.lambda_frame))
        np.testing.assert_array_equal(out["seg_idx"][b].cpu().numpy(), r["seg_idx"])
        np.testing.assert_array_equal(out["frame_idx"][b].cpu().numpy(), r["frame_idx"])
        assert np.abs(out["seg_score"][b].cpu().numpy() - r["seg_score"]).max() <= 1e-5
        assert np.abs(out["frame_score"][b].cpu().numpy() - r["frame_score"]).max() <= 1e-5
        ko, vo, n_tok = ref.gather(r["frame_idx"])
        assert int(nt[b]) == n_tok
        np.testing.assert_array_equal(np_view(kg[b]), ko)
        np.testing.assert_array_equal(np_view(vg[b]), vo)
        hits.append(r["frame_idx"])
    return hits


def check_patch_questions(w, gpu, ref, questions, mode, k_patch=20):
    """Super-patch level of the search (k_g = 20 as the paper's patch level) and its gather."""
    offs = np.zeros(len(questions) + 1, np.int32)
    offs[1:] = np.cumsum([q.shape[0] for q in questions])
    qt = torch.cat(questions).cuda().contiguous()
    out = gpu.retrieve_patches(qt, torch.from_numpy(offs).cuda(), mode=mode, k_seg=w.k_seg, k_patch=k_patch,
                               lambda_patch=w.lambda_frame)
    kg, vg, nt = gpu.gather_patches(out["patch_idx"])
    torch.cuda.synchronize()
    for b, q in enumerate(questions):
        r = ref.retrieve(np_view(q.cpu()), orc.RetrieveParams(mode, w.k_seg, k_patch, w.lambda_frame), level="patch")
        np.testing.assert_array_equal(out["patch_idx"][b].cpu().numpy(), r["frame_idx"])
        assert np.abs(out["patch_score"][b].cpu().numpy() - r["frame_score"]).max() <= 1e-5
        ko, vo, n_tok = ref.gather_patches(r["frame_idx"])
        assert int(nt[b]) == n_tok
        np.testing.assert_array_equal(np_view(kg[b]), ko)
        np.testing.assert_array_equal(np_view(vg[b]), vo)


def check_union(w, gpu, ref, question):
    """Combined gather fed by the two searches: the paper's k_g = 12 segments, 32 frames, 20 super-patches."""
    offs = torch.tensor([0, question.shape[0]], dtype=torch.int32, device="cuda")
    qt = question.cuda().contiguous()
    o1 = gpu.retrieve(qt, offs, mode=mk.MUKV_SEMI, k_seg=12, k_frame=32, lambda_frame=w.lambda_frame)
    o2 = gpu.retrieve_patches(qt, offs, mode=mk.MUKV_SEMI, k_seg=12, k_patch=20, lambda_patch=w.lambda_frame)
    kg, vg, nt = gpu.gather_union(o1["seg_idx"], o1["frame_idx"], o2["patch_idx"])
    torch.cuda.synchronize()
    ko, vo, n = ref.gather_union(o1["seg_idx"][0].cpu().numpy(), o1["frame_idx"][0].cpu().numpy(),
                                 o2["patch_idx"][0].cpu().numpy(), rows_cap=kg.shape[3])
    assert int(nt[0]) == n
    np.testing.assert_array_equal(np_view(kg[0]), ko)
    np.testing.assert_array_equal(np_view(vg[0]), vo)
    return n


def check_decode(w, gpu, ref, hits, layers, n_q=1, n_local=32, seed=0):
    """The step after the path (Eq. 9) at full size: new tokens of every question attend to the kept
    rows of the frames retrieved for it (hits: per-question index lists) plus local rows."""
    B = len(hits)
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, n_q, w.n_q_heads, w.head_dim, generator=g).to(w.torch_dtype)
    kl = torch.randn(B * n_local, w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    vl = torch.randn(B * n_local, w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    lo = (torch.arange(B + 1, dtype=torch.int32) * n_local).cuda()
    idx = torch.tensor(np.asarray(hits), dtype=torch.int32, device="cuda")
    worst = 0.0
    for layer in layers:
        out = gpu.attend(layer, q.cuda(), idx, kl.cuda(), vl.cuda(), lo, True)
        torch.cuda.synchronize()
        got = np_view(out.cpu())
        got = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if got.dtype == np.uint16 else got.astype(np.float64)
        for b in range(B):
            want = ref.attend(layer, np_view(q[b]), hits[b], np_view(kl[b * n_local:(b + 1) * n_local]),
                              np_view(vl[b * n_local:(b + 1) * n_local]), True)
            err = out_err(got[b], want)
            assert err <= (2e-2 if w.dtype == "bf16" else 1e-5), (layer, b, err)
            worst = max(worst, err)
    return worst


def check_prefill(w, gpu, ref, hits, layer, n_q, n_old=0, seed=0):
    """The step before the path at full size: the prefill of n_q new tokens of one question over the kept rows
    of the frames in hits plus n_old older local rows; output and received-attention signal (Eq. 1)."""
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(1, n_q, w.n_q_heads, w.head_dim, generator=g).to(w.torch_dtype)
    kl = torch.randn(n_old + n_q, w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    vl = torch.randn(n_old + n_q, w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    lo = torch.tensor([0, n_old + n_q], dtype=torch.int32).cuda()
    idx = torch.tensor([list(hits)], dtype=torch.int32, device="cuda")
    out, sig = gpu.prefill_attend(layer, q.cuda(), idx, kl.cuda(), vl.cuda(), lo, True)
    torch.cuda.synchronize()
    got = np_view(out.cpu())
    got = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if got.dtype == np.uint16 else got.astype(np.float64)
    want, want_sig = ref.prefill_attend(layer, np_view(q[0]), list(hits), np_view(kl), np_view(vl), True)
    err = out_err(got[0], want)
    err_sig = float(np.abs(sig[0].cpu().numpy().astype(np.float64) - want_sig).max())
    assert err <= (2e-2 if w.dtype == "bf16" else 1e-5), err
    assert err_sig <= 1e-6, err_sig
    return err, err_sig


def test_config2_7b_256_frames():
    w = W["7b"]
    gpu, ref, info = run_full(w, seed=1002)
    print("7b:", info)
    for mode in (mk.MUKV_SEMI, mk.MUKV_HIER, mk.MUKV_PARALLEL):
        hits = check_questions(w, gpu, ref, [synth.random_question(w, w.question_tokens, 77)], mode)
    print("7b: decode attention over the retrieved rows, worst error", check_decode(w, gpu, ref, hits, (0, w.n_layers - 1), seed=5))
    print("7b: prefill of one frame / of a chunk of 8 frames over the retrieved rows, (output, signal) errors",
          check_prefill(w, gpu, ref, hits[0], w.n_layers - 1, w.tokens_per_frame, n_old=40, seed=8),
          check_prefill(w, gpu, ref, hits[0], 0, 8 * w.tokens_per_frame, seed=9))
    gpu.close()


def test_config3_and_4_one_hour_stream():
    w = W["hour"]
    wq = W["retrieval"]
    gpu, ref, info = run_full(w, seed=1003, max_questions=wq.n_questions)
    print("hour:", info)
    # config 3: one 32-token question, all three retrieval modes
    for mode in (mk.MUKV_SEMI, mk.MUKV_HIER, mk.MUKV_PARALLEL):
        check_questions(w, gpu, ref, [synth.random_question(w, w.question_tokens, 78)], mode)
        check_patch_questions(w, gpu, ref, [synth.random_question(w, w.question_tokens, 78)], mode)   # 14 400 keys
    print("hour: combined gather of 12 segments + 32 frames + 20 super-patches:",
          check_union(w, gpu, ref, synth.random_question(w, w.question_tokens, 78)), "tokens")
    # config 4: 64 concurrent questions of 16..64 tokens with planted target frames (planted from
    # the ORACLE's frame keys), one batched retrieve + gather
    lens = synth.question_lengths(wq.n_questions, 16, wq.question_tokens, 79)
    g = torch.Generator().manual_seed(80)
    qs, targets = [], []
    for i, n in enumerate(lens):
        tgt = torch.randint(0, w.n_frames, (4,), generator=g)
        targets.append(set(tgt.tolist()))
        qs.append(synth.planted_question(wq, torch.from_numpy(ref.rep_frame_k[tgt.numpy()]), n, 81 + i))
    hits = check_questions(wq, gpu, ref, qs)
    print("retrieval-heavy: decode attention of 64 questions, worst error",
          check_decode(wq, gpu, ref, hits, (w.n_layers - 1,), seed=6),
          "; 3 new tokens of 8 questions:", check_decode(wq, gpu, ref, hits[:8], (0,), n_q=3, seed=7))
    check_patch_questions(wq, gpu, ref, qs[:20], mk.MUKV_SEMI)
    found = sum(len(t & set(int(x) for x in h)) for t, h in zip(targets, hits))
    total = sum(len(t) for t in targets)
    print(f"retrieval-heavy: {found}/{total} planted frames retrieved")
    assert found >= 0.9 * total
    gpu.close()


def test_config5_72b_shape():
    w = W["72b"]
    gpu, ref, info = run_full(w, seed=1005, oracle_chunk=64)
    print("72b:", info)
    for mode in (mk.MUKV_SEMI, mk.MUKV_HIER, mk.MUKV_PARALLEL):
        check_questions(w, gpu, ref, [synth.random_question(w, w.question_tokens, 82)], mode)
        check_patch_questions(w, gpu, ref, [synth.random_question(w, w.question_tokens, 82)], mode)
    gpu.close()
