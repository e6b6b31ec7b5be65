#!/usr/bin/env python3
"""Benchmark of the MuKV hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic stream that is
already resident in HBM: mukv_compress_chunk for every chunk of the stream
(attention + frequency signals, fusion, per-frame keep, all-layer KV compaction,
block keys), then mukv_retrieve + mukv_gather_kv for the workload's questions.
Prints ONE JSON line: throughput of the whole step, per-kernel times from HIP
events, the HBM roofline of the dominant kernel, and the CPU oracle's rate on
a sample of the same stream.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload hour] [--chunk-frames 8]
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
# HBM bytes actually moved per algorithmic byte, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# on the 1-hour shape, calibrated with a plain copy kernel.  The figures live in ONE place: lines
# "traffic_ratio <kernel> <moved MB> / <algorithmic MB>" of the summary of those runs under profiles/.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "traffic_probe_hbm_counters.md")


def traffic_ratios():
    out = {}
    try:
        for line in open(TRAFFIC_SUMMARY):
            t = line.split()
            if len(t) >= 5 and t[0] == "traffic_ratio" and t[3] == "/":
                out[t[1]] = float(t[2]) / float(t[4])
    except (OSError, ValueError):
        pass
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="hour", choices=["tiny", "7b", "hour", "retrieval", "72b"])
    ap.add_argument("--chunk-frames", type=int, default=0, help="frames per mukv_compress_chunk call (0: workload's)")
    ap.add_argument("--batch-chunks", type=int, default=64,
                    help="chunks the library gathers before it launches their kernels together (1: launch per chunk)")
    ap.add_argument("--frames", type=int, default=0, help="override the stream length (debugging)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--overlap-copy", type=int, default=1, choices=(0, 1),
                    help="1: the copy of a batch's kept rows shares a launch with the next batch's frequency "
                         "kernel (mukv_config.overlap_copy; the whole stream is resident, so inputs outlive the copies)")
    ap.add_argument("--freq-axis", default="feature", choices=["feature", "token"],
                    help="axis of the transform in the frequency indicator (mukv_config.freq_axis); "
                         "the default is the reading the build takes, 'token' the other one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--core-only", action="store_true",
                    help="print the step's own figures and stop (no extras, no other configurations, no oracle timing)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short passes over the 7B-class and 72B-class streams that the default run appends")
    ap.add_argument("--cpu-sample-frames", type=int, default=2048)
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="size in MiB of the plain-copy reference run (default 1024)")
    ap.add_argument("--seed", type=int, default=2605)
    return ap.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (asked for --gpus {a.gpus}); "
              "there is no multi-GPU path to measure.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_22269_amd import binding as mk
    from paper_2605_22269_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda", 0)
    w = synth.WORKLOADS[a.workload]
    if a.frames:
        w = w.scaled(n_frames=a.frames)
    chunk = a.chunk_frames or w.chunk_frames
    L, Hq, Hkv, D, P = w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.tokens_per_frame
    n_frames = w.n_frames
    n_chunks = (n_frames + chunk - 1) // chunk
    B = w.n_questions
    esz = w.elem_bytes

    # ---- synthetic stream, resident in HBM before anything is timed ------------------------
    t_gen = time.perf_counter()
    stream = synth.SynthStream(w, a.seed, device=dev)
    ks, vs, qs = [], [], []
    K = torch.empty(n_chunks, L, Hkv, chunk * P, D, dtype=w.torch_dtype, device=dev)
    V = torch.empty_like(K)
    Q = torch.empty(n_chunks, Hq, chunk * P, D, dtype=w.torch_dtype, device=dev)
    for c in range(n_chunks):
        n = min(chunk, n_frames - c * chunk)
        k, v, q = stream.next_chunk(n)
        K[c, :, :, : n * P], V[c, :, :, : n * P], Q[c, :, : n * P] = k, v, q
        ks.append(K[c, :, :, : n * P])
        vs.append(V[c, :, :, : n * P])
        qs.append(Q[c, :, : n * P])
    del k, v, q
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    ctx = mk.MuKV(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, tokens_per_frame=P,
                  frames_per_segment=w.frames_per_segment, superpatches_per_frame=w.superpatches_per_frame,
                  dtype=w.torch_dtype, keep_ratio=w.keep_ratio, alpha=w.alpha, max_frames=n_frames,
                  max_chunk_frames=chunk, max_questions=max(B, 64), batch_chunks=a.batch_chunks, overlap_copy=a.overlap_copy,
                  freq_axis=mk.MUKV_FREQ_TOKEN if a.freq_axis == "token" else mk.MUKV_FREQ_FEATURE)
    kappa = ctx.kappa

    # questions: random for the single-question workloads, planted targets for the batched one
    if B == 1:
        lens = [w.question_tokens]
    else:
        lens = synth.question_lengths(B, 16, w.question_tokens, a.seed + 1)
    q_list = [synth.random_question(w, n, a.seed + 10 + i, device=dev) for i, n in enumerate(lens)]

    def compress_all():
        ctx.reset()
        for c in range(n_chunks):
            ctx.compress_chunk(ks[c], vs[c], qs[c])
        ctx.flush()

    if B > 1:  # plant 4 target frames per question, using the cache's own frame keys
        compress_all()
        reps = ctx.state()["rep_frame_k"]
        g = torch.Generator().manual_seed(a.seed + 2)
        q_list = []
        for i, n in enumerate(lens):
            tgt = torch.randint(0, n_frames, (4,), generator=g)
            q_list.append(synth.planted_question(w, reps[tgt.to(dev)], n, a.seed + 10 + i, device=dev))
    q_tokens = torch.cat(q_list).contiguous()
    offs = torch.zeros(B + 1, dtype=torch.int32)
    offs[1:] = torch.cumsum(torch.tensor(lens), 0)
    offs = offs.to(dev)
    r_out = {
        "seg_idx": torch.empty(B, w.k_seg, dtype=torch.int32, device=dev),
        "seg_score": torch.empty(B, w.k_seg, dtype=torch.float32, device=dev),
        "frame_idx": torch.empty(B, w.k_frame, dtype=torch.int32, device=dev),
        "frame_score": torch.empty(B, w.k_frame, dtype=torch.float32, device=dev),
    }
    g_shape = (B, L, Hkv, w.k_frame * kappa, D)
    g_out = (torch.empty(g_shape, dtype=w.torch_dtype, device=dev), torch.empty(g_shape, dtype=w.torch_dtype, device=dev),
             torch.empty(B, dtype=torch.int32, device=dev))

    def retrieve_all():
        ctx.retrieve(q_tokens, offs, mode=mk.MUKV_SEMI, k_seg=w.k_seg, k_frame=w.k_frame,
                     lambda_frame=w.lambda_frame, out=r_out)
        ctx.gather_kv(r_out["frame_idx"], out=g_out)

    def step_eager():
        compress_all()
        retrieve_all()

    # ---- launch mode: replay one HIP graph per step, or eager launches --------------------
    step_eager()
    torch.cuda.synchronize()
    launch = "eager"
    step = step_eager
    if not a.no_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step_eager()
            torch.cuda.synchronize()
            step = graph.replay
            launch = "hipgraph"
        except Exception as e:  # capture not possible: stay eager, and say so
            print(f"bench.py: graph capture failed ({e!r}); timing eager launches", file=sys.stderr)
            torch.cuda.synchronize()

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    tokens = n_frames * P
    value = tokens / (ms_per_step * 1e-3)

    # ---- sub-phase timings with HIP events on the launch stream ---------------------------
    def timed(fn, reps):
        out = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            out.append(e0.elapsed_time(e1))
        return statistics.median(out)

    compress_ms = timed(compress_all, 3)
    retrieve_ms = timed(retrieve_all, 20)

    # ---- per-kernel durations: the library brackets every launch with HIP events ----------
    mk.mukv_profile_begin(ctx.h)
    step_eager()
    prof = mk.mukv_profile_end(ctx.h)
    per_kernel = {n: (p["ms"] / p["launches"] * 1e3 if p["launches"] else None) for n, p in prof.items()}  # us

    b_tok = 2 * Hkv * D * esz                      # K+V bytes of one token in one layer
    copy_frame = 2 * kappa * L * b_tok             # kept rows of one frame, read + written
    freq_frame = P * Hkv * D * esz                 # scoring-layer keys of one frame, read once
    # frames per batch: batch_chunks chunks each
    batches, left = [], n_chunks
    while left:
        batches.append(min(a.batch_chunks, left))
        left -= batches[-1]
    batches = [min(b * chunk, n_frames - sum(batches[:i]) * chunk) for i, b in enumerate(batches)]
    att_frame = P * D * esz * (Hq + Hkv)           # queries and keys of the scoring layer, read once
    chain_ok = [n * Hq >= 1792 for n in batches]    # batches the one-launch chain takes (the library's own rule)
    if a.overlap_copy and prof["chain"]["launches"]:
        # ONE launch per batch: the rows of batch i-2 copied, Eq. 2-3 and Eq. 1 of batch i
        dom, dom_kernel = "chain", "chain_kernel"
        idx = [i for i in range(len(batches)) if chain_ok[i]]
        assert prof[dom]["launches"] == len(idx)
        dom_bytes = sum((copy_frame * batches[i - 2] if i >= 2 else 0) + att_frame * batches[i] for i in idx) / len(idx)
    elif a.overlap_copy and prof["copy_freq"]["launches"]:
        # the launch that copies batch i-2's rows and computes batch i's frequency signal
        dom, dom_kernel = "copy_freq", "copy_freq_kernel"
        assert prof[dom]["launches"] == len(batches) - 2
        dom_bytes = sum(copy_frame * batches[i - 2] + freq_frame * batches[i] for i in range(2, len(batches))) / (len(batches) - 2)
    else:
        dom, dom_kernel = "compact", "compact_kernel"
        dom_bytes = copy_frame * n_frames / prof[dom]["launches"]
    dom_us = per_kernel[dom]
    dom_gbs = dom_bytes / (dom_us * 1e-6) / 1e9
    gather_bytes = 2 * B * w.k_frame * kappa * L * b_tok
    gather_us = per_kernel["gather"]
    ratios = traffic_ratios()
    gather_gbs = gather_bytes / (gather_us * 1e-6) / 1e9
    # whole-path algorithmic bytes: signals' inputs + kept rows in and out
    path_bytes_frame = P * D * esz * (Hq + Hkv) + 2 * kappa * L * b_tok
    # over the timed step (which also holds the retrieval and the gather): the eager pass issues its
    # calls one by one from Python and is bound by the host, not by the device
    path_gbs = path_bytes_frame * n_frames / (ms_per_step * 1e-3) / 1e9

    res = {
        "metric": "visual tokens compressed/s + retrieve latency per question (ms), % HBM peak",
        "value": value,
        "unit": "visual tokens/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {n_frames} frames x {P} tokens, L={L} Hq={Hq} Hkv={Hkv} D={D} {w.dtype}, "
                               f"chunks of {chunk} frames, F={w.frames_per_segment}, keep {kappa}/{P}, "
                               f"{B} question(s), top-{w.k_seg} segments / top-{w.k_frame} frames",
                   "launch": launch, "chunk_frames": chunk, "n_chunks": n_chunks,
                   "batch_chunks": a.batch_chunks, "overlap_copy": a.overlap_copy, "freq_axis": a.freq_axis},
        "compress_ms_per_stream_eager_calls": compress_ms,
        "compress_tokens_per_s_eager_calls": tokens / (compress_ms * 1e-3),
        "retrieve_gather_ms_per_batch": retrieve_ms,
        "retrieve_gather_ms_per_question": retrieve_ms / B,
        "path_hbm": {"algorithmic_bytes_per_token": path_bytes_frame / P, "achieved_GBs": path_gbs,
                     "frac_of_peak": path_gbs / HBM_PEAK_GBS, "over": "ms_per_step"},
        "kernel_us": per_kernel,
        "roofline": {"kernel": dom_kernel, "bound": "hbm", "achieved": dom_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS,
                     "traffic": dom_bytes * ratios[dom] if dom in ratios else None,
                     "bytes_per_launch": dom_bytes, "us_per_launch": dom_us},
        "roofline_gather": {"kernel": "gather_kv_kernel", "bound": "hbm", "achieved": gather_gbs, "peak": HBM_PEAK_GBS,
                            "unit": "GB/s", "frac": gather_gbs / HBM_PEAK_GBS,
                            "traffic": gather_bytes * ratios["gather"] if "gather" in ratios else None,
                            "bytes_per_launch": gather_bytes, "us_per_launch": gather_us},
        "setup_s": {"generate_stream": t_gen},
        # the paper's device-independent proxies (Sec. 4.1): tokens held in the cache, tokens handed to the LLM
        "memory_tokens": n_frames * kappa,
        "inference_tokens_per_question": w.k_frame * kappa,
        # context only, not comparable: end to end including the LLM's answer decoding
        "paper_context": {"source": "real-deployment table of the paper (Sec. 4)", "hardware": "1x NVIDIA A5000 24 GB",
                          "seconds_per_question_incl_llm_decode": {"ReKV": 0.92, "MuKV uncompressed": 0.72,
                                                                   "MuKV compress 2/3 (default)": 0.65,
                                                                   "MuKV compress 3/4": 0.59},
                          "cache_GB_per_hour_of_video": {"ReKV": 4.00, "MuKV compress 2/3": 1.23},
                          "note": "the paper reports no compression throughput and no retrieval or KV-loading "
                                  "latency in isolation, hence vs_baseline is null"},
    }

    if a.core_only:
        ctx.close()
        print(json.dumps(res))
        return

    # ---- the same cache under 64 concurrent questions of 16..64 tokens (one batched call each) --
    if B == 1:
        Bq = 64
        lens_q = synth.question_lengths(Bq, 16, 64, a.seed + 3)
        qt64 = torch.cat([synth.random_question(w, n, a.seed + 100 + i, device=dev) for i, n in enumerate(lens_q)]).contiguous()
        offs64 = torch.zeros(Bq + 1, dtype=torch.int32)
        offs64[1:] = torch.cumsum(torch.tensor(lens_q), 0)
        offs64 = offs64.to(dev)
        r64 = {"seg_idx": torch.empty(Bq, w.k_seg, dtype=torch.int32, device=dev),
               "seg_score": torch.empty(Bq, w.k_seg, dtype=torch.float32, device=dev),
               "frame_idx": torch.empty(Bq, w.k_frame, dtype=torch.int32, device=dev),
               "frame_score": torch.empty(Bq, w.k_frame, dtype=torch.float32, device=dev)}
        shape64 = (Bq, L, Hkv, w.k_frame * kappa, D)
        g64 = (torch.empty(shape64, dtype=w.torch_dtype, device=dev), torch.empty(shape64, dtype=w.torch_dtype, device=dev),
               torch.empty(Bq, dtype=torch.int32, device=dev))

        def retrieve_64():
            ctx.retrieve(qt64, offs64, mode=mk.MUKV_SEMI, k_seg=w.k_seg, k_frame=w.k_frame,
                         lambda_frame=w.lambda_frame, out=r64)
            ctx.gather_kv(r64["frame_idx"], out=g64)

        retrieve_64()
        ms64 = timed(retrieve_64, 10)
        res["retrieve_gather_64_questions"] = {
            "ms_per_batch": ms64, "ms_per_question": ms64 / Bq,
            "gather_bytes": Bq * gather_bytes, "path_GBs": Bq * gather_bytes / (ms64 * 1e-3) / 1e9}
        del g64

        # ---- the step after the path (Eq. 9): one new token per question attends to the kept rows of
        # its retrieved frames, read in place, plus 32 local rows; one call per layer, all L layers ----
        n_loc = 32
        gen = torch.Generator(device=dev).manual_seed(a.seed + 7)
        q_dec = torch.randn(Bq, 1, Hq, D, generator=gen, device=dev).to(w.torch_dtype)
        kl = torch.randn(Bq * n_loc, Hkv, D, generator=gen, device=dev).to(w.torch_dtype)
        vl = torch.randn(Bq * n_loc, Hkv, D, generator=gen, device=dev).to(w.torch_dtype)
        lo = (torch.arange(Bq + 1, dtype=torch.int32) * n_loc).to(dev)
        o_dec = torch.empty_like(q_dec)
        rows_q = w.k_frame * kappa + n_loc
        res["decode_attention"] = {"new_tokens_per_question": 1, "retrieved_rows": w.k_frame * kappa, "local_rows": n_loc,
                                   "layers": L}
        for nb in (Bq, 1):
            def decode_layers(nb=nb):
                for layer in range(L):
                    ctx.attend(layer, q_dec[:nb], r64["frame_idx"][:nb], kl[:nb * n_loc], vl[:nb * n_loc], lo[:nb + 1],
                               True, out=o_dec[:nb])
            decode_layers()
            dms_eager = timed(decode_layers, 10)
            dms, how = dms_eager, "eager"
            if not a.no_graph:      # a serving loop would replay the decode step as one graph
                try:
                    torch.cuda.synchronize()
                    dgraph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(dgraph):
                        decode_layers()
                    torch.cuda.synchronize()
                    dgraph.replay()
                    dms, how = timed(dgraph.replay, 10), "hipgraph"
                except Exception as e:
                    print(f"bench.py: decode graph capture failed ({e}); eager timing kept", file=sys.stderr)
            kv_bytes = nb * rows_q * b_tok                      # K and V rows of one layer, read once
            res["decode_attention"][f"{nb}_questions"] = {
                "launch": how, "ms_all_layers": dms, "us_per_layer_call": dms / L * 1e3, "ms_all_layers_eager": dms_eager,
                "kv_bytes_per_layer_call": kv_bytes, "GBs": kv_bytes * L / (dms * 1e-3) / 1e9}

    # ---- the super-patch level of the search on the same cache: one question, k_g = 20 --------
    p_out = {"patch_idx": torch.empty(B, 20, dtype=torch.int32, device=dev),
             "patch_score": torch.empty(B, 20, dtype=torch.float32, device=dev)}
    pshape = (B, L, Hkv, 20 * ctx.patch_cap, D)
    pg_out = (torch.empty(pshape, dtype=w.torch_dtype, device=dev), torch.empty(pshape, dtype=w.torch_dtype, device=dev),
              torch.empty(B, dtype=torch.int32, device=dev))

    def retrieve_patches():
        ctx.retrieve_patches(q_tokens, offs, mode=mk.MUKV_SEMI, k_seg=w.k_seg, k_patch=20, lambda_patch=w.lambda_frame,
                             out=p_out)
        ctx.gather_patches(p_out["patch_idx"], out=pg_out)

    retrieve_patches()
    pms = timed(retrieve_patches, 20)
    torch.cuda.synchronize()
    # ---- combined gather over the three levels with the paper's k_g = 12 / 32 / 20 ------------
    u_seg = {"seg_idx": torch.empty(B, 12, dtype=torch.int32, device=dev), "seg_score": None,
             "frame_idx": torch.empty(B, w.k_frame, dtype=torch.int32, device=dev), "frame_score": None}
    u_cap = (12 * w.frames_per_segment + w.k_frame) * kappa + 20 * ctx.patch_cap
    ushape = (B, L, Hkv, u_cap, D)
    ug_out = (torch.empty(ushape, dtype=w.torch_dtype, device=dev), torch.empty(ushape, dtype=w.torch_dtype, device=dev),
              torch.empty(B, dtype=torch.int32, device=dev))

    def retrieve_union():
        mk.mukv_retrieve(ctx.h, q_tokens.data_ptr(), offs.data_ptr(), B,
                         mk.mukv_retrieve_params(mk.MUKV_SEMI, 12, w.k_frame, 0, -1, 0, w.lambda_frame),
                         u_seg["seg_idx"].data_ptr(), None, u_seg["frame_idx"].data_ptr(), None,
                         torch.cuda.current_stream().cuda_stream)
        ctx.retrieve_patches(q_tokens, offs, mode=mk.MUKV_SEMI, k_seg=12, k_patch=20, lambda_patch=w.lambda_frame, out=p_out)
        ctx.gather_union(u_seg["seg_idx"], u_seg["frame_idx"], p_out["patch_idx"], rows_cap=u_cap, out=ug_out)

    retrieve_union()
    ums = timed(retrieve_union, 20)
    torch.cuda.synchronize()
    u_tok = int(ug_out[2][0])
    res["retrieve_gather_three_levels"] = {"k_seg": 12, "k_frame": w.k_frame, "k_patch": 20, "ms_per_batch": ums,
                                           "tokens_gathered_q0": u_tok,
                                           "gather_bytes_q0": 2 * u_tok * L * b_tok}
    del ug_out

    # ---- three independently compressed stores (Sec. 3.3, Sec. 4.1): segment units of 4 frames (rho 0.8,
    # alpha 0.8), the middle frame of each (0.1, 0.7) and that frame's 4 super-patches (0.1, 0.5), each a context
    # of its own fed from the same resident stream with the attention signal handed over; the question ranks the
    # segment store (k = 12), whose global query reranks the frame (k = 32) and patch (k = 20) stores, and one
    # gather packs the 12 * 627 + 32 * 19 + 20 * 4 = 8212 kept rows in temporal order ----
    if a.workload == "hour" and not a.frames and chunk % 4 == 0 and P % 4 == 0:
        Fs, Ts = 4, n_frames // 4
        specs = [(Fs * P, 0.8, 0.8, Ts, chunk // Fs), (P, 0.1, 0.7, Ts, 1), (P // 4, 0.1, 0.5, Ts * 4, 4)]
        stores = [mk.MuKV(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, tokens_per_frame=u, frames_per_segment=1,
                          superpatches_per_frame=1, dtype=w.torch_dtype, keep_ratio=rho, alpha=al, max_frames=nu,
                          max_chunk_frames=mc, max_questions=B, batch_chunks=1, overlap_copy=0)
                  for u, rho, al, nu, mc in specs]
        sig = [synth.handed_over_attention(nu, u, a.seed + 70 + i, tie_fraction=0.0).to(dev) for i, (u, _, _, nu, _) in enumerate(specs)]
        per = chunk // Fs  # time steps per chunk of the stream
        for c in range(n_chunks):
            stores[0].compress_chunk(ks[c], vs[c], None, att_signal=sig[0][c * per:(c + 1) * per])
            for j in range(per):
                t, lo = c * per + j, (j * Fs + Fs // 2) * P
                kf, vf = ks[c][:, :, lo:lo + P], vs[c][:, :, lo:lo + P]
                stores[1].compress_chunk(kf, vf, None, att_signal=sig[1][t:t + 1])
                stores[2].compress_chunk(kf, vf, None, att_signal=sig[2][4 * t:4 * t + 4])
        for st_ in stores:
            st_.flush()
        torch.cuda.synchronize()
        kap3 = [st_.kappa for st_ in stores]
        k3 = [12, 32, 20]
        cap3 = sum(k * c for k, c in zip(k3, kap3))

        def three_stores():
            g0 = stores[0].retrieve_units(q_tokens, offs, k3[0], want_g=True)
            g1 = stores[1].retrieve_units(q_tokens, offs, k3[1], 0.3, g_in=g0["g"])
            g2 = stores[2].retrieve_units(q_tokens, offs, k3[2], 0.3, g_in=g0["g"])
            return mk.gather_multi(stores, [g0["idx"], g1["idx"], g2["idx"]], [1, 1, 4], cap3)

        out3 = three_stores()
        t3 = timed(three_stores, 20)
        torch.cuda.synchronize()
        n3 = int(out3[2][0])
        res["retrieve_gather_three_stores"] = {"units": [sp[3] for sp in specs], "unit_tokens": [sp[0] for sp in specs],
                                               "kept_per_unit": kap3, "k": k3, "ms_per_batch": t3, "launch": "eager calls",
                                               "tokens_gathered_q0": n3, "gather_bytes_q0": 2 * n3 * L * b_tok,
                                               "gather_GBs_over_whole_call": 2 * n3 * L * b_tok / (t3 * 1e-3) / 1e9}
        del out3, stores, sig

    res["retrieve_gather_super_patches"] = {"k_patch": 20, "keys_scored": n_frames * w.superpatches_per_frame,
                                            "ms_per_batch": pms, "ms_per_question": pms / B,
                                            "tokens_gathered_q0": int(pg_out[2][0])}

    # ---- what a plain copy reaches on this machine: the library's 16-byte streaming copy on 1 GiB ----
    nb = (a.calibrate_copy_mib or 1024) << 20
    src = torch.empty(nb, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    cur = torch.cuda.current_stream().cuda_stream
    mk.mukv_plain_copy(dst.data_ptr(), src.data_ptr(), nb, cur)
    copy_ms = timed(lambda: mk.mukv_plain_copy(dst.data_ptr(), src.data_ptr(), nb, cur), 10)
    res["plain_copy"] = {"bytes_read_plus_written": 2 * nb, "ms": copy_ms, "GBs": 2 * nb / (copy_ms * 1e-3) / 1e9,
                         "frac_of_peak": 2 * nb / (copy_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del src, dst

    # ---- the same kernels fed by single calls of 512 frames (no gathering of small chunks) -----
    if a.workload == "hour" and not a.frames:
        nbig = 512
        kb = torch.cat([ks[c] for c in range(nbig // chunk)], dim=2)
        vb = torch.cat([vs[c] for c in range(nbig // chunk)], dim=2)
        qb = torch.cat([qs[c] for c in range(nbig // chunk)], dim=1)
        big = mk.MuKV(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, tokens_per_frame=P,
                      frames_per_segment=w.frames_per_segment, superpatches_per_frame=w.superpatches_per_frame,
                      dtype=w.torch_dtype, keep_ratio=w.keep_ratio, alpha=w.alpha, max_frames=7 * nbig,
                      max_chunk_frames=nbig, max_questions=1, batch_chunks=1, overlap_copy=a.overlap_copy)

        def big_calls():
            big.reset()
            for _ in range(7):
                big.compress_chunk(kb, vb, qb)
            big.flush()

        big_calls()
        big_ms = timed(big_calls, 3)
        res["compress_single_calls_of_512_frames"] = {"calls": 7, "ms": big_ms,
                                                      "tokens_per_s": 7 * nbig * P / (big_ms * 1e-3)}
        big.close()

        # ---- the coarsest granularity of Sec. 3.3: a segment of 32 frames ranked as ONE unit of Eq. 4,
        # 80 % of its tokens kept, alpha = 0.8, its frames as super-patches, the attention signal handed
        # over; the same 512 frames as 16 units per call, 7 calls ----
        seg_P, seg_units = 32 * P, nbig // 32
        seg = mk.MuKV(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, tokens_per_frame=seg_P,
                      frames_per_segment=1, superpatches_per_frame=32, dtype=w.torch_dtype, keep_ratio=0.8, alpha=0.8,
                      max_frames=7 * seg_units, max_chunk_frames=seg_units, max_questions=1, batch_chunks=1,
                      overlap_copy=a.overlap_copy)
        att_u = synth.handed_over_attention(seg_units, seg_P, a.seed + 5, tie_fraction=0.0).to(dev)

        def seg_calls():
            seg.reset()
            for _ in range(7):
                seg.compress_chunk(kb, vb, None, att_signal=att_u)
            seg.flush()

        seg_calls()
        seg_ms = timed(seg_calls, 3)
        mk.mukv_profile_begin(seg.h)
        seg_calls()
        seg_prof = mk.mukv_profile_end(seg.h)
        seg_tok = 7 * nbig * P
        seg_bytes = 2 * seg.kappa * L * b_tok / seg_P + Hkv * D * esz + 4   # per token: kept rows in and out, keys, the signal
        res["compress_segments_as_units"] = {
            "unit_tokens": seg_P, "kept_per_unit": seg.kappa, "units_per_call": seg_units, "calls": 7, "ms": seg_ms,
            "tokens_per_s": seg_tok / (seg_ms * 1e-3), "algorithmic_bytes_per_token": seg_bytes,
            "achieved_GBs": seg_bytes * seg_tok / (seg_ms * 1e-3) / 1e9,
            "frac_of_peak": seg_bytes * seg_tok / (seg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "refined_units": int(seg.state()["refined"].sum()),
            "kernel_us": {n: p["ms"] / p["launches"] * 1e3 for n, p in seg_prof.items() if p["launches"]}}
        seg.close()
        del kb, vb, qb, att_u

    # ---- the step before the path (Sec. 3.2 / Eq. 1): the prefill of a frame's, or a chunk's, new tokens at one
    # layer over [kept rows of the 32 retrieved frames, the new tokens themselves], which also emits the attention
    # each new token receives -- the att_signal of mukv_compress_chunk with no second pass over Q and K ----
    if a.workload == "hour" and not a.frames:
        res["prefill_attention"] = {"retrieved_rows": w.k_frame * kappa, "layers_timed": 1}
        for n_new in (1, chunk):
            n_q = n_new * P
            q_new = qs[0][:, :n_q].transpose(0, 1).contiguous()[None]          # [1][n_q][Hq][D]
            k_new = ks[0][L - 1][:, :n_q].transpose(0, 1).contiguous()         # [n_q][Hkv][D]
            v_new = vs[0][L - 1][:, :n_q].transpose(0, 1).contiguous()
            lo_new = torch.tensor([0, n_q], dtype=torch.int32, device=dev)
            ws = torch.empty(mk.mukv_prefill_workspace_size(ctx.h, n_q, w.k_frame, 1), dtype=torch.uint8, device=dev)
            o_new, s_new = torch.empty_like(q_new), torch.empty(1, n_q, dtype=torch.float32, device=dev)

            def prefill_layer():
                ctx.prefill_attend(L - 1, q_new, r_out["frame_idx"][:1], k_new, v_new, lo_new, True, out=o_new,
                                   signal=s_new, workspace=ws)

            prefill_layer()
            torch.cuda.synchronize()
            p_us, how = timed(prefill_layer, 10) * 1e3, "eager"
            if not a.no_graph:
                try:
                    pgraph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(pgraph):
                        for _ in range(8):
                            prefill_layer()
                    torch.cuda.synchronize()
                    pgraph.replay()
                    p_us, how = timed(pgraph.replay, 10) * 1e3 / 8, "hipgraph (8 calls per replay)"
                except Exception as e:
                    print(f"bench.py: capture of the prefill call failed ({e}); eager timing kept", file=sys.stderr)
            rows_ret = w.k_frame * kappa
            flop = 2 * 2 * Hq * D * (n_q * rows_ret + n_q * (n_q + 1) / 2)        # QK^T and PV under the causal mask
            res["prefill_attention"][f"{n_q}_new_tokens"] = {
                "launch": how, "us_per_layer_call": p_us, "workspace_MB": ws.numel() / 1e6,
                "roofline": {"bound": "mfma", "achieved": flop / (p_us * 1e-6) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                             "frac": flop / (p_us * 1e-6) / 1e12 / 2500.0, "flop_per_call": flop}}
            del ws, o_new, s_new, q_new, k_new, v_new

    # ---- the attention signal handed over by the caller (the paper takes it from the prefill that
    # produced the KV, at no extra cost): the same stream, Eq. 1 skipped, Q not read --
    if a.workload == "hour" and not a.frames:
        ctx.reset()
        att_sigs = []
        for c in range(n_chunks):
            att_sigs.append(ctx.compress_chunk(ks[c], vs[c], qs[c], want_signals=True)["att"])
        ctx.flush()
        torch.cuda.synchronize()

        def compress_att_given():
            ctx.reset()
            for c in range(n_chunks):
                ctx.compress_chunk(ks[c], vs[c], None, att_signal=att_sigs[c])
            ctx.flush()

        compress_att_given()
        torch.cuda.synchronize()
        ag_ms, how = timed(compress_att_given, 3), "eager"
        if not a.no_graph:
            try:
                agraph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(agraph):
                    compress_att_given()
                torch.cuda.synchronize()
                agraph.replay()
                ag_ms, how = timed(agraph.replay, 5), "hipgraph"
            except Exception as e:
                print(f"bench.py: capture of the attention-given pass failed ({e}); eager timing kept", file=sys.stderr)
        ag_bytes = 2 * kappa * L * b_tok / P + Hkv * D * esz + 4       # per token: kept rows in and out, keys, the signal
        res["compress_attention_signal_given"] = {
            "launch": how, "ms_per_stream": ag_ms, "tokens_per_s": n_frames * P / (ag_ms * 1e-3),
            "algorithmic_bytes_per_token": ag_bytes, "achieved_GBs": ag_bytes * n_frames * P / (ag_ms * 1e-3) / 1e9,
            "frac_of_peak": ag_bytes * n_frames * P / (ag_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del att_sigs

    # ---- the oracle on the host cores, on a bounded sample of the same stream -------------
    if not a.no_cpu_baseline:
        from oracle import oracle as orc

        n_s = min(a.cpu_sample_frames, n_frames)
        n_sc = (n_s + chunk - 1) // chunk
        axis = orc.TOKEN_AXIS if a.freq_axis == "token" else orc.FEATURE_AXIS
        ref = orc.OracleMuKV(orc.OracleConfig(L, Hq, Hkv, D, P, w.frames_per_segment, w.superpatches_per_frame,
                                              w.keep_ratio, w.alpha, freq_axis=axis))
        host = [(synth.as_numpy(ks[c]), synth.as_numpy(vs[c]), synth.as_numpy(qs[c])) for c in range(n_sc)]
        orc.lib()
        t0 = time.perf_counter()
        for kn, vn, qn in host:
            ref.compress_chunk(kn, vn, q_last=qn)
        t_cpu = time.perf_counter() - t0
        # the same on one host thread, on a sample an order of magnitude smaller
        n_all = int(orc.lib().orc_num_threads())
        orc.lib().orc_set_num_threads(1)
        ref1 = orc.OracleMuKV(orc.OracleConfig(L, Hq, Hkv, D, P, w.frames_per_segment, w.superpatches_per_frame,
                                               w.keep_ratio, w.alpha, freq_axis=axis))
        t0 = time.perf_counter()
        for kn, vn, qn in host[: max(1, 128 // chunk)]:
            ref1.compress_chunk(kn, vn, q_last=qn)
        t_one = time.perf_counter() - t0
        orc.lib().orc_set_num_threads(n_all)
        res["cpu_baseline_one_thread"] = {"value": ref1.n_frames * P / t_one, "unit": "visual tokens/s", "cores": 1,
                                          "kind": "oracle", "sample": f"first {ref1.n_frames} frames ({t_one:.1f} s)"}
        res["cpu_baseline"] = {"value": ref.n_frames * P / t_cpu, "unit": "visual tokens/s",
                               "cores": int(orc.lib().orc_num_threads()), "kind": "oracle",
                               "sample": f"first {ref.n_frames} frames of the same stream through the oracle's "
                                         f"compress_chunk ({t_cpu:.1f} s) on {cpu_model()}"}
    ctx.close()

    # ---- the other stream shapes of the task (7B-class short stream, 72B-class hour), each as a short run of
    # this same program in a process of its own once this one has given its memory back ----
    if a.workload == "hour" and not a.frames and not a.no_other_configs:
        import subprocess

        K = V = Q = ks = vs = qs = g_out = None   # (the side runs would fit beside them as well: 40 + 85 GB of 288)
        torch.cuda.empty_cache()
        res["other_configs"] = {}
        for wl in ("7b", "72b"):
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", wl, "--core-only", "--steps", "3", "--warmup", "1",
                   "--batch-chunks", str(a.batch_chunks), "--overlap-copy", str(a.overlap_copy), "--seed", str(a.seed)]
            try:
                out = subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=240).stdout.strip().splitlines()
                r = json.loads(out[-1])
                res["other_configs"][wl] = {
                    "workload": r["config"]["workload"], "visual_tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
                    "path_hbm_frac_of_peak": r["path_hbm"]["frac_of_peak"],
                    "path_algorithmic_bytes_per_token": r["path_hbm"]["algorithmic_bytes_per_token"],
                    "retrieve_gather_ms_per_question": r["retrieve_gather_ms_per_question"],
                    "dominant_kernel": r["roofline"]["kernel"], "dominant_kernel_frac": r["roofline"]["frac"],
                    "gather_frac": r["roofline_gather"]["frac"], "steps": r["steps"]}
            except Exception as e:   # a failed side run must not lose the main line
                res["other_configs"][wl] = {"error": repr(e)[:300]}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
