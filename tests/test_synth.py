"""The seeded input generators both sides draw from: reproducible, of the stated shape, and
independent of how a stream is cut into chunks.  No GPU, no method arithmetic."""
import numpy as np
import torch

from paper_2605_22269_amd import synth


def test_stream_does_not_depend_on_chunking():
    w = synth.WORKLOADS["tiny"].scaled(n_frames=6)
    a = synth.SynthStream(w, 3).next_chunk(6)
    s = synth.SynthStream(w, 3)
    parts = [s.next_chunk(n) for n in (1, 3, 2)]
    for i, name in enumerate("kvq"):
        whole = a[i]
        cut = torch.cat([p[i] for p in parts], dim=2 if name != "q" else 1)
        assert torch.equal(whole, cut), name
    assert a[0].shape == (w.n_layers, w.n_kv_heads, 6 * w.tokens_per_frame, w.head_dim)
    assert a[2].shape == (w.n_q_heads, 6 * w.tokens_per_frame, w.head_dim)


def test_stream_is_seeded():
    w = synth.WORKLOADS["tiny"].scaled(n_frames=2)
    k1, _, _ = synth.SynthStream(w, 5).next_chunk(2)
    k2, _, _ = synth.SynthStream(w, 5).next_chunk(2)
    k3, _, _ = synth.SynthStream(w, 6).next_chunk(2)
    assert torch.equal(k1, k2) and not torch.equal(k1, k3)


def test_handed_over_attention_shape_sink_and_ties():
    a = synth.handed_over_attention(3, 1000, 7)
    assert a.shape == (3, 1000) and a.dtype == torch.float32
    assert torch.equal(a, synth.handed_over_attention(3, 1000, 7))
    x = a.numpy()
    assert (x >= 0).all() and (x[:, 0] == x.max(axis=1)).all()          # the sink on the first token
    assert len(np.unique(x[0])) < 900                                   # snapped values repeat
    smooth = synth.handed_over_attention(3, 1000, 7, tie_fraction=0.0).numpy()
    assert len(np.unique(smooth[0])) > 990


def test_question_lengths_are_in_range_and_seeded():
    lens = synth.question_lengths(64, 16, 64, 9)
    assert len(lens) == 64 and min(lens) >= 16 and max(lens) <= 64
    assert lens == synth.question_lengths(64, 16, 64, 9)
