"""The seeded generator: shapes and distributions of the five configurations, determinism."""
import numpy as np

from paper_2510_03283_amd import synth


def test_counter_based_streams_are_sliceable_and_deterministic():
    a = synth.normal(3, 5, 0, 1000)
    b = synth.normal(3, 5, 400, 100)
    assert np.array_equal(a[400:500], b)
    assert not np.array_equal(synth.normal(3, 6, 0, 100), a[:100])
    z = synth.normal(11, 0, 0, 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    r = synth.randint(1, 2, 0, 10000, 128, 512)
    assert r.min() == 128 and r.max() == 512


def test_bf16_rounding():
    x = np.array([1.0, 1.00390625, 1.005859375, 3.14159, -2.71828], np.float32)
    r = synth.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0078125      # tie to even, then above the tie
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(synth.round_to_bf16(r), r)
    bits = synth.bf16_bits(r)
    assert bits.dtype == np.uint16 and bits[0] == 0x3F80


def test_config_shapes():
    expect = {"tiny": (112, 4, 128, 64), "7b": (4096, 64, 16 * 768, 4096), "7b_decode": (0, 256, 4 * 384, 512),
              "7b_ft": (1024, 16, 64 * 1024, 32768)}
    for name, (tp, td, tf, R) in expect.items():
        b = synth.make_batch(synth.CONFIGS[name])
        assert (b.t_prefill, b.t_decode, b.t_ft, b.n_loss_rows) == (tp, td, tf, R), name
    b = synth.make_batch(synth.CONFIGS["edge"])
    assert b.n_prefill == 8 and b.n_decode == 32 and b.n_ft_seq == 8
    assert b.prefill_lens.min() >= 128 and b.prefill_lens.max() <= 512
    assert b.decode_ctx.min() >= 256 and b.decode_ctx.max() <= 2048
    resp = b.ft_lens - b.ft_prompt_lens
    assert resp.min() >= 64 and resp.max() <= 256 and np.all(b.ft_prompt_lens == 256)
    # block tables: disjoint blocks, enough for context + the new token
    used = np.concatenate([t for t in b.prefill_block_tables] + [row[row >= 0] for row in b.decode_block_tables])
    assert len(np.unique(used)) == len(used) and used.max() < b.num_blocks
    for j, n in enumerate(b.decode_ctx):
        assert (b.decode_block_tables[j] >= 0).sum() == -(-(int(n) + 1) // b.block_size)


def test_tiny_workload_values():
    w = synth.make_workload("tiny")
    assert w.x.shape == (244, 256) and w.x.dtype == np.float32
    assert abs(w.weights["wq"].std() - 0.02) < 0.002 and abs(w.weights["g1"].mean() - 1.0) < 0.01
    b = w.batch
    o0, o1 = b.seg_offsets[6], b.seg_offsets[7]
    assert np.array_equal(b.token_ids[o0:o0 + 32], b.token_ids[o1:o1 + 32])      # shared prompt
    assert not np.array_equal(b.token_ids[o0 + 32:o0 + 64], b.token_ids[o1 + 32:o1 + 64])
    assert [len(k) for k in w.ctx_k] == [32, 64, 96, 128]
    sub = synth.make_workload("edge", n_prefill=1, n_decode=2, n_pairs=1, weights={k: v[:8] for k, v in w.weights.items()} | {"E": np.zeros((32000, 4), np.float32)})
    full = synth.make_batch(synth.CONFIGS["edge"])
    assert sub.batch.prefill_lens[0] == full.prefill_lens[0] and np.array_equal(sub.batch.decode_ctx, full.decode_ctx[:2])
