"""The seeded workload generators: shapes and structure of the five configurations."""
import numpy as np

from paper_2511_00101_amd import synth


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.3, 0.0, 65280.0], np.float32)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0, 1.015625, -3.296875, 0.0, 65280.0]


def test_config_shapes():
    p1 = synth.config1()
    assert (p1.n_tokens, p1.d_in, p1.d_out, p1.n_adapters) == (102, 256, 256, 4)
    assert (p1.batch.token_kind == 0).sum() == 64 and (p1.batch.token_kind == 1).sum() == 32
    b2 = synth.batch_decode_heavy(np.random.default_rng(2500))
    assert b2.n_tokens == 256 and set(b2.token_kind.tolist()) == {2} and b2.token_adapter.max() < 64
    b3 = synth.batch_unified(np.random.default_rng(3500))
    assert b3.n_tokens == 4864
    b4 = synth.batch_zipf(np.random.default_rng(4500))
    ft = (b4.token_kind == 0).sum()
    assert b4.n_tokens == 8192 and 819 <= ft <= 819 + 1024
    b5 = synth.config5_batch()
    assert b5.n_tokens == 5632 and (b5.token_kind == 0).sum() == 4096 and (b5.token_kind == 2).sum() == 512
    # kinds come in the order fine-tune | prefill | decode
    for b in (b3, b4, b5):
        assert np.all(np.diff(b.token_kind.astype(np.int32)) >= 0)


def test_generators_are_deterministic():
    a, b = synth.config1(), synth.config1()
    assert np.array_equal(a.x, b.x) and np.array_equal(a.A[3], b.A[3]) and np.array_equal(a.batch.token_adapter,
                                                                                         b.batch.token_adapter)
    lens = synth.zipf_lengths(np.random.default_rng(1), 8192)
    assert lens.sum() == 8192 and lens.max() <= 1024 and lens.min() >= 1
