"""Shapes and determinism of the synthetic workloads (no method arithmetic)."""
import numpy as np

from paper_2302_06058_amd import synth


def test_bf16_round_trip_and_rne():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e-5], dtype=np.float32)
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[3] == -2.5 and back[4] == 0.0
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0)
    assert back[1] == 1.0
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even)
    assert back[2] == np.float32(1.015625)
    assert (synth.f32_to_bf16_bits(back) == b).all()


def test_resnet50_shape_table():
    shapes = synth.resnet50_gemm_shapes(64)
    assert len(shapes) == 54
    assert sum(I * J for _, I, J, _ in shapes) == 25_502_912 + 0  # conv + fc weights
    assert shapes[0][1:] == (64, 147, 802816)
    assert shapes[-1][1:] == (1000, 2048, 64)
    assert sum(1 for _, I, J, T in shapes if (I, J, T) == (256, 2304, 12544)) == 6
    c3 = synth.get_config(3)
    assert c3[0].J == 148 and c3[0].j_real == 147
    assert all(l.I % 4 == 0 and l.J % 4 == 0 for l in c3)


def test_configs_and_determinism():
    c1 = synth.get_config(1)[0]
    d1, d2 = synth.gen_layer(c1), synth.gen_layer(c1)
    assert d1.W.dtype == np.float32 and d1.W.shape == (64, 128)
    assert d1.X.shape == (32, 128) and d1.dY.shape == (32, 64) and d1.perms.shape == (4, 64)
    assert (d1.W == d2.W).all() and (d1.perms == d2.perms).all()
    assert all(sorted(p) == list(range(64)) for p in d1.perms)
    c2 = synth.get_config(2)[0]
    assert (c2.I, c2.J, c2.T, c2.K, c2.dtype) == (256, 2304, 12544, 100, synth.BF16)
    x = synth.gen_activations(c2, T=16)
    assert x.dtype == np.uint16 and (synth.bf16_bits_to_f32(x) >= 0).all()   # ReLU'd
    assert len(synth.get_config(4)) == 12 and len(synth.get_config(5)) == 2
    stem = synth.get_config(3)[0]
    w = synth.to_f64(synth.gen_weights(stem), stem.dtype)
    assert (w[:, 147] == 0).all() and (w[:, :147] != 0).any()
