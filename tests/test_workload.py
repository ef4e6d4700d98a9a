"""The synthetic input generators: determinism, shapes, value structure, and bit-exact agreement
of the generator's torch quantizer with the oracle's independent numpy quantizer (CPU)."""
import numpy as np
import pytest
import torch

import workload as W
from oracle import moe_oracle as O


def test_streams_are_deterministic_and_distinct():
    a = W.expert_matrix(0, 3, 5, W.generate.W1, 64, 128)
    b = W.expert_matrix(0, 3, 5, W.generate.W1, 64, 128)
    c = W.expert_matrix(0, 3, 5, W.generate.W3, 64, 128)
    d = W.expert_matrix(1, 3, 5, W.generate.W1, 64, 128)
    assert torch.equal(a, b) and not torch.equal(a, c) and not torch.equal(a, d)
    assert a.shape == (128, 64) and W.expert_matrix(0, 0, 0, W.generate.W2, 64, 128).shape == (64, 128)
    assert abs(float(a.std()) - 0.02) < 0.002
    g = W.gate_weight(0, 0, 8, 256)
    assert g.dtype == torch.float32 and g.shape == (8, 256) and abs(float(g.std()) - 0.02) < 0.003


def test_ar1_stream_statistics_and_batch_prefix_property():
    x = W.hidden_ar1(0, 400, 2, 512).float()
    assert x.shape == (400, 2, 512)
    assert abs(float(x.var()) - 1.0 / (1 - 0.64)) < 0.25
    lag1 = float((x[1:, 0] * x[:-1, 0]).mean() / x[:, 0].var())
    assert abs(lag1 - 0.8) < 0.03
    assert abs(float((x[:, 0] * x[:, 1]).mean())) < 0.1          # batch rows are independent
    assert torch.equal(W.hidden_ar1(0, 50, 1, 512)[:, 0], W.hidden_ar1(0, 50, 3, 512)[:, 0])
    y = W.hidden_iid(0, 64, 1, 256).float()
    assert abs(float(y.std()) - 1.0) < 0.05


@pytest.mark.parametrize("bits,group", [(4, 64), (3, 64), (2, 16)])
def test_generator_quantizer_matches_oracle_quantizer_bit_for_bit(bits, group):
    w = W.expert_matrix(0, 0, 1, W.generate.W1, 256, 96)
    w[3, :group] = 0.01
    q, s, z = W.quantize_minmax(w, bits, group)
    qo, so, zo = O.quantize_minmax(w.numpy(), bits, group)
    assert (q.numpy() == qo).all()
    assert (s.numpy().view(np.uint16) == so.view(np.uint16)).all()
    assert (z.numpy().view(np.uint16) == zo.view(np.uint16)).all()


def test_generator_second_level_matches_oracle_bit_for_bit():
    w = W.expert_matrix(0, 0, 2, W.generate.W2, 256, 512)           # w2: [256][512], 8 groups of 64 per row
    q, s, z = W.quantize_minmax(w, 4, 64)
    degenerate = 0
    for scale_group in (1, 2, 4, 256):                              # short runs hit the "stored as a constant" rule
        qs, qz, meta, r = W.quantize_meta8(s, z, scale_group)
        qso, qzo, metao, ro = O.quantize_meta8(s.numpy(), z.numpy(), scale_group)
        assert r == ro == min(scale_group, 8)
        assert (qs.numpy() == qso).all() and (qz.numpy() == qzo).all()
        assert (meta.numpy().view(np.uint16) == metao.view(np.uint16)).all()
        assert np.isfinite(metao.astype(np.float64)).all()
        degenerate += int((metao[:, :, 0] == 1).sum())
    assert degenerate > 0
    ex = W.quantized_expert(0, 0, 1, 256, 512, 4, 64, scale_group=256)
    assert len(ex) == 3 and all(len(m) == 5 for m in ex) and ex[0][3].shape == (512, 1, 4) and ex[2][3].shape == (256, 1, 4)
    assert ex[0][4] == 4 and ex[2][4] == 8
    # rows that end in a shorter run (3-bit and 2-bit schemes), against the oracle's quantizer
    for bits, g, cols, scale_group in ((3, 64, 448, 4), (2, 16, 176, 8)):
        w = W.expert_matrix(0, 1, 3, W.generate.W2, 64, cols)
        q, s, z = W.quantize_minmax(w, bits, g)
        qs, qz, meta, r = W.quantize_meta8(s, z, scale_group)
        qso, qzo, metao, ro = O.quantize_meta8(s.numpy(), z.numpy(), scale_group)
        assert r == ro == scale_group and meta.shape[1] == -(-(cols // g) // scale_group) and (cols // g) % scale_group != 0
        assert (qs.numpy() == qso).all() and (qz.numpy() == qzo).all()
        assert (meta.numpy().view(np.uint16) == metao.view(np.uint16)).all()


def test_layer_formats():
    assert W.layer_formats(W.CONFIGS["mixtral_stack"]) == [(4, 64)] * 32
    f = W.layer_formats(W.CONFIGS["mixtral_stack_lowbit"])
    assert len(f) == 32 and set(f) == {(2, 16), (3, 64)} and f == W.layer_formats(W.CONFIGS["mixtral_stack_lowbit"])
