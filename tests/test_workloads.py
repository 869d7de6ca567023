"""The seeded input generators: layer lists of the five benchmark configurations (sizes computed from
the public architecture shapes), the byte model, and determinism of the generated values."""
import numpy as np
import pytest
import torch

from paper_2403_04206_amd import workloads as W

SHAPES = {  # configuration: (K, L, P, bytes per gradient element, minimum bytes per update)
    0: (4, 20, 269_722, 4, 4 * 269_722 * 12),
    1: (4, 62, 11_689_512, 4, 4 * 11_689_512 * 12),
    2: (16, 80, 36_536_884, 4, 16 * 36_536_884 * 12),
    3: (8, 291, 353_511_424, 2, 8 * 353_511_424 * 10),
    4: (32, 161, 25_557_032, 4, 32 * 25_557_032 * 16),      # fused with the SGD step: g is read twice
}


@pytest.mark.parametrize("i", sorted(SHAPES))
def test_configuration_shapes_and_byte_model(i):
    w = W.config(i)
    K, L, P, sg, nbytes = SHAPES[i]
    assert (w.K, w.L, w.P, w.grad_bytes) == (K, L, P, sg)
    assert w.update_bytes() == nbytes
    off = w.offsets
    assert off[0] == 0 and off[-1] == P and np.all(np.diff(off) > 0)


def test_layer_lists_against_the_architectures():
    assert len(W.resnet20_layers(False)) == 59 and sum(W.resnet20_layers(False)) == 269_722     # per-tensor split
    r18 = W.resnet18_layers()
    assert r18[0] == 64 * 3 * 7 * 7 and r18[-2:] == [512 * 1000, 1000] and min(r18) == 64 and max(r18) == 512 * 512 * 9
    wrn = W.wrn28_10_layers()
    assert wrn[0] == 16 * 3 * 9 and wrn[-2:] == [640 * 100, 100] and max(wrn) == 640 * 640 * 9
    tr = W.transformer_350m_layers()
    assert tr[0] == 50_000 * 1024 and tr.count(1024 * 4096) == 48 and tr.count(1024 * 3072) == 24
    r50 = W.resnet50_layers()
    assert r50[-2:] == [2048 * 1000, 1000] and sum(1 for n in r50 if n < 1024) == 85


def test_inputs_are_seeded_and_shaped():
    w = W.config(0)
    x1, g1 = W.make_inputs(w)
    x2, g2 = W.make_inputs(w)
    assert torch.equal(x1, x2) and torch.equal(g1, g2)
    ld = W.round_up(w.P, W.ROW_ALIGN)
    assert x1.shape == (w.K, ld) and g1.shape == (w.K, ld) and x1.dtype == torch.float32
    assert torch.all(x1[:, w.P:] == 7.0e7)                                    # sentinels in the padding
    # gradient scale of worker k in layer l follows the table: sample std within a factor of 2 on big layers
    s = W.grad_scales(w)
    big = int(np.argmax(np.diff(w.offsets)))
    a, b = int(w.offsets[big]), int(w.offsets[big + 1])
    for k in range(w.K):
        ratio = float(g1[k, a:b].std()) / s[k, big]
        assert 0.9 < ratio < 1.1
    assert abs(float(x1[:, :w.P].std()) - 0.05) < 0.002
    # bf16 gradients are the rounded fp32 draws
    _, _, gb = W.make_small(3, 2, [100, 7], grad_dtype="bf16")
    assert gb.dtype == torch.bfloat16
    # the configuration with one tiny-gradient worker
    w4 = W.config(4)
    assert w4.tiny_worker == 0 and np.all(W.grad_scales(w4)[0] == 1e-6) and w4.fused_sgd


def test_explicit_scale_table_is_honoured():
    # the extreme-magnitude parity cases put chosen standard deviations on chosen (worker, layer) blocks
    table = np.array([[1e-30, 1e20, 1.0], [3e-30, 1e-21, 0.1]])
    w = W.Workload("explicit", 2, [5000, 3000, 4000], scale_table=table, seed=(9, 9))
    assert np.array_equal(W.grad_scales(w), table)
    _, g = W.make_inputs(w)
    for k in range(2):
        for l in range(3):
            blk = g[k, int(w.offsets[l]):int(w.offsets[l + 1])].double()
            assert 0.9 < float(blk.std()) / table[k, l] < 1.1
    with np.testing.assert_raises(ValueError):
        W.grad_scales(W.Workload("bad", 2, [10, 10], scale_table=np.ones((3, 2))))
