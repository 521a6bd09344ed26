"""The seeded generators: determinism, shapes, and the stated distributions."""
import numpy as np

from glowq_inputs import (CONFIGS, config_units, from_act_bits, gen_activations,
                          gen_direct_unit, gen_module_weight, gen_restore_mask, to_act_bits)


def test_workload_table_matches_the_stated_shapes():
    assert config_units(2)[0].d_outs == (4096, 4096, 4096)
    assert config_units(3)[0].d_outs == (11008, 11008)
    blk = config_units(4)
    assert [u.d_in for u in blk] == [4096, 4096, 4096, 14336]
    assert blk[0].d_outs == (4096, 1024, 1024) and blk[2].d_outs == (14336, 14336)
    assert len(config_units(5)) == 160
    assert CONFIGS[5]["T"] == (1, 1024) and CONFIGS[3]["act"] == "bf16"


def test_weights_and_activations_are_reproducible_and_distinct():
    a = gen_module_weight(2, 0, 1, 64, 256)
    b = gen_module_weight(2, 0, 1, 64, 256)
    c = gen_module_weight(2, 0, 2, 64, 256)
    assert a.dtype == np.float32 and np.array_equal(a, b) and not np.array_equal(a, c)
    assert abs(a.std() - 0.02) < 0.002
    x = gen_activations(2, 0, 8, 4096, "f16", True)
    assert x.dtype == np.uint16 and x.shape == (8, 4096)
    assert np.array_equal(x, gen_activations(2, 0, 8, 4096, "f16", True))
    v = from_act_bits(x, "f16")
    ch = np.sqrt((v ** 2).mean(axis=0))
    assert (ch > 10).sum() >= 20          # about 1 % outlier channels, 20x larger
    assert np.all(np.isfinite(v))


def test_casts_round_trip():
    v = np.array([1.0, -0.333, 1e-5, 300.0], np.float32)
    for act in ("f16", "bf16"):
        bits = to_act_bits(v, act)
        assert np.array_equal(to_act_bits(from_act_bits(bits, act), act), bits)


def test_restore_mask_count():
    m = gen_restore_mask(5, 160, 0.25)
    assert m.dtype == np.uint8 and m.sum() == 40 and set(m.tolist()) == {0, 1}
    assert np.array_equal(m, gen_restore_mask(5, 160, 0.25))


def test_direct_unit_shapes_and_ranges():
    import torch

    shape = config_units(1)[0]
    u = gen_direct_unit(1, 0, shape, 4, 16, 64, "f16")
    assert u["X"].shape == (4, 256) and u["B"].shape == (16, 256)
    for m in u["modules"]:
        assert m["wq"].dtype == torch.int32 and m["wq"].shape == (256, 32)
        assert m["scales"].dtype == torch.float16 and m["scales"].shape == (256, 4)
        z = m["zeros"].float()
        assert torch.all((z >= 5) & (z <= 10) & (z == z.round()))
        assert m["A"].shape == (256, 16)
