"""Host-only checks of the synthetic workload generators."""
import numpy as np

from oracle import dag
from workloads import configs, dags, rng


def test_generator_is_counter_based_and_normal():
    a = rng.normal(5, 3, 1001, chunk=64)
    np.testing.assert_array_equal(a[:501], rng.normal(5, 3, 501))
    x = rng.normal(0, 0, 1 << 18)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1) < 0.01 and abs((x ** 4).mean() - 3) < 0.1
    assert abs(np.corrcoef(x[0::2], x[1::2])[0, 1]) < 0.01
    assert not np.array_equal(rng.normal(0, 1, 100), rng.normal(0, 0, 100))
    assert not np.array_equal(rng.normal(1, 0, 100), rng.normal(0, 0, 100))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.005, -2.5, 3.0e38], np.float64)
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7; 1 + 3*2^-8 ties up to even 1 + 2^-6
    np.testing.assert_array_equal(rng.round_to_bf16_bits(x),
                                  np.array([0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x7F62], np.uint16))


def test_named_configs_have_the_stated_byte_counts():
    assert configs.cfg1_add_layernorm().algorithmic_bytes == 595968
    w = configs.cfg2_masked_softmax(heads=1)
    assert w.algorithmic_bytes == 2 * 2 * 512 * 512 + 2 * 512 * 512
    # full-size figures follow from the shapes alone
    assert 2 * 2 * 32 * 512 * 512 + 2 * 512 * 512 == 34078720
    assert 3 * 2 * 8192 * 11008 + 2 * 11008 == 541087232
    assert 2 * 2 * 4 * 2048 * 32 * 128 + 2 * 4 * 2048 * 128 + 2 * 128 == 136315136


def test_random_dags_are_deterministic_and_well_formed():
    att = dags.accepted_attempts()
    assert sorted(att) == list(range(dags.N_DAGS))
    seen_ops = set()
    for k in range(dags.N_DAGS):
        w = dags.draw_dag(k, att[k], with_inputs=False)
        assert w.text == dags.draw_dag(k, att[k], with_inputs=False, max_rows=None).text
        g = dag.parse(w.text)
        n_ops = sum(1 for n in g.nodes if n.op not in ("input", "const"))
        assert 4 <= n_ops <= 16, (k, n_ops)
        assert len(g.outputs) >= 1
        seen_ops.update(n.op for n in g.nodes)
        full = int(np.prod(w.meta["shape"]))
        assert 8000 <= full <= 1.01e7
    assert {"add", "sub", "mul", "div", "exp", "tanh", "sigmoid", "gelu", "rsqrt",
            "sum", "max", "mean", "transpose"} <= seen_ops


def test_capped_copy_keeps_the_structure():
    w = dags.cfg5(7, with_inputs=False)
    s = dags.cfg5(7, max_rows=8)
    strip = lambda t: [l.split(":")[0] for l in t.splitlines() if not l.startswith("in")]
    assert strip(w.text) == strip(s.text)
    out = dag.run(s.text, s.inputs)
    assert all(np.isfinite(o).all() for o in out)
