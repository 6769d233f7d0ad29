"""Host checks of the seeded input recipe (no method arithmetic involved)."""
import numpy as np
import synth_inputs as si


def test_lengths_follow_the_stated_laws():
    rng = np.random.default_rng(0)
    T = si.draw_lengths(("uniform", 256, 2048), 20000, rng)
    assert T.min() >= 256 and T.max() <= 2048 and abs(T.mean() - 1152) < 15
    T = si.draw_lengths(("lognormal", 2048, 0.5, 1, 8192), 20000, rng)
    assert T.max() <= 8192 and T.min() >= 1 and abs(np.median(T) - 2048) < 40
    T = si.draw_lengths(("pareto", 1.5, 128, 32768), 200000, rng)
    assert T.min() >= 128 and T.max() <= 32768
    assert abs((T > 256).mean() - 2 ** -1.5) < 0.01        # Pareto tail: P(T > 2 t_min) = 2^-alpha


def test_batches_are_seed_deterministic_and_bf16_representable():
    a = si.make_batch_numpy("qwen3_0p6b_head", 3, P=1, G=2, lengths=("uniform", 4, 8), V=64)
    b = si.make_batch_numpy("qwen3_0p6b_head", 3, P=1, G=2, lengths=("uniform", 4, 8), V=64)
    for k in ("hidden", "W", "ids", "logp_noise", "cu_seqlens", "rewards"):
        assert np.array_equal(a[k], b[k])
    again, bits = si.round_to_bf16(a["hidden"])
    assert np.array_equal(again, a["hidden"]) and bits.dtype == np.uint16
    c = si.make_batch_numpy("qwen3_0p6b_head", 4, P=1, G=2, lengths=("uniform", 4, 8), V=64)
    assert not np.array_equal(a["ids"], c["ids"]) or not np.array_equal(a["cu_seqlens"], c["cu_seqlens"])


def test_round_to_bf16_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0], dtype=np.float32)
    r, _ = si.round_to_bf16(x)
    assert r.tolist() == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0]


def test_equal_reward_groups_and_workload_table():
    rng = np.random.default_rng(2)
    R = si.draw_rewards(32, 8, rng, 0.1)
    assert all(len(set(R[i])) == 1 for i in range(4))
    assert [si.WORKLOADS[n]["H"] for n in si.WORKLOAD_ORDER] == [64, 1024, 4096, 4096, 5120, 3584]
    assert si.WORKLOADS["qwen3_8b_head_rpc"]["V"] == 151936
