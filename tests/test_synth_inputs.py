"""Host-side checks of the seeded input generator (no GPU, no oracle)."""
import numpy as np
import torch

from paper_2507_21276_amd import synth_inputs as S


def test_normal_is_counter_based_and_standard():
    a = S.normal(0, "X", (1000, 50))
    b = S.normal(0, "X", (50000,))
    assert np.array_equal(a.ravel(), b)
    c = S.normal(0, "X", (100,), start=12345)
    assert np.array_equal(c, b[12345:12445])
    assert not np.array_equal(S.normal(1, "X", (100,)), b[:100])
    assert not np.array_equal(S.normal(0, "Y", (100,)), b[:100])
    big = S.normal(0, "moments", (1 << 21,), dtype=np.float64)   # spans two chunks
    assert abs(big.mean()) < 3e-3 and abs(big.std() - 1) < 3e-3
    assert abs((big ** 4).mean() - 3) < 0.05
    assert abs(S.normal(0, "W", (200000,), std=0.02).std() - 0.02) < 2e-4


def test_bf16_round_trip_matches_torch():
    x = S.normal(0, "r", (100000,))
    x[:4] = [1.0, 1.00390625, 1.01171875, -3.0e-39]   # ties and a subnormal
    ours = S.round_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, ref)
    assert np.array_equal(S.to_bf16_bits(x).view(np.int16),
                          torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy())


def test_param_layout_and_recipe():
    for name, cfg in S.CONFIGS.items():
        lay = S.param_layout(cfg)
        assert all(off % 8 == 0 for _, off, _, _ in lay), name   # 16-byte aligned in bf16
    cfg = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=1, d_model=256, n_heads=2, d_ff=384)
    p = S.make_params(cfg)
    assert p.size == S.param_count(cfg) == 256 + 3 * 256 * 256 + 256 * 256 + 256 + 2 * 384 * 256 + 256 * 384
    assert np.all(p[:256] == 1.0)
    w = p[256:256 + 3 * 256 * 256]
    assert abs(w.std() - 0.02) < 5e-4 and np.array_equal(S.round_bf16(w), w)
    # LLaMA-7B quarter stage: 8 * (4 d^2 + 3 d F + 2 d) parameters
    c7 = S.CONFIGS["llama7b_bf16"]
    assert S.param_count(c7) == 8 * (4 * 4096 ** 2 + 3 * 4096 * 11008 + 2 * 4096)


def test_context_lengths_and_page_tables():
    for wl in ("cfg2", "cfg4", "cfg5"):
        serve = S.WORKLOADS[wl]["serve"]
        ctx = S.context_lengths(serve)
        assert len(ctx) == serve["B"]
        if serve["kind"] == "decode_uniform":
            assert ctx.min() >= 128 and ctx.max() <= 2048 and len(set(ctx.tolist())) > 32
        if serve["kind"] == "decode_lognormal":
            assert ctx.min() >= 64 and ctx.max() <= 4096
            assert 700 < np.median(ctx) < 1500
        table, n_pages = S.page_tables(ctx, np.ones_like(ctx), 16)
        used = table[table >= 0]
        assert len(set(used.tolist())) == len(used) and used.max() < n_pages
        need = -(-(ctx + 1) // 16)
        assert np.array_equal((table >= 0).sum(axis=1), need)
        assert n_pages >= 1.05 * need.sum() - 1
        # shuffled: physical ids are not monotone
        assert np.any(np.diff(table[0, : need[0]]) < 0)
    p = S.permutation(0, "p", 1000)
    assert sorted(p.tolist()) == list(range(1000))
