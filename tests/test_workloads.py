"""The seeded input generators: storage encoders against torch's CPU casts, shapes of the five configurations."""
import numpy as np
import torch

from paper_2506_19830_amd import workloads as W


def test_bf16_encoder_matches_torch_rne():
    x = (np.random.default_rng(0).standard_normal(200_000) * 37).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40]   # ties and extremes
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(W.encode_bf16(x), ref)


def test_fp8_encoder_matches_torch_rne_and_saturates():
    x = (np.random.default_rng(1).standard_normal(200_000) * 120).astype(np.float32)
    x[:10] = [0.0, -0.0, 448.0, -448.0, 17.0, 19.0, 2.0 ** -10, 2.0 ** -9 * 1.5, 0.0009765625, 464.0]
    inside = np.abs(x) <= 448
    ref = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = W.encode_fp8_e4m3(x)
    np.testing.assert_array_equal(got, ref)
    assert (got[~inside] & 0x7F == 0x7E).all()          # saturated to +-448, never NaN


def test_configs_have_the_stated_shapes():
    a1, c1 = W.config(1)
    assert (a1.prefix_lens, a1.gamma, a1.L, a1.Hq, a1.Hkv, a1.D, a1.q_dtype) == ((256,), 2, 8, 4, 1, 64, "f32")
    assert (c1.V, c1.K, c1.logits_dtype) == (512, 4, "f32")
    a2, c2 = W.config(2)
    assert (a2.prefix_lens, a2.gamma, a2.L, a2.Hq, a2.Hkv, a2.D) == ((4096,), 4, 32, 64, 8, 128)
    assert (c2.NB, c2.K, c2.V, c2.logits_dtype) == (4, 4, 152064, "bf16")
    a3, c3 = W.config(3)
    assert (a3.prefix_lens, a3.gamma, a3.L, a3.Hq, a3.Hkv) == ((16384,), 8, 64, 40, 8)
    assert (c3.NB, c3.K, c3.logits_dtype) == (8, 8, "f32")
    a4, c4 = W.config(4)
    assert a4.prefix_lens == (8192, 16384, 24576, 32768) and a4.paged and a4.block_size == 16 and a4.L == 48
    assert c4.NB == 32
    a5, c5 = W.config(5)
    assert (a5.prefix_lens, a5.kv_dtype, a5.q_dtype, a5.gamma, a5.L) == ((32768,), "fp8_e4m3", "bf16", 8, 64)
    # arithmetic-intensity bookkeeping used by the benchmark
    assert a5.flops() == 4 * 128 * (8 * 64 * 40) * (32768 + 32.5)
    assert a5.algorithmic_bytes() == 2 * 8 * 32768 * 128 + 2 * 512 * 8 * 128 + 512 * 40 * 128 * 4


def test_generators_are_seeded_and_layouts_are_right():
    case = W.AttnCase("t", (40, 9), 2, 3, 4, 2, 8, "bf16", "fp8_e4m3", "fp8_e4m3", "bf16", block_size=16, paged=True)
    a, b = W.make_attention_inputs(case), W.make_attention_inputs(case)
    for k in a:
        if a[k] is not None:
            np.testing.assert_array_equal(a[k], b[k])
    assert a["q"].shape == (2, 2, 3, 4, 8) and a["q"].dtype == np.uint16
    assert a["k_cache"].shape == (4, 2, 16, 8) and a["k_cache"].dtype == np.uint8      # 3 + 1 blocks in the pool
    assert a["block_tables"].shape == (2, 3)
    used = np.concatenate([a["block_tables"][0, :3], a["block_tables"][1, :1]])
    assert sorted(used.tolist()) == [0, 1, 2, 3]
    assert a["k_scale"].shape == (2,) and (a["k_scale"] > 0).all()
    other = W.make_attention_inputs(W.with_layer(case, 1))
    assert not np.array_equal(other["q"], a["q"])
    acc = W.make_accept_inputs(W.AcceptCase("a", 3, 2, 64, "bf16"))
    assert acc["target_logits"].shape == (3, 3, 64) and acc["draft_logits"].shape == (3, 2, 64)
    assert acc["draft_tokens"].min() >= 0 and acc["draft_tokens"].max() < 64
    assert (acc["u_accept"] >= 0).all() and (acc["u_accept"] < 1).all()


def test_drafted_tokens_follow_the_draft_distribution():
    case = W.AcceptCase("a", 20000, 1, 6, "f32", target_std=1.0, draft_noise_std=None, seed=3)
    inp = W.make_accept_inputs(case)
    d = inp["draft_logits"][:, 0].astype(np.float64)
    q = np.exp(d); q /= q.sum(-1, keepdims=True)
    # mean one-hot minus mean probability -> 0
    onehot = np.eye(6)[inp["draft_tokens"][:, 0]]
    assert np.abs(onehot.mean(0) - q.mean(0)).max() < 0.012


def test_point_mass_accept_recipe():
    """Prompt-lookup style drafts: tokens without draft logits, the target row peaked at each drafted token."""
    c = W.AcceptCase("pm", 6, 3, 1000, "f32", point_mass=True, peak=9.0, seed=3)
    a, b = W.make_accept_inputs(c), W.make_accept_inputs(c)
    assert a["draft_logits"] is None
    np.testing.assert_array_equal(a["target_logits"], b["target_logits"])
    np.testing.assert_array_equal(a["draft_tokens"], b["draft_tokens"])
    t, tok = a["target_logits"], a["draft_tokens"]
    assert t.shape == (6, 4, 1000) and tok.shape == (6, 3) and (tok >= 0).all() and (tok < 1000).all()
    picked = np.take_along_axis(t[:, :3, :], tok[:, :, None], axis=2)[..., 0]
    assert picked.mean() > 6.0 and abs(float(np.median(t))) < 0.5      # N(0, 3^2) + 9 at the drafted tokens
    assert c.algorithmic_bytes() == 6 * 4 * 1000 * 4


def test_late_key_shift_raises_the_scores_of_the_late_keys():
    case = W.AttnCase("late", (300,), 2, 3, 4, 2, 128, "bf16", "bf16", "bf16", "bf16", late_key_shift=20.0, late_from=100)
    inp = W.make_attention_inputs(case)
    dec = lambda bits: (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    q, kc, kb = dec(inp["q"]), dec(inp["k_cache"]), dec(inp["k_branch"])
    keys = kc.transpose(1, 0, 2, 3).reshape(2, -1, 128)[:, :300]            # contiguous cache: [Hkv, token, D]
    for h in range(4):
        s = keys[h // 2] @ q[0, 1, 2, h] * case.scale                        # one query row against the prefix
        # (the row's own noise along u moves its shift by 20 / sqrt(128) = 1.8 rms)
        assert abs(s[100:].mean() - s[:100].mean() - 20.0) < 6.0 and s[:100].std() < 2.5 and s[100:].std() < 2.5
        sb = kb[0, 1, :, h // 2] @ q[0, 1, 2, h] * case.scale                # and against its branch's keys
        assert abs(sb.mean() - s[100:].mean()) < 3.0
    plain = W.make_attention_inputs(W.AttnCase("late", (300,), 2, 3, 4, 2, 128, "bf16", "bf16", "bf16", "bf16"))
    np.testing.assert_array_equal(plain["v_cache"], inp["v_cache"])          # nothing else moves
