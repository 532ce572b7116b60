"""The seeded input generator: the tensor hash equals its integer definition, values are
reproducible, sliceable and bf16-exact, and the distribution has the stated shape."""
import numpy as np
import torch

from paper_2602_16839_amd import inputs as I


def test_mix64_tensor_matches_python_integers():
    xs = [0, 1, 2, 0x7FFFFFFFFFFFFFFF, 0x8000000000000000, 0xFFFFFFFFFFFFFFFF, 0x123456789ABCDEF0, 12345678901234567]
    t = torch.tensor([I._signed(x) for x in xs], dtype=torch.int64)
    got = [int(v) & I.MASK64 for v in I.mix64(t).tolist()]
    assert got == [I.mix64_int(x) for x in xs]
    # splitmix64 reference point: mixing the golden-ratio increment gives the generator's first
    # output for seed 0 (Steele, Lea & Flood 2014)
    assert I.mix64_int(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF


def test_gaussian_is_a_pure_function_of_its_coordinates():
    wl = I.WORKLOADS["qwen3b"].replace(batch=6)
    q, k, v = I.qkv_steps(wl, 0, 5)
    q2, k2, v2 = I.qkv_steps(wl, 3, 5, b0=2, b1=4)
    assert torch.equal(q[3:5, 2:4], q2) and torch.equal(k[3:5, 2:4], k2) and torch.equal(v[3:5, 2:4], v2)
    assert q.dtype == torch.bfloat16 and q.shape == (5, 6, 16, 128) and k.shape == (5, 6, 2, 128)
    assert not torch.equal(k, v)
    # one element from the integer definition
    t, b, h, i = 4, 5, 1, 77
    counter = ((t * 6 + b) * 2 + h) * 128 + i
    idx = I.mix64_int(counter ^ I.stream_key(wl.seed, I.STREAM_K)) & 0xFFFF
    z = I.normal_table()[idx] * torch.tensor(np.float32(0.088))
    assert k[t, b, h, i] == z.to(torch.bfloat16)


def test_distribution_shape_and_head_scales():
    wl = I.WORKLOADS["qwen7b"].replace(batch=4)
    q, k, v = I.qkv_steps(wl, 0, 16)
    sq, sk, sv = I.qkv_head_scales(wl)
    assert sq.shape == (28,) and sk.shape == (4,) and float(sq.min()) >= 0.5 and float(sq.max()) < 1.5
    assert not torch.equal(sk, sv)
    std = q.float().std(dim=(0, 1, 3))
    assert torch.allclose(std, 0.088 * sq, rtol=0.05)
    f = I.WORKLOADS["tiny_f32"]
    q, _, _ = I.qkv_steps(f, 0, 64)
    assert q.dtype == torch.float32 and abs(float(q.std()) - 0.125) < 0.005 and abs(float(q.mean())) < 0.002


def test_ragged_lengths_and_masks():
    wl = I.WORKLOADS["ragged"]
    L = I.rollout_lengths(wl)
    assert L.shape == (512,) and L.min() >= 1 and L.max() <= 16384
    assert 2500 < np.median(L) < 3600
    assert np.array_equal(L, I.rollout_lengths(wl))
    assert I.active_mask(L, 0).all() and not I.active_mask(L, 16384).any()
    assert (I.rollout_lengths(I.WORKLOADS["qwen3b"]) == 4096).all()


def test_encoder_params_shapes():
    wl = I.WORKLOADS["qwen3b"]
    p = I.encoder_params(wl)
    assert p["q_g"].shape == (32, 2048) and p["WaQ"].shape == (2048, 32)
    assert p["WaK"].shape == (256, 32) and p["k_g"].shape == (32, 256) and p["WaV"].dtype == torch.bfloat16
    assert "k_g" not in I.encoder_params(wl, with_global_kv=False)


def test_bench_byte_model_gives_the_workloads_published_totals():
    # the algorithmic bytes bench.py prices a run at (K and V stream over the live window, q in / out out,
    # append, chunk re-read and S update per eviction) summed over the three model-shaped runs, against the
    # totals worked out by hand from the shapes (GB, 4 significant digits)
    import bench
    for name, total_gb in (("qwen3b", 410.7), ("qwen7b", 6547.7), ("llama8b", 104557.0)):
        wl = I.WORKLOADS[name]
        lengths = I.rollout_lengths(wl)
        tot, tokens = bench.path_bytes(wl, lengths, 0, wl.steps)
        assert abs(tot / 1e9 - total_gb) / total_gb < 2e-4, (name, tot / 1e9)
        assert tokens == wl.batch * wl.steps
        # a run priced in pieces adds up to the run priced at once (the last-K-steps window of the benchmark)
        a, ta = bench.path_bytes(wl, lengths, 0, wl.steps - 20)
        b, tb = bench.path_bytes(wl, lengths, wl.steps - 20, wl.steps)
        assert abs(a + b - tot) <= 1e-9 * tot and ta + tb == tokens
        # closed form of the live-token count behind it: t for t <= W, then cycling W - C + 1 .. W
        W, C = wl.window, wl.chunk
        for t in (1, W, W + 1, W + C, W + C + 1, wl.steps):
            expect = t if t <= W else W - C + ((t - W - 1) % C) + 1
            assert bench.n_live_at(t, W, C) == expect
    # the last 20 steps of the qwen7b run by hand: 128 rollouts, windows of 4077 .. 4096 tokens, no eviction
    wl = I.WORKLOADS["qwen7b"]
    got, _ = bench.path_bytes(wl, I.rollout_lengths(wl), wl.steps - 20, wl.steps)
    per_rollout = sum(2 * 512 * 2 * n for n in range(4077, 4097)) + 20 * (2 * 3584 * 2 + 2 * 512 * 2)
    assert got == 128 * per_rollout
