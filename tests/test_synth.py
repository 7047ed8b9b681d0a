"""The seeded input generator: numpy and torch forms agree bit for bit, workloads have the
stated shapes, and the structured parts (outlier channels, planted spans) are where they are
said to be.  CPU only."""
import numpy as np
import pytest
import torch

import wkv_synth as S


def _bits(t):
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_numpy_and_torch_generators_agree(dtype):
    st = S.stream_id(S.KIND_K, 5)
    a = S.normal_np(42, st, 123, 70000, dtype)
    b = S.normal_torch(42, st, 70000, dtype, "cpu", start=123, chunk=4096)
    b = b.numpy() if dtype == "f32" else _bits(b)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, S.normal_np(43, st, 123, 70000, dtype))


def test_distribution_is_standard_normal():
    x = S.normal_np(1, 2, 0, 400000, "f32").astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs((np.abs(x) < 1.0).mean() - 0.6827) < 0.01


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927], dtype=np.float32)
    got = S.f32_to_bf16_bits(x)
    want = _bits(torch.from_numpy(x).to(torch.bfloat16))
    assert np.array_equal(got, want)
    assert np.array_equal(S.bf16_bits_to_f64(got), torch.from_numpy(x).to(torch.bfloat16).double().numpy())


def test_half_stream_rounds_to_nearest_and_uses_halfs_mantissa():
    x = S.normal_table_f32()
    bits = S.normal_table_f16_bits()
    assert np.array_equal(bits, _bits(torch.from_numpy(x.copy()).to(torch.float16)))
    wide = S.f16_bits_to_f64(bits)
    assert np.array_equal(wide, torch.from_numpy(x.copy()).to(torch.float16).double().numpy())
    assert np.abs(wide - x).max() <= 2.0 ** -10 * np.abs(x).max()
    # most entries are NOT representable in bf16: the stream carries more than 8 significant bits
    assert (S.bf16_bits_to_f64(S.f32_to_bf16_bits(wide.astype(np.float32))) != wide).mean() > 0.8
    w = S.Workload(name="h", seed=3, dtype="f16", n_groups=1, gamma=1, n_q_heads=2, n_kv_heads=1, head_dim=64, w_obs=4,
                   seq_len=[50], win=[8], top_p=[8], k_windows=[1], outlier_channels=2)
    full = _bits(w.kv_torch(S.KIND_K, 0, "cpu"))
    assert np.array_equal(full[0, 0], w.kv_np(S.KIND_K, 0, 0, 0))
    assert np.array_equal(w.to_f64(w.kv_np(S.KIND_K, 0, 0, 0)), w.kv_torch(S.KIND_K, 0, "cpu")[0, 0].double().numpy())


def test_workload_table():
    w = {n: S.make_workload(n) for n in S.WORKLOAD_NAMES}
    assert (w["c1"].seq_len, w["c1"].k_windows, w["c1"].nkeep_max, w["c1"].dtype) == ([512], [8], 72, "f32")
    assert (w["c2"].k_windows, w["c2"].nkeep_max) == ([64], 544)
    assert w["c3a"].k_windows == [256] and w["c3b"].k_windows == [64]
    assert (w["c4"].n_layers, w["c4"].k_windows, w["c4"].nkeep_max) == (32, [256], 4128)
    c5 = w["c5"]
    assert c5.batch == 8 and all(4096 <= L <= 32768 for L in c5.seq_len)
    assert set(c5.win) == {8, 32}
    for L, wn, k in zip(c5.seq_len, c5.win, c5.k_windows):
        assert k * wn <= 0.12 * L < (k + 1) * wn
    assert any((L - 32) % wn for L, wn in zip(c5.seq_len, c5.win))   # partial tail windows occur


def test_host_slices_match_device_tensor_small():
    w = S.scaled_workload(S.make_workload("c2"), seq_len=[300], k_windows=[4], n_groups=1, gamma=2)
    for kind in (S.KIND_K, S.KIND_V):
        full = _bits(w.kv_torch(kind, 1, "cpu"))
        for h in (0, 7):
            assert np.array_equal(full[0, h], w.kv_np(kind, 1, 0, h))
            rows = np.array([0, 17, 299])
            assert np.array_equal(full[0, h][rows], w.kv_np(kind, 1, 0, h, rows))
    k = w.to_f64(w.kv_np(S.KIND_K, 0, 0, 2))
    ch = w.outlier_channel_ids(0, S.KIND_K, 2)
    assert len(ch) == 4
    sd = k.std(0)
    assert np.all(sd[ch] > 6.0) and np.all(np.delete(sd, ch) < 1.5)
    assert np.array_equal(_bits(w.q_obs_torch(0, "cpu")), w.q_obs_np(0))


def test_planted_spans_are_aligned_with_mean_query():
    w = S.scaled_workload(S.make_workload("c4"), seq_len=[2048], k_windows=[16], n_groups=2)
    starts = w.span_starts()[0]
    assert len(starts) == 3 and all(s % 64 == 0 and s + 64 <= 2048 - 32 for s in starts)
    for g in (0, 1):
        kt = _bits(w.kv_torch(S.KIND_K, g * w.gamma, "cpu"))
        for h in (0, 5):
            k = w.to_f64(w.kv_np(S.KIND_K, g * w.gamma, 0, h))
            assert np.array_equal(kt[0, h], w.kv_np(S.KIND_K, g * w.gamma, 0, h))
            q = w.to_f64(w.q_obs_np(g))[0, h * 4:(h + 1) * 4].reshape(-1, 128).mean(0)
            cos = (k @ q) / (np.linalg.norm(k, axis=1) * np.linalg.norm(q))
            inside = np.zeros(2048, bool)
            for s0 in starts:
                inside[s0:s0 + 64] = True
            assert np.all(np.abs(cos[inside] - 0.9) < 0.01)
            assert np.abs(cos[~inside]).max() < 0.5
    # non-scoring layers carry no spans: their rows there are plain noise
    k1 = w.to_f64(w.kv_np(S.KIND_K, 1, 0, 0))
    q = w.to_f64(w.q_obs_np(0))[0, 0:4].reshape(-1, 128).mean(0)
    cos1 = (k1 @ q) / (np.linalg.norm(k1, axis=1) * np.linalg.norm(q))
    assert np.abs(cos1).max() < 0.5
