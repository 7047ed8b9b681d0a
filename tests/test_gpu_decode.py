"""GPU parity of the decode step over the compact cache: wkv_decode_step (through the C ABI)
against the fp64 oracle, on caches produced by wkv_compress_groups and on hand-made ones."""
import itertools

import numpy as np
import pytest
import torch

import paper_2503_17922_amd as W
import wkv_synth as S
from oracle import wkv_oracle as O
from tests import parity as P

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-3, 2e-5     # fp32 accumulation and a hardware exp2 against fp64; values are O(1)
KIND_DECODE = 9             # generator stream of the new-token tensors


def _new_token(w, device, step, what, shape, as_f16=False):
    numel = int(np.prod(shape))
    t = S.normal_torch(w.seed, S.stream_id(KIND_DECODE, step, what), numel, w.dtype, device).view(*shape)
    return t.to(torch.float16) if as_f16 else t          # exact: see DeviceState(as_f16=True)


def _decode_and_check(w, device, n_steps, extra_rows, as_f16=False):
    """Compress a workload straight into caches with room for ``extra_rows`` more tokens, then
    generate ``n_steps`` tokens on the first layer and follow every step with the oracle."""
    base = P.make_problem(w)
    nk = W.wkv_get_dims(base).nkeep_max
    cap = nk + extra_rows
    B, H, Hq, d, G = w.batch, w.n_kv_heads, w.n_q_heads, w.head_dim, w.q_per_kv
    st = P.DeviceState(w, device, as_f16=as_f16)
    # the compact caches ARE the decode caches: same tensors, strides for `cap` rows
    st.problem = P.make_problem(w, out_strides=(H * cap * d, cap * d, d), **(dict(dtype=W.WKV_F16) if as_f16 else {}))
    dt = st.k[0].dtype
    st.k_out = [torch.full((B, H, cap, d), 7.0, dtype=dt, device=device) for _ in range(w.n_layers)]
    st.v_out = [torch.full((B, H, cap, d), 7.0, dtype=dt, device=device) for _ in range(w.n_layers)]
    st.compress()
    layer, g = 0, 0
    n_valid = st.n_keep[g].clone()                                   # [B, H]
    shape = W.DecodeShape(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, capacity=cap,
                          dtype=W.WKV_F16 if as_f16 else {"f32": W.WKV_F32, "bf16": W.WKV_BF16, "f16": W.WKV_F16}[w.dtype])
    ws = torch.empty(W.wkv_decode_workspace_bytes(shape), dtype=torch.uint8, device=device)
    out = torch.full((B, Hq, d), -5.0, dtype=torch.float32, device=device)
    # oracle state: the retained rows of every (b, h), widened exactly
    n0 = n_valid.cpu().numpy()
    ok = {(b, h): P.host_f64(w, st.k_out[layer][b, h, : n0[b, h]]) for b in range(B) for h in range(H)}
    ov = {(b, h): P.host_f64(w, st.v_out[layer][b, h, : n0[b, h]]) for b in range(B) for h in range(H)}
    for step in range(n_steps):
        q = _new_token(w, device, step, 0, (B, Hq, d), as_f16)
        kn = _new_token(w, device, step, 1, (B, H, d), as_f16)
        vn = _new_token(w, device, step, 2, (B, H, d), as_f16)
        k_before, v_before = st.k_out[layer].clone(), st.v_out[layer].clone()
        W.wkv_decode_step(shape, q, kn, vn, st.k_out[layer], st.v_out[layer], n_valid, out, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        nv = n_valid.cpu().numpy()
        for b, h in itertools.product(range(B), range(H)):
            want, ok[b, h], ov[b, h] = O.decode_step(P.host_f64(w, q[b, h * G:(h + 1) * G]), ok[b, h], ov[b, h],
                                                     P.host_f64(w, kn[b, h]), P.host_f64(w, vn[b, h]))
            n = ok[b, h].shape[0]
            assert nv[b, h] == n, f"step {step} b{b} h{h}: n_valid {nv[b, h]} != {n}"
            np.testing.assert_allclose(got[b, h * G:(h + 1) * G], want, rtol=RTOL, atol=ATOL,
                                       err_msg=f"{w.name} decode step {step} b{b} h{h}")
            # the appended rows are in the cache, bit for bit, and nothing else moved
            assert torch.equal(st.k_out[layer][b, h, n - 1], kn[b, h]) and torch.equal(st.v_out[layer][b, h, n - 1], vn[b, h])
            assert np.array_equal(P.host_f64(w, st.k_out[layer][b, h, :n]), ok[b, h])
            k_before[b, h, n - 1] = kn[b, h]; v_before[b, h, n - 1] = vn[b, h]
        assert torch.equal(k_before, st.k_out[layer]) and torch.equal(v_before, st.v_out[layer]), "a row other than the appended one changed"
    return st, shape, n_valid, out, ws


def test_decode_after_compression_bf16(device):
    # Llama-shaped heads (G = 4, d = 128); two sequences of different length and window size
    w = S.Workload(name="dec_bf16", seed=91, dtype="bf16", n_groups=1, gamma=2, n_q_heads=8, n_kv_heads=2, head_dim=128,
                   w_obs=16, seq_len=[3000, 1111], win=[8, 16], top_p=[8, 6], k_windows=[120, 20])
    _decode_and_check(w, device, n_steps=3, extra_rows=8)


def test_decode_full_size_cache(device):
    # the retained cache of the 32K configuration's shape on one group: 4128 rows per head, 8 KV heads
    w = S.scaled_workload(S.make_workload("c4"), n_groups=1, gamma=1)
    _decode_and_check(w, device, n_steps=2, extra_rows=64)


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", head_dim=64, n_q_heads=4, n_kv_heads=2, w_obs=8),                 # c1-like, fp32, G = 2
    dict(dtype="f32", head_dim=128, n_q_heads=3, n_kv_heads=3, w_obs=4),                # G = 1
    dict(dtype="bf16", head_dim=64, n_q_heads=12, n_kv_heads=2, w_obs=4),               # G = 6, d = 64
    dict(dtype="bf16", head_dim=128, n_q_heads=16, n_kv_heads=2, w_obs=8),              # G = 8
    dict(dtype="bf16", head_dim=128, n_q_heads=14, n_kv_heads=2, w_obs=8),              # G = 7 (28q/4kv models)
    dict(dtype="bf16", head_dim=64, n_q_heads=10, n_kv_heads=2, w_obs=8),               # G = 5
    dict(dtype="f32", head_dim=128, n_q_heads=6, n_kv_heads=2, w_obs=8),                # G = 3, fp32
    dict(dtype="bf16", head_dim=128, n_q_heads=8, n_kv_heads=2, w_obs=16, seq_len=[16], k_windows=[0]),   # only the observation rows
])
def test_decode_shapes(device, kw):
    base = dict(name="dec_mini", seed=92, dtype="bf16", n_groups=1, gamma=1, n_q_heads=8, n_kv_heads=2, head_dim=128,
                w_obs=16, seq_len=[700], win=[8], top_p=[8], k_windows=[30])
    base.update(kw)
    _decode_and_check(S.Workload(**base), device, n_steps=2, extra_rows=5)


@pytest.mark.parametrize("kw", [
    dict(),                                                                             # G = 4, d = 128
    dict(head_dim=64, n_q_heads=14, n_kv_heads=2, w_obs=8),                             # G = 7, d = 64
])
def test_decode_fp16(device, kw):
    # IEEE half caches: the same values as the bf16 workload (exactly representable), another format
    base = dict(name="dec_f16", seed=95, dtype="bf16", n_groups=1, gamma=1, n_q_heads=8, n_kv_heads=2, head_dim=128,
                w_obs=16, seq_len=[900, 300], win=[8, 16], top_p=[8, 8], k_windows=[30, 6])
    base.update(kw)
    _decode_and_check(S.Workload(**base), device, n_steps=3, extra_rows=8, as_f16=True)


def test_decode_half_values(device):
    # IEEE half tensors drawn as half (11 significant bits: values bf16 cannot hold)
    w = S.Workload(name="dec_half", seed=96, dtype="f16", n_groups=1, gamma=1, n_q_heads=8, n_kv_heads=2, head_dim=128,
                   w_obs=16, seq_len=[900, 300], win=[8, 16], top_p=[8, 8], k_windows=[30, 6])
    st, *_ = _decode_and_check(w, device, n_steps=3, extra_rows=8)
    assert not torch.equal(st.k[0].to(torch.bfloat16).to(torch.float16), st.k[0]), "the inputs fit bf16: not a test of half"


def test_decode_all_layers_of_a_group_share_one_counter(device):
    # Section 2.2.2: the gamma layers of a group share one index set, hence one row count per
    # (sequence, KV head).  The n_keep row of the compression call itself serves as that counter:
    # the first gamma-1 layers run with WKV_DECODE_KEEP_COUNT, the last one advances it.
    w = S.Workload(name="dec_group", seed=97, dtype="bf16", n_groups=2, gamma=3, n_q_heads=8, n_kv_heads=2, head_dim=128,
                   w_obs=16, seq_len=[1200, 500], win=[8, 16], top_p=[8, 6], k_windows=[40, 9])
    B, H, Hq, d, G = w.batch, w.n_kv_heads, w.n_q_heads, w.head_dim, w.q_per_kv
    nk = W.wkv_get_dims(P.make_problem(w)).nkeep_max
    cap = nk + 4
    st = P.DeviceState(w, device)
    st.problem = P.make_problem(w, out_strides=(H * cap * d, cap * d, d))
    st.k_out = [torch.full((B, H, cap, d), 7.0, dtype=torch.bfloat16, device=device) for _ in range(w.n_layers)]
    st.v_out = [torch.full((B, H, cap, d), 7.0, dtype=torch.bfloat16, device=device) for _ in range(w.n_layers)]
    st.compress()
    keep = W.DecodeShape(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, capacity=cap, dtype=W.WKV_BF16,
                         flags=W.WKV_DECODE_KEEP_COUNT)
    bump = W.DecodeShape(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, capacity=cap, dtype=W.WKV_BF16)
    ws = torch.empty(W.wkv_decode_workspace_bytes(bump), dtype=torch.uint8, device=device)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=device)
    g = 1
    n0 = st.n_keep[g].cpu().numpy().copy()
    ok = {(l, b, h): P.host_f64(w, st.k_out[g * w.gamma + l][b, h, : n0[b, h]]) for l in range(w.gamma) for b in range(B) for h in range(H)}
    ov = {(l, b, h): P.host_f64(w, st.v_out[g * w.gamma + l][b, h, : n0[b, h]]) for l in range(w.gamma) for b in range(B) for h in range(H)}
    for step in range(2):
        for l in range(w.gamma):
            layer = g * w.gamma + l
            q = _new_token(w, device, 10 * step + l, 0, (B, Hq, d))
            kn = _new_token(w, device, 10 * step + l, 1, (B, H, d)); vn = _new_token(w, device, 10 * step + l, 2, (B, H, d))
            W.wkv_decode_step(keep if l < w.gamma - 1 else bump, q, kn, vn, st.k_out[layer], st.v_out[layer], st.n_keep[g], out, ws)
            torch.cuda.synchronize()
            want_count = n0 + step + (1 if l == w.gamma - 1 else 0)
            assert np.array_equal(st.n_keep[g].cpu().numpy(), want_count), f"step {step} layer {l}: counter"
            for b, h in itertools.product(range(B), range(H)):
                want, ok[l, b, h], ov[l, b, h] = O.decode_step(P.host_f64(w, q[b, h * G:(h + 1) * G]), ok[l, b, h], ov[l, b, h],
                                                               P.host_f64(w, kn[b, h]), P.host_f64(w, vn[b, h]))
                np.testing.assert_allclose(out[b, h * G:(h + 1) * G].cpu().numpy(), want, rtol=RTOL, atol=ATOL,
                                           err_msg=f"step {step} layer {l} b{b} h{h}")
                n = ok[l, b, h].shape[0]
                assert np.array_equal(P.host_f64(w, st.k_out[layer][b, h, :n]), ok[l, b, h])
                assert np.array_equal(P.host_f64(w, st.v_out[layer][b, h, :n]), ov[l, b, h])
    assert np.array_equal(st.n_keep[0].cpu().numpy(), _fresh_n_keep(st, 0))


def _fresh_n_keep(st, g):
    """The other group's counters are what a fresh compression gives (nothing touched them)."""
    ref = P.DeviceState(st.w, st.device)
    ref.compress()
    return ref.n_keep[g].cpu().numpy()


def test_decode_full_cache_is_refused_per_row(device):
    # capacity reached on some rows: those rows are left alone and flagged with NaN, the others proceed
    w = S.Workload(name="dec_full", seed=93, dtype="bf16", n_groups=1, gamma=1, n_q_heads=4, n_kv_heads=2, head_dim=128,
                   w_obs=8, seq_len=[400, 200], win=[8, 8], top_p=[8, 8], k_windows=[10, 5])
    st, shape, n_valid, out, ws = _decode_and_check(w, device, n_steps=1, extra_rows=1)
    # sequence 0 (10 windows) filled its cache with that one step; sequence 1 still has room
    cap = shape.c.capacity
    assert n_valid[0].tolist() == [cap, cap] and max(n_valid[1].tolist()) < cap
    before_k = st.k_out[0].clone(); before_n = n_valid.clone()
    q = _new_token(w, device, 50, 0, (2, 4, 128)); kn = _new_token(w, device, 50, 1, (2, 2, 128)); vn = _new_token(w, device, 50, 2, (2, 2, 128))
    W.wkv_decode_step(shape, q, kn, vn, st.k_out[0], st.v_out[0], n_valid, out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out[0]).all()) and not bool(torch.isnan(out[1]).any())
    assert torch.equal(n_valid[0], before_n[0]) and torch.equal(n_valid[1], before_n[1] + 1)
    assert torch.equal(st.k_out[0][0], before_k[0])


def test_decode_strided_cache_and_explicit_scale(device):
    # token-major caches [B, capacity, Hkv, d] and a caller-chosen logit scale; hand-made rows, no compression
    rng_seed, B, H, G, d, cap = 94, 2, 3, 2, 64, 300
    w = S.Workload(name="dec_strided", seed=rng_seed, dtype="bf16", n_groups=1, gamma=1, n_q_heads=H * G, n_kv_heads=H,
                   head_dim=d, w_obs=4, seq_len=[64], win=[8], top_p=[8], k_windows=[1])     # only the generator's seed and dtype are used
    kc = _new_token(w, device, 100, 0, (B, cap, H, d)); vc = _new_token(w, device, 100, 1, (B, cap, H, d))
    n0 = torch.tensor([[257, 0, 13], [299, 64, 1]], dtype=torch.int32, device=device)       # includes an empty cache and a nearly full one
    n_valid = n0.clone()
    shape = W.DecodeShape(batch=B, n_q_heads=H * G, n_kv_heads=H, head_dim=d, capacity=cap, dtype=W.WKV_BF16, scale=0.37,
                          cache_strides=(cap * H * d, d, H * d))
    ws = torch.empty(W.wkv_decode_workspace_bytes(shape), dtype=torch.uint8, device=device)
    out = torch.empty((B, H * G, d), dtype=torch.float32, device=device)
    q = _new_token(w, device, 101, 0, (B, H * G, d)); kn = _new_token(w, device, 101, 1, (B, H, d)); vn = _new_token(w, device, 101, 2, (B, H, d))
    k_before, v_before = kc.clone(), vc.clone()
    W.wkv_decode_step(shape, q, kn, vn, kc, vc, n_valid, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(n_valid, n0 + 1)
    for b, h in itertools.product(range(B), range(H)):
        n = int(n0[b, h])
        want, _, _ = O.decode_step(P.host_f64(w, q[b, h * G:(h + 1) * G]), P.host_f64(w, k_before[b, :n, h]),
                                   P.host_f64(w, v_before[b, :n, h]), P.host_f64(w, kn[b, h]), P.host_f64(w, vn[b, h]), scale=0.37)
        np.testing.assert_allclose(out[b, h * G:(h + 1) * G].cpu().numpy(), want, rtol=RTOL, atol=ATOL, err_msg=f"b{b} h{h}")
        k_before[b, n, h] = kn[b, h]; v_before[b, n, h] = vn[b, h]
    assert torch.equal(k_before, kc) and torch.equal(v_before, vc)
