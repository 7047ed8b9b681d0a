"""wkv_decode_step_static (the entry point that allocates nothing: its scratch memory is a static
array of the library's device image) against wkv_decode_step with a caller workspace, through the
C ABI: two calls in a row, the second on a smaller input, must reproduce the other entry point's
outputs bit for bit (same kernels, same summation order), and a shape beyond the static array is
refused."""
import pytest
import torch

import paper_2503_17922_amd as W

pytestmark = pytest.mark.gpu


def _case(device, batch, n_rows, seed, dtype=torch.bfloat16, Hq=32, H=8, d=128):
    g = torch.Generator(device=device).manual_seed(seed)
    cap = n_rows + 8
    mk = lambda *shape: torch.randn(shape, device=device, dtype=torch.float32, generator=g).to(dtype)
    kc, vc = mk(batch, H, cap, d), mk(batch, H, cap, d)
    q, kn, vn = mk(batch, Hq, d), mk(batch, H, d), mk(batch, H, d)
    n_valid = torch.randint(max(n_rows - 300, 1), n_rows + 1, (batch, H), device=device, generator=g, dtype=torch.int32)
    shape = W.DecodeShape(batch=batch, n_q_heads=Hq, n_kv_heads=H, head_dim=d, capacity=cap,
                          dtype=W.WKV_BF16 if dtype == torch.bfloat16 else W.WKV_F32)
    return shape, q, kn, vn, kc, vc, n_valid


def _both(device, batch, n_rows, seed, **kw):
    shape, q, kn, vn, kc, vc, n_valid = _case(device, batch, n_rows, seed, **kw)
    kc2, vc2, nv2 = kc.clone(), vc.clone(), n_valid.clone()
    out = torch.full((batch, q.shape[1], q.shape[2]), -3.0, dtype=torch.float32, device=device)
    out2 = torch.full_like(out, -4.0)
    ws = torch.empty(W.wkv_decode_workspace_bytes(shape), dtype=torch.uint8, device=device)
    assert ws.numel() <= W.WKV_DECODE_STATIC_SCRATCH_BYTES
    W.wkv_decode_step(shape, q, kn, vn, kc, vc, n_valid, out, ws)
    W.wkv_decode_step_static(shape, q, kn, vn, kc2, vc2, nv2, out2)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    assert torch.equal(out, out2), "outputs differ from the entry point with a caller workspace"
    assert torch.equal(kc, kc2) and torch.equal(vc, vc2) and torch.equal(n_valid, nv2)


def test_static_scratch_entry_matches_workspace_entry_on_two_calls_in_a_row(device):
    _both(device, batch=16, n_rows=4128, seed=1)        # 128 (sequence, KV head) rows, 8 key ranges each
    _both(device, batch=2, n_rows=700, seed=2)          # smaller: fewer rows, other range count, stale partials beside it
    _both(device, batch=3, n_rows=333, seed=3, dtype=torch.float32, Hq=4, H=2, d=64)


def test_static_scratch_entry_refuses_shapes_beyond_its_array(device):
    shape, q, kn, vn, kc, vc, n_valid = _case(device, batch=2, n_rows=64, seed=4)
    big = W.DecodeShape(batch=4000, n_q_heads=32, n_kv_heads=8, head_dim=128, capacity=72, dtype=W.WKV_BF16)
    assert W.wkv_decode_workspace_bytes(big) > W.WKV_DECODE_STATIC_SCRATCH_BYTES
    out = torch.zeros((2, 32, 128), dtype=torch.float32, device=device)
    with pytest.raises(W.WkvError) as e:
        W.wkv_decode_step_static(big, q, kn, vn, kc, vc, n_valid, out)
    assert e.value.status == W.WKV_ERR_WORKSPACE
