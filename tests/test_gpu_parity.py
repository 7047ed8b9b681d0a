"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded
inputs — the five named configurations at full size plus edge cases."""
import itertools

import numpy as np
import pytest
import torch

import paper_2503_17922_amd as W
import wkv_synth as S
from oracle import wkv_oracle as O
from tests import parity as P

pytestmark = pytest.mark.gpu


def _sample(items, n, seed):
    items = list(items)
    if n is None or n >= len(items):
        return items
    rng = np.random.default_rng(seed)
    pick = rng.choice(len(items), size=n, replace=False)
    return [items[i] for i in sorted(pick)]


def batched_intermediates(st):
    """What the batched call left in its workspace: (t or None, s or None) as float64 host arrays
    [G, B, H, t_stride] / [G, B, H, nw_max] (the library says which of the two it writes)."""
    w, d = st.w, st.dims
    lay = W.wkv_get_workspace_layout(st.problem, w.n_groups)
    assert lay.t_written + lay.s_written == 1
    rows = w.n_groups * w.batch * w.n_kv_heads

    def view(offset, cols):
        n = rows * max(cols, 1)
        x = st.workspace[offset: offset + 4 * n].view(torch.float32).view(w.n_groups, w.batch, w.n_kv_heads, max(cols, 1))
        with np.errstate(invalid="ignore"):          # entries past a row's end are whatever the workspace held
            return x.cpu().numpy().astype(np.float64)
    return (view(lay.t_offset, d.t_stride) if lay.t_written else None,
            view(lay.s_offset, d.nw_max) if lay.s_written else None)


def run_and_check(w: S.Workload, device, n_oracle=None, n_gather_cpu=None, stage_groups=None, as_f16=False, flags=0):
    """One wkv_compress_groups call checked against the oracle.

    n_oracle: how many (group, b, h) problems the oracle recomputes (None = all).
    n_gather_cpu: how many (layer, K|V, b, h) slices are compared on the CPU with the oracle's
    gather (None = all); every slice is additionally compared on the device.
    stage_groups: the groups whose four stage calls are run and compared too (None = all).
    For every oracle problem the token scores t and window scores s of the stage calls AND what the
    batched call itself computed (its s, or its t when it pools in the selection kernel, read back
    from the workspace) are compared element by element.
    """
    st = P.DeviceState(w, device, as_f16=as_f16, flags=flags)
    print(f"[{w.name}] L={w.seq_len} win={w.win} p={w.top_p} k={w.k_windows} groups={w.n_groups}x{w.gamma} "
          f"ws={st.ws_bytes >> 10} KiB", flush=True)
    if not as_f16 and w.dtype != "f16":
        P.check_generator_matches(w, S.KIND_K, 0, st.k[0], 0, 0)
        P.check_generator_matches(w, S.KIND_V, w.n_layers - 1, st.v[-1], w.batch - 1, w.n_kv_heads - 1)
    k_before = st.k[0][0, 0, : min(64, w.seq_len[0])].clone()
    st.compress()
    assert torch.equal(k_before, st.k[0][0, 0, : min(64, w.seq_len[0])]), "inputs were modified"
    t_fused, s_fused = batched_intermediates(st)

    win_idx = st.win_idx.cpu().numpy()[..., : st.dims.k_max]          # (allocated with >= 1 column)
    tok_idx = st.tok_idx.cpu().numpy(); n_keep = st.n_keep.cpu().numpy()
    B, H = w.batch, w.n_kv_heads

    # ---- stage calls reproduce the batched call bit for bit, and expose t and s ----------------
    stage_groups = list(range(w.n_groups)) if stage_groups is None else list(stage_groups)
    t_stage, s_stage = {}, {}
    for g0 in stage_groups:
        t_dev, s_dev, wi, ti, nk = st.stages(g0)
        assert np.array_equal(wi.cpu().numpy()[..., : st.dims.k_max], win_idx[g0]) and np.array_equal(ti.cpu().numpy(), tok_idx[g0])
        assert np.array_equal(nk.cpu().numpy(), n_keep[g0])
        # the gather stage, one layer at a time (as prefill would produce them), equals the batched gather
        for l in range(g0 * w.gamma, (g0 + 1) * w.gamma):
            ko = torch.full_like(st.k_out[l], 9.0); vo = torch.full_like(st.v_out[l], 9.0)
            W.wkv_gather_group(st.problem, [st.k[l]], [st.v[l]], ti, nk, [ko], [vo])
            torch.cuda.synchronize()
            assert torch.equal(ko, st.k_out[l]) and torch.equal(vo, st.v_out[l]), f"{w.name}: stage gather of layer {l}"
        t_stage[g0] = t_dev.cpu().numpy().astype(np.float64)[..., : st.dims.t_stride]
        s_stage[g0] = s_dev.cpu().numpy().astype(np.float64)[..., : st.dims.nw_max]

    # ---- structure of every index row -------------------------------------------------------------
    sels = {}
    for g, b, h in itertools.product(range(w.n_groups), range(B), range(H)):
        sels[g, b, h] = P.check_indices_structure(w, b, win_idx[g, b, h], tok_idx[g, b, h], int(n_keep[g, b, h]),
                                                  st.dims.k_max, st.dims.nkeep_max, f"{w.name} g{g} b{b} h{h}")

    # ---- oracle on (sampled) problems ----------------------------------------------------------------
    problems = _sample(itertools.product(range(w.n_groups), range(B), range(H)), n_oracle, 1)
    exact = 0
    for g, b, h in problems:
        t, s, sel, idx = P.oracle_problem(w, st.q[g], st.k[g * w.gamma], b, h)
        what = f"{w.name} g{g} b{b} h{h}"
        n_rev = w.seq_len[b] - w.w_obs
        if g in t_stage:
            P.assert_scores_close(t_stage[g][b, h, :n_rev], t, what + " t (stage call)")
            assert np.all(t_stage[g][b, h, n_rev:] == 0.0), what + " t padding"
            P.assert_scores_close(s_stage[g][b, h, : len(s)], s, what + " s (stage call)")
            assert np.all(np.isneginf(s_stage[g][b, h, len(s):])), what + " s padding"
        if s_fused is not None:
            P.assert_scores_close(s_fused[g, b, h, : len(s)], s, what + " s (batched call)")
        if t_fused is not None and n_rev > 0:
            P.assert_scores_close(t_fused[g, b, h, :n_rev], t, what + " t (batched call)")
        same = P.check_selection(s, sel, sels[g, b, h], w.k_windows[b], what)
        exact += same
        if same:
            assert np.array_equal(tok_idx[g, b, h, : len(idx)], idx), what + " tok_idx"
    print(f"[{w.name}] oracle problems: {len(problems)} of {w.n_groups * B * H}, identical selections: {exact}", flush=True)

    # ---- gather: every layer, bit exact ----------------------------------------------------------------
    slices = list(itertools.product(range(w.n_layers), (S.KIND_K, S.KIND_V), range(B), range(H)))
    for l, kind, b, h in _sample(slices, n_gather_cpu, 2):
        g = l // w.gamma
        src = (st.k if kind == S.KIND_K else st.v)[l]
        out = (st.k_out if kind == S.KIND_K else st.v_out)[l]
        n = int(n_keep[g, b, h])
        rows = src[b, h, : w.seq_len[b]].cpu()
        rows = rows.numpy() if w.dtype == "f32" else rows.view(torch.int16).numpy()
        got = out[b, h].cpu()
        got = got.numpy() if w.dtype == "f32" else got.view(torch.int16).numpy()
        want = O.gather_rows(rows, tok_idx[g, b, h, :n])
        assert np.array_equal(got[:n], want), f"{w.name} gather layer {l} kind {kind} b{b} h{h}"
        assert not got[n:].any(), f"{w.name} gather zero padding layer {l} b{b} h{h}"
    for l in range(w.n_layers):          # all slices, compared in device memory
        g = l // w.gamma
        for b in range(B):
            idx_dev = st.tok_idx[g, b].to(torch.int64)
            for src, out in ((st.k[l], st.k_out[l]), (st.v[l], st.v_out[l])):
                for h in range(H):
                    n = int(n_keep[g, b, h])
                    assert torch.equal(out[b, h, :n], src[b, h].index_select(0, idx_dev[h, :n]))
                    assert not out[b, h, n:].any()
    return st, sels


# ---------------------------------------------------------------------------------------
# the named configurations, full size
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c1", "c2", "c3a", "c3b"])
def test_config_small(name, device):
    run_and_check(S.make_workload(name), device)


def test_config_c4_full_model(device):
    w = S.make_workload("c4")
    st, sels = run_and_check(w, device, n_gather_cpu=12)          # the oracle on all 64 (group, KV head) problems
    # every window inside a planted span is kept, in every KV head of every scoring layer
    for (g, b, h), sel in sels.items():
        kept = set(int(x) for x in sel)
        for s0 in w.span_starts()[b]:
            want = set(range(s0 // w.win[b], (s0 + w.span_len) // w.win[b]))
            assert want <= kept, f"planted span at {s0} not kept in g{g} h{h}"


def test_config_c4_eight_query_heads_per_kv_head(device):
    # the 32K configuration with 64 query heads on 8 KV heads (70B-class): 256 softmax rows per KV
    # head, the two-half workgroups at their full chunk plan (3 groups of 2 layers keep it light)
    w = S.scaled_workload(S.make_workload("c4"), name="c4g8", n_q_heads=64, n_groups=3, gamma=2)
    run_and_check(w, device, n_gather_cpu=8)


def test_config_c5_batched_mixed(device):
    w = S.make_workload("c5")
    run_and_check(w, device, n_gather_cpu=16)                     # the oracle on all 512 (group, sequence, KV head) problems


def test_longest_supported_window_count(device):
    # 32768 windows per sequence (the library's limit) = a 262 176-token prefix at window size 8:
    # 128 KB of selection keys in LDS, 94 key chunks per row in the score passes
    w = S.Workload(name="long", seed=1006, dtype="bf16", n_groups=1, gamma=1, n_q_heads=32, n_kv_heads=8, head_dim=128,
                   w_obs=32, seq_len=[8 * 32768 + 32], win=[8], top_p=[8], k_windows=[3000])
    assert W.wkv_get_dims(P.make_problem(w)).nw_max == W.WKV_MAX_WINDOWS
    run_and_check(w, device, n_gather_cpu=4)
    with pytest.raises(W.WkvError) as e:                 # one window more is refused on the host
        W.wkv_get_dims(P.make_problem(S.scaled_workload(w, seq_len=[8 * 32768 + 33])))
    assert e.value.status == W.WKV_ERR_UNSUPPORTED


# ---------------------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------------------
def _mini(**kw):
    base = dict(name="mini", seed=77, dtype="bf16", n_groups=2, gamma=2, n_q_heads=8, n_kv_heads=2, head_dim=128,
                w_obs=16, seq_len=[700], win=[8], top_p=[8], k_windows=[10])
    base.update(kw)
    return S.Workload(**base)


@pytest.mark.parametrize("kw", [
    dict(),                                                               # ragged: 684 review tokens, tail of 4
    dict(seq_len=[700], win=[8], k_windows=[86]),                         # keep every window incl. the partial one
    dict(seq_len=[700], k_windows=[0]),                                   # keep only the observation window
    dict(seq_len=[16], k_windows=[0]),                                    # no review context at all
    dict(seq_len=[17], win=[8], k_windows=[1]),                           # one review token
    dict(seq_len=[1000, 16, 333, 2048], win=[8, 8, 32, 128], top_p=[4, 8, 1, 64], k_windows=[20, 0, 3, 5]),
    dict(win=[1], top_p=[1], k_windows=[100]),                            # token-level selection
    dict(win=[128], top_p=[128], k_windows=[2]),
    dict(win=[24], top_p=[7], k_windows=[9]),                             # window size not a power of two
    dict(n_q_heads=6, n_kv_heads=2, w_obs=5),                             # 15 softmax rows
    dict(n_q_heads=12, n_kv_heads=2, w_obs=4, seq_len=[5000], k_windows=[30]),    # Qwen-like G=6, alpha=4
    dict(n_q_heads=4, n_kv_heads=4, w_obs=1),                             # a single observation query per head
    dict(head_dim=64, seq_len=[3000], k_windows=[40]),
    dict(n_q_heads=16, n_kv_heads=2, w_obs=32, seq_len=[1500]),           # 256 rows: two row halves per workgroup
    dict(n_q_heads=10, n_kv_heads=2, w_obs=32, seq_len=[9000, 700], win=[16, 8], top_p=[8, 8], k_windows=[40, 9]),   # 160 rows, several chunks
    dict(n_q_heads=16, n_kv_heads=2, w_obs=32, head_dim=64, seq_len=[2500], win=[24], top_p=[5], k_windows=[17]),     # 256 rows, d=64, pooling in the selection kernel
    dict(n_q_heads=14, n_kv_heads=2, w_obs=19, seq_len=[3100]),           # 133 rows: 9 row tiles
    dict(dtype="f32", head_dim=128, seq_len=[900]),
    dict(dtype="f32", head_dim=64, n_q_heads=4, n_kv_heads=1, w_obs=64, seq_len=[600]),
    dict(n_groups=1, gamma=1, seq_len=[4097], win=[16], top_p=[8], k_windows=[31]),
    dict(n_groups=1, gamma=1, seq_len=[20016], win=[1], top_p=[1], k_windows=[700]),   # 20000 windows: >48 KB of LDS keys
])
def test_edge_cases(kw, device):
    run_and_check(_mini(**kw), device)


def test_largest_batch(device):
    # 64 sequences in one call (the library's limit), lengths 16 .. 646, alternating task modes
    B = W.WKV_MAX_BATCH
    seq_len = [16 + 10 * b for b in range(B)]
    win = [8 if b % 2 else 16 for b in range(B)]
    top_p = [8 if b % 2 else 5 for b in range(B)]
    k = [min((seq_len[b] - 16) // win[b], 1 + b % 7) for b in range(B)]
    w = S.Workload(name="b64", seed=1064, dtype="bf16", n_groups=2, gamma=1, n_q_heads=4, n_kv_heads=2, head_dim=64,
                   w_obs=16, seq_len=seq_len, win=win, top_p=top_p, k_windows=k)
    run_and_check(w, device)
    with pytest.raises(W.WkvError) as e:
        W.wkv_get_dims(P.make_problem(S.scaled_workload(w, seq_len=seq_len + [100], win=win + [8], top_p=top_p + [8],
                                                        k_windows=k + [1])))
    assert e.value.status == W.WKV_ERR_UNSUPPORTED


def _random_workload(i):
    """A seeded draw from the supported shape space (small enough for the oracle)."""
    rng = np.random.default_rng(4242 + i)
    d = int(rng.choice([64, 128]))
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
    w_obs = int(rng.integers(1, min(64, W.WKV_MAX_OBS_ROWS // G) + 1))
    B = int(rng.choice([1, 1, 2, 3]))
    seq_len, win, top_p, k = [], [], [], []
    for _ in range(B):
        L = w_obs + int(rng.choice([0, 1, int(rng.integers(2, 300)), int(rng.integers(300, 3000))]))
        wn = int(rng.choice([1, 2, 4, 8, 16, 32, 64, 128, int(rng.integers(1, 129))]))
        nw = -(-(L - w_obs) // wn)
        seq_len.append(L); win.append(wn); top_p.append(int(rng.integers(1, wn + 1)))
        k.append(int(rng.choice([0, nw] + [int(rng.integers(0, nw + 1)) for _ in range(4)])))
    n_groups = int(rng.choice([1, 2, 3])); gamma = int(rng.choice([1, 2, 3]))
    return S.Workload(name=f"rand{i}", seed=9000 + i, dtype=dtype, n_groups=n_groups, gamma=gamma, n_q_heads=G * hkv,
                      n_kv_heads=hkv, head_dim=d, w_obs=w_obs, seq_len=seq_len, win=win, top_p=top_p, k_windows=k)


@pytest.mark.parametrize("i", range(24))
def test_random_shapes(i, device):
    run_and_check(_random_workload(i), device)


@pytest.mark.parametrize("kw", [
    dict(),                                                               # 128 rows, ragged tail
    dict(seq_len=[1000, 16, 333, 2048], win=[8, 8, 32, 128], top_p=[4, 8, 1, 64], k_windows=[20, 0, 3, 5]),
    dict(head_dim=64, seq_len=[3000], k_windows=[40]),
    dict(n_q_heads=16, n_kv_heads=2, w_obs=32, seq_len=[1500]),           # 256 rows
    dict(n_q_heads=6, n_kv_heads=2, w_obs=5),                             # 15 rows
])
def test_fp16_inputs(kw, device):
    # IEEE half tensors holding the values of the bf16 workload (all exactly representable)
    run_and_check(_mini(**kw), device, as_f16=True)


def test_fp16_config_c2(device):
    run_and_check(S.make_workload("c2"), device, as_f16=True)


@pytest.mark.parametrize("kw", [
    dict(),                                                               # 128 rows, ragged tail
    dict(n_q_heads=16, n_kv_heads=2, w_obs=32, seq_len=[2500, 900], win=[16, 8], top_p=[8, 8], k_windows=[20, 11]),   # 256 rows
    dict(head_dim=64, seq_len=[3000], win=[24], top_p=[7], k_windows=[40]),     # pooling in the selection kernel
])
def test_half_inputs_with_half_values(kw, device):
    # IEEE half tensors drawn as half: 11 significant bits, so the _f16 MFMA operands carry mantissa
    # bits that bf16-valued inputs never set
    w = _mini(dtype="f16", **kw)
    st, _ = run_and_check(w, device)
    assert not torch.equal(st.k[0].to(torch.bfloat16).to(torch.float16), st.k[0]), "the inputs fit bf16: not a test of half"


def test_half_values_config_c2_shape(device):
    run_and_check(S.scaled_workload(S.make_workload("c2"), name="c2h", dtype="f16"), device)


def test_single_group_entry_point(device):
    # wkv_compress_group (one group, the call Section 2.2 describes) gives what the batched call gives
    w = _mini(seq_len=[1500, 700], win=[8, 16], top_p=[8, 5], k_windows=[40, 9], n_groups=1, gamma=3)
    ref = P.DeviceState(w, device); ref.compress()
    st = P.DeviceState(w, device)
    W.wkv_compress_group(st.problem, w.gamma, st.q[0], None, st.k, st.v, st.k_out, st.v_out, st.win_idx[0], st.tok_idx[0],
                         st.n_keep[0], st.workspace)
    torch.cuda.synchronize()
    for a, b in zip((st.win_idx, st.tok_idx, st.n_keep, *st.k_out, *st.v_out),
                    (ref.win_idx, ref.tok_idx, ref.n_keep, *ref.k_out, *ref.v_out)):
        assert torch.equal(a, b)
    lse = st.oracle_lse(0)                      # and with the normalisers handed over
    ref.compress(lse=[lse])
    W.wkv_compress_group(st.problem, w.gamma, st.q[0], lse, st.k, st.v, st.k_out, st.v_out, st.win_idx[0], st.tok_idx[0],
                         st.n_keep[0], st.workspace)
    torch.cuda.synchronize()
    assert torch.equal(st.tok_idx, ref.tok_idx) and torch.equal(st.k_out[2], ref.k_out[2])


# ---------------------------------------------------------------------------------------
# the single-read score kernel (keys stay on chip between the statistics and the score phase)
# ---------------------------------------------------------------------------------------
SINGLE_READ_CASES = [
    dict(),                                                               # 3 slices per row, ragged tail
    dict(seq_len=[1000, 16, 333, 2048], win=[8, 8, 32, 128], top_p=[4, 8, 1, 64], k_windows=[20, 0, 3, 5]),
    dict(seq_len=[16], k_windows=[0]),                                    # no review context at all
    dict(seq_len=[17], win=[8], k_windows=[1]),                           # one review token
    dict(seq_len=[272, 256, 528], win=[8, 16, 8], top_p=[8, 8, 3], k_windows=[5, 7, 9]),   # review context ends exactly on slice boundaries
    dict(win=[24], top_p=[7], k_windows=[9]),                             # token scores to memory, pooled by the selection kernel
    dict(n_q_heads=6, n_kv_heads=2, w_obs=5),                             # 15 softmax rows
    dict(n_q_heads=4, n_kv_heads=4, w_obs=1),
    dict(head_dim=64, seq_len=[3000], k_windows=[40]),
    dict(n_groups=3, gamma=1, seq_len=[9000, 700, 4097], win=[16, 8, 16], top_p=[8, 8, 16], k_windows=[40, 9, 31]),   # 36 slices per row
    dict(n_q_heads=16, n_kv_heads=2, w_obs=32, seq_len=[1500]),           # 256 rows: not covered by this kernel, the flag is ignored
]


@pytest.mark.parametrize("kw", SINGLE_READ_CASES)
def test_single_read_kernel(kw, device):
    run_and_check(_mini(**kw), device, flags=W.WKV_SCORE_SINGLE_READ)


@pytest.mark.parametrize("kw", [SINGLE_READ_CASES[1], SINGLE_READ_CASES[5], SINGLE_READ_CASES[9]])
def test_single_read_kernel_gives_up_and_the_two_pass_kernels_take_over(kw, device):
    # every cross-workgroup wait of the single-read kernel is told to give up at once (a limit of
    # zero polls, set from the host): the kernel exits normally, raises its fall-back word, and
    # the two-pass kernels enqueued behind it recompute the scores
    w = _mini(**kw)
    run_and_check(w, device, flags=W.WKV_SCORE_SINGLE_READ | W.WKV_DEBUG_WAIT_GIVES_UP)
    ref = P.DeviceState(w, device, flags=W.WKV_SCORE_TWO_PASS); ref.compress()
    st = P.DeviceState(w, device, flags=W.WKV_SCORE_SINGLE_READ | W.WKV_DEBUG_WAIT_GIVES_UP); st.compress()
    assert torch.equal(ref.tok_idx, st.tok_idx) and torch.equal(ref.win_idx, st.win_idx)      # the very same kernels produced both


def test_single_read_kernel_on_the_mixed_batch_at_full_size(device):
    # c5 through the single-read kernel: 512 ragged rows of 16 .. 128 slices, ten rounds of the
    # persistent grid; every problem against the oracle, the batched call's own window scores included
    run_and_check(S.make_workload("c5"), device, n_gather_cpu=8, stage_groups=[2], flags=W.WKV_SCORE_SINGLE_READ)


def test_single_read_and_two_pass_agree_at_full_size(device):
    w = S.make_workload("c4")
    a = P.DeviceState(w, device, flags=W.WKV_SCORE_SINGLE_READ); a.compress()
    _, s_a = batched_intermediates(a)
    b = P.DeviceState(w, device, flags=W.WKV_SCORE_TWO_PASS); b.compress()
    _, s_b = batched_intermediates(b)
    nw = w.n_windows(0)
    np.testing.assert_allclose(s_a[..., :nw], s_b[..., :nw], rtol=1e-5)
    same = (a.win_idx == b.win_idx).all(dim=-1).float().mean().item()
    assert same > 0.9, f"only {same:.2f} of the rows select the same windows"


def test_large_logits_are_stable(device):
    # keys scaled so that logits reach hundreds: exponentials must never overflow
    w = _mini(seq_len=[2000], k_windows=[12], n_groups=1, gamma=1)
    st = P.DeviceState(w, device)
    st.k[0].mul_(24.0)
    st.compress()
    t_dev, s_dev, *_ = st.stages(0)
    assert torch.isfinite(t_dev).all()
    for h in range(w.n_kv_heads):
        t, s, sel, idx = P.oracle_problem(w, st.q[0], st.k[0], 0, h)
        got = t_dev[0, h, : len(t)].cpu().numpy().astype(np.float64)
        big = t > 1e-6 * t.max()
        P.assert_scores_close(got[big], t[big], f"large logits h{h}")
        assert np.all(got[~big] <= 2e-6 * t.max())
        P.check_selection(s, sel, st.win_idx[0, 0, h, : w.k_windows[0]].cpu().numpy(), w.k_windows[0], f"h{h}")


@pytest.mark.parametrize("direction", ["rising", "falling"])
def test_logit_scale_ramps_along_the_sequence(direction, device):
    # keys scaled by a factor that runs from 1 to 64 along the sequence (or back): the running
    # reference of the statistics pass is re-referenced many times (rising) or stays far above the
    # later logits (falling); several chunks per row, 128 and 256 softmax rows
    for heads in (8, 16):
        w = _mini(n_q_heads=heads, n_kv_heads=2, w_obs=32, seq_len=[6000], k_windows=[20], n_groups=1, gamma=1)
        st = P.DeviceState(w, device)
        L = w.seq_len[0]
        ramp = torch.linspace(0.0, 6.0, L, device=device).exp2()            # 1 .. 64
        if direction == "falling":
            ramp = ramp.flip(0)
        st.k[0] = (st.k[0].float() * ramp.view(1, 1, L, 1)).to(st.k[0].dtype)
        st.compress()
        t_dev, s_dev, *_ = st.stages(0)
        assert torch.isfinite(t_dev).all()
        for h in range(w.n_kv_heads):
            t, s, sel, idx = P.oracle_problem(w, st.q[0], st.k[0], 0, h)
            got = t_dev[0, h, : len(t)].cpu().numpy().astype(np.float64)
            big = t > 1e-6 * t.max()
            P.assert_scores_close(got[big], t[big], f"{direction} ramp, {heads} heads, h{h}")
            assert np.all(got[~big] <= 2e-6 * t.max())
            P.check_selection(s, sel, st.win_idx[0, 0, h, : w.k_windows[0]].cpu().numpy(), w.k_windows[0], f"h{h}")


def test_strided_layout(device):
    # K/V stored [B, L, Hkv, d] (token-major), q [B, w_obs, Hq, d], compact cache [B, n, Hkv, d]
    w = _mini(seq_len=[1234, 600], win=[8, 8], top_p=[8, 3], k_windows=[17, 9], n_groups=1, gamma=2)
    st = P.DeviceState(w, device)
    st.compress()
    B, H, Lm, d, Hq, a = w.batch, w.n_kv_heads, w.max_seq_len, w.head_dim, w.n_q_heads, w.w_obs
    nk = st.dims.nkeep_max
    prob = P.make_problem(w, q_strides=(a * Hq * d, d, Hq * d), kv_strides=(Lm * H * d, d, H * d),
                          out_strides=(nk * H * d, d, H * d))
    q2 = [q.permute(0, 2, 1, 3).contiguous() for q in st.q]
    k2 = [k.permute(0, 2, 1, 3).contiguous() for k in st.k]
    v2 = [v.permute(0, 2, 1, 3).contiguous() for v in st.v]
    ko = [torch.full((B, nk, H, d), 5.0, dtype=k.dtype, device=device) for k in st.k]
    vo = [torch.full((B, nk, H, d), 5.0, dtype=k.dtype, device=device) for k in st.k]
    wi, ti, nkp = torch.empty_like(st.win_idx), torch.empty_like(st.tok_idx), torch.empty_like(st.n_keep)
    W.wkv_compress_groups(prob, 1, 2, q2, None, k2, v2, ko, vo, wi, ti, nkp, st.workspace)
    torch.cuda.synchronize()
    assert torch.equal(wi, st.win_idx) and torch.equal(ti, st.tok_idx) and torch.equal(nkp, st.n_keep)
    for l in range(2):
        assert torch.equal(ko[l].permute(0, 2, 1, 3), st.k_out[l]) and torch.equal(vo[l].permute(0, 2, 1, 3), st.v_out[l])


def _check_lse_handoff(w, device, groups_oracle):
    """With the oracle's normalisers handed over, the score stage must meet the same bar as the
    two-pass path, and the batched call must pick what the two-pass call picks (up to near-ties)."""
    st = P.DeviceState(w, device)
    st.compress()
    base_win = st.win_idx.cpu().numpy()[..., : st.dims.k_max].copy()
    lse = [st.oracle_lse(g) if g in groups_oracle else None for g in range(w.n_groups)]
    B, H = w.batch, w.n_kv_heads
    for g in groups_oracle:
        t_dev, s_dev, wi, ti, nk = st.stages(g, lse=lse[g])
        t_two, _, wi_two, _, _ = st.stages(g)
        t_host = t_dev.cpu().numpy().astype(np.float64)
        for b, h in itertools.product(range(B), range(H)):
            t, s, sel, idx = P.oracle_problem(w, st.q[g], st.k[g * w.gamma], b, h)
            n_rev = w.seq_len[b] - w.w_obs
            P.assert_scores_close(t_host[b, h, :n_rev], t, f"{w.name} lse hand-over g{g} b{b} h{h} t")
            assert np.all(t_host[b, h, n_rev: st.dims.t_stride] == 0.0)
            got = wi.cpu().numpy()[b, h, : w.k_windows[b]]
            P.check_selection(s, sel, got, w.k_windows[b], f"{w.name} lse hand-over g{g} b{b} h{h}")
        # against the library's own two-pass scores: same values to fp32 rounding of the normaliser
        np.testing.assert_allclose(t_dev.cpu().numpy(), t_two.cpu().numpy(), rtol=2e-4, atol=1e-12)
    if len(groups_oracle) == w.n_groups:
        st.win_idx.fill_(-7); st.tok_idx.fill_(-7); st.n_keep.fill_(-7)
        for o in st.k_out + st.v_out:
            o.fill_(7.0)
        st.compress(lse=lse)
        win = st.win_idx.cpu().numpy()[..., : st.dims.k_max]
        tok = st.tok_idx.cpu().numpy(); nkeep = st.n_keep.cpu().numpy()
        differ = 0
        for g, b, h in itertools.product(range(w.n_groups), range(B), range(H)):
            P.check_indices_structure(w, b, win[g, b, h], tok[g, b, h], int(nkeep[g, b, h]), st.dims.k_max,
                                      st.dims.nkeep_max, f"{w.name} batched lse g{g} b{b} h{h}")
            t, s, sel, idx = P.oracle_problem(w, st.q[g], st.k[g * w.gamma], b, h)
            P.check_selection(s, sel, win[g, b, h, : w.k_windows[b]], w.k_windows[b], f"{w.name} batched lse g{g} b{b} h{h}")
            differ += not np.array_equal(win[g, b, h], base_win[g, b, h])
            n = int(nkeep[g, b, h])
            rows = torch.from_numpy(tok[g, b, h, :n].astype(np.int64)).to(device)
            for l in range(w.gamma):
                layer = g * w.gamma + l
                assert torch.equal(st.k_out[layer][b, h, :n], st.k[layer][b, h].index_select(0, rows))
                assert torch.equal(st.v_out[layer][b, h, :n], st.v[layer][b, h].index_select(0, rows))
        print(f"[{w.name}] lse hand-over: {differ} index rows differ from the two-pass call (near-ties only)", flush=True)


def test_lse_handoff_small_configs(device):
    _check_lse_handoff(S.make_workload("c1"), device, groups_oracle=[0])          # fp32, generic kernels
    _check_lse_handoff(S.make_workload("c2"), device, groups_oracle=[0])          # bf16, MFMA kernels, outlier channels
    w = _mini(seq_len=[777, 130, 2049], win=[8, 16, 32], top_p=[8, 5, 16], k_windows=[20, 3, 11], n_groups=2, gamma=2)
    _check_lse_handoff(w, device, groups_oracle=[0, 1])                           # ragged batch, two groups
    w = _mini(n_q_heads=16, n_kv_heads=2, w_obs=32, seq_len=[2100, 600], win=[8, 16], top_p=[8, 8], k_windows=[20, 5])
    _check_lse_handoff(w, device, groups_oracle=[0, 1])                           # 256 softmax rows per KV head


def test_lse_handoff_full_model(device):
    # the 32K configuration with the oracle's normalisers handed over for all 8 groups: the
    # selections must be the oracle's (near-ties aside) and the gather exact for what was selected
    w = S.make_workload("c4")
    st = P.DeviceState(w, device)
    lse = [st.oracle_lse(g) for g in range(w.n_groups)]
    st.compress(lse=lse)
    win = st.win_idx.cpu().numpy(); tok = st.tok_idx.cpu().numpy(); nkeep = st.n_keep.cpu().numpy()
    problems = list(itertools.product(range(w.n_groups), range(w.batch), range(w.n_kv_heads)))      # all 64
    for g, b, h in problems:
        P.check_indices_structure(w, b, win[g, b, h], tok[g, b, h], int(nkeep[g, b, h]), st.dims.k_max, st.dims.nkeep_max,
                                  f"c4 lse g{g} b{b} h{h}")
    _, s_fused = batched_intermediates(st)
    for g, b, h in problems:
        t, s, sel, idx = P.oracle_problem(w, st.q[g], st.k[g * w.gamma], b, h)
        P.assert_scores_close(s_fused[g, b, h, : len(s)], s, f"c4 lse g{g} b{b} h{h} s (batched call)")
        if P.check_selection(s, sel, win[g, b, h, : w.k_windows[b]], w.k_windows[b], f"c4 lse g{g} b{b} h{h}"):
            assert np.array_equal(tok[g, b, h, : len(idx)], idx)
        rows = torch.from_numpy(tok[g, b, h, : nkeep[g, b, h]].astype(np.int64)).to(device)
        for l in range(w.gamma):
            layer = g * w.gamma + l
            assert torch.equal(st.k_out[layer][b, h, : len(rows)], st.k[layer][b, h].index_select(0, rows))
            assert torch.equal(st.v_out[layer][b, h, : len(rows)], st.v[layer][b, h].index_select(0, rows))


def test_lse_handoff_rejects_partial_arrays(device):
    w = _mini(seq_len=[300], n_groups=2, gamma=1)
    st = P.DeviceState(w, device)
    with pytest.raises(W.WkvError) as e:
        st.compress(lse=[st.oracle_lse(0), None])
    assert e.value.status == W.WKV_ERR_INVALID_ARG


def test_pyramid_budgets_per_group(device):
    # Section 2.2.3: Eq. 5-7 budgets (lambda = 14) turned into whole windows per group (floor), the
    # lower groups keeping more; each group is checked against the oracle run with its own k.
    n_groups, lam = 4, 14.0
    seq_len, win = [3000, 1111], [8, 16]
    total = [0.12 * L * n_groups for L in seq_len]            # 12 % of the prefix per group on average
    budgets = [W.wkv_group_budgets(tb, n_groups, lam) for tb in total]
    k_groups = [[int(budgets[b][g] // win[b]) for b in range(2)] for g in range(n_groups)]
    assert k_groups[0][0] > k_groups[-1][0] > 0
    cap = [max(k_groups[g][b] for g in range(n_groups)) for b in range(2)]
    w = _mini(seq_len=seq_len, win=win, top_p=[8, 6], k_windows=cap, n_groups=n_groups, gamma=2)
    st = P.DeviceState(w, device)
    st.compress(k_groups=k_groups)
    win_idx = st.win_idx.cpu().numpy(); tok = st.tok_idx.cpu().numpy(); nkeep = st.n_keep.cpu().numpy()
    for g, b, h in itertools.product(range(n_groups), range(2), range(w.n_kv_heads)):
        k = k_groups[g][b]
        what = f"pyramid g{g} b{b} h{h}"
        G, L = w.q_per_kv, seq_len[b]
        t, s, sel, idx = O.select_indices(P.host_f64(w, st.q[g][b, h * G:(h + 1) * G]),
                                          P.host_f64(w, st.k[g * w.gamma][b, h, :L]), win[b], w.top_p[b], k)
        assert np.all(win_idx[g, b, h, k:] == -1), what + " win_idx padding"
        same = P.check_selection(s, sel, win_idx[g, b, h, :k], k, what)
        want_tok = O.token_indices(win_idx[g, b, h, :k], win[b], L, w.w_obs)
        n = int(nkeep[g, b, h])
        assert n == len(want_tok) and np.array_equal(tok[g, b, h, :n], want_tok) and np.all(tok[g, b, h, n:] == -1), what
        if same:
            assert np.array_equal(tok[g, b, h, :n], idx)
        rows = torch.from_numpy(tok[g, b, h, :n].astype(np.int64)).to(device)
        for l in range(w.gamma):
            layer = g * w.gamma + l
            assert torch.equal(st.k_out[layer][b, h, :n], st.k[layer][b, h].index_select(0, rows)), what
            assert torch.equal(st.v_out[layer][b, h, :n], st.v[layer][b, h].index_select(0, rows)), what
            assert not st.k_out[layer][b, h, n:].any() and not st.v_out[layer][b, h, n:].any(), what + " zero fill"


def test_keep_padding_flag(device):
    # WKV_KEEP_PADDING: identical indices and kept rows; rows past n_keep keep the caller's bytes
    w = _mini(seq_len=[1000, 16, 333, 2048], win=[8, 8, 32, 128], top_p=[4, 8, 1, 64], k_windows=[20, 0, 3, 5])
    ref = P.DeviceState(w, device); ref.compress()
    st = P.DeviceState(w, device, flags=W.WKV_KEEP_PADDING); st.compress()
    assert torch.equal(ref.tok_idx, st.tok_idx) and torch.equal(ref.n_keep, st.n_keep)
    n_keep = st.n_keep.cpu().numpy()
    padded = 0
    for l in range(w.n_layers):
        g = l // w.gamma
        for b, h in itertools.product(range(w.batch), range(w.n_kv_heads)):
            n = int(n_keep[g, b, h])
            for out, want in ((st.k_out[l], ref.k_out[l]), (st.v_out[l], ref.v_out[l])):
                assert torch.equal(out[b, h, :n], want[b, h, :n])
                assert bool((out[b, h, n:] == 7.0).all()), "padding rows were written"
                assert not want[b, h, n:].any()
            padded += st.dims.nkeep_max - n
    assert padded > 0
    # the stage call honours the flag too
    k_out = [torch.full_like(t, 3.0) for t in st.k_out[: w.gamma]]
    v_out = [torch.full_like(t, 3.0) for t in st.v_out[: w.gamma]]
    W.wkv_gather_group(st.problem, st.k[: w.gamma], st.v[: w.gamma], st.tok_idx[0], st.n_keep[0], k_out, v_out)
    torch.cuda.synchronize()
    for l in range(w.gamma):
        for b, h in itertools.product(range(w.batch), range(w.n_kv_heads)):
            n = int(n_keep[0, b, h])
            assert torch.equal(k_out[l][b, h, :n], ref.k_out[l][b, h, :n]) and bool((k_out[l][b, h, n:] == 3.0).all())
            assert torch.equal(v_out[l][b, h, :n], ref.v_out[l][b, h, :n]) and bool((v_out[l][b, h, n:] == 3.0).all())


def test_largest_group_count_with_budgets_of_their_own(device):
    # 64 groups of one layer (the library's limits for groups and layers), 16 sequences: 1024
    # (group, sequence) budgets, the size of the kernel-argument table
    n_groups, B = W.WKV_MAX_GROUPS, 16
    seq_len = [40 + 23 * b for b in range(B)]
    win = [4] * B
    nw = [-(-(L - 8) // 4) for L in seq_len]
    k_groups = [[(g * 7 + b * 3) % (nw[b] + 1) for b in range(B)] for g in range(n_groups)]
    cap = [max(k_groups[g][b] for g in range(n_groups)) for b in range(B)]
    w = S.Workload(name="g64", seed=1065, dtype="bf16", n_groups=n_groups, gamma=1, n_q_heads=2, n_kv_heads=1, head_dim=64,
                   w_obs=8, seq_len=seq_len, win=win, top_p=[3] * B, k_windows=cap)
    st = P.DeviceState(w, device)
    st.compress(k_groups=k_groups)
    win_idx = st.win_idx.cpu().numpy(); tok = st.tok_idx.cpu().numpy(); nkeep = st.n_keep.cpu().numpy()
    for g, b in itertools.product(range(n_groups), range(B)):
        k, L = k_groups[g][b], seq_len[b]
        what = f"g{g} b{b}"
        t, s, sel, idx = O.select_indices(P.host_f64(w, st.q[g][b, 0:2]), P.host_f64(w, st.k[g][b, 0, :L]), 4, 3, k)
        assert np.all(win_idx[g, b, 0, k:] == -1), what
        if P.check_selection(s, sel, win_idx[g, b, 0, :k], k, what):
            assert np.array_equal(tok[g, b, 0, : len(idx)], idx), what
        n = int(nkeep[g, b, 0])
        assert n == len(O.token_indices(win_idx[g, b, 0, :k], 4, L, 8)), what
        rows = torch.from_numpy(tok[g, b, 0, :n].astype(np.int64)).to(device)
        assert torch.equal(st.k_out[g][b, 0, :n], st.k[g][b, 0].index_select(0, rows)), what
        assert torch.equal(st.v_out[g][b, 0, :n], st.v[g][b, 0].index_select(0, rows)), what
    with pytest.raises(W.WkvError):          # one sequence more would not fit the budget table
        w2 = S.scaled_workload(w, seq_len=seq_len + [50], win=[4] * 17, top_p=[3] * 17, k_windows=cap + [1])
        st2 = P.DeviceState(w2, device)
        st2.compress(k_groups=[row + [0] for row in k_groups])


def test_other_layers_do_not_influence_indices(device):
    w = _mini(seq_len=[900], n_groups=1, gamma=3)
    st = P.DeviceState(w, device)
    st.compress()
    first = st.tok_idx.clone()
    st.k[1].normal_(); st.k[2].normal_(); st.v[0].normal_()
    st.compress()
    assert torch.equal(first, st.tok_idx)


def test_topk_ties_and_arbitrary_scores(device):
    # wkv_topk_windows alone on hand-made score rows: duplicates, negatives, zeros, -inf padding
    rng = np.random.default_rng(5)
    L, a, win = 8 * 300 + 16, 16, 8
    for k in (0, 1, 7, 150, 300):
        prob = W.Problem(n_q_heads=4, n_kv_heads=4, head_dim=64, w_obs=a, seq_len=[L], win=[win], top_p=[win],
                         k_windows=[k], dtype=W.WKV_BF16)
        s = np.stack([rng.integers(0, 12, 300).astype(np.float32) / 4 - 1,          # many exact ties
                      rng.standard_normal(300).astype(np.float32),
                      np.zeros(300, np.float32),
                      np.where(rng.random(300) < 0.5, np.float32(0.25), np.float32(-np.inf))])
        s_dev = torch.from_numpy(s).to(device)[None]
        wi = torch.empty((1, 4, max(k, 1)), dtype=torch.int32, device=device)
        ti = torch.empty((1, 4, k * win + a), dtype=torch.int32, device=device)
        nk = torch.empty((1, 4), dtype=torch.int32, device=device)
        W.wkv_topk_windows(prob, s_dev, wi, ti, nk)
        torch.cuda.synchronize()
        for h in range(4):
            want = O.select_windows(s[h].astype(np.float64), k)
            assert np.array_equal(wi[0, h, :k].cpu().numpy(), want), (k, h)
            assert np.array_equal(ti[0, h].cpu().numpy(), O.token_indices(want, win, L, a))
            assert int(nk[0, h]) == k * win + a


def test_window_pool_alone(device):
    rng = np.random.default_rng(6)
    a = 16
    for win, p, L in ((8, 8, 1000), (8, 3, 1001), (32, 16, 5000), (128, 17, 4000), (5, 2, 333), (1, 1, 100)):
        prob = W.Problem(n_q_heads=2, n_kv_heads=2, head_dim=64, w_obs=a, seq_len=[L], win=[win], top_p=[p],
                         k_windows=[0], dtype=W.WKV_BF16)
        t = rng.random((1, 2, L - a)).astype(np.float32)
        m = len(t[0, 1, 1::3])
        t[0, 1, ::3][:m] = t[0, 1, 1::3]                       # repeated values inside windows
        nw = -(-(L - a) // win)
        s_dev = torch.empty((1, 2, nw), dtype=torch.float32, device=device)
        W.wkv_window_pool(prob, torch.from_numpy(t).to(device), s_dev)
        torch.cuda.synchronize()
        for h in range(2):
            want = O.window_scores(t[0, h].astype(np.float64), win, p)
            np.testing.assert_allclose(s_dev[0, h].cpu().numpy(), want, rtol=2e-6)


def test_profiled_call_gives_the_same_results_and_sane_times(device):
    w = _mini(seq_len=[1500, 700], win=[8, 16], top_p=[8, 5], k_windows=[40, 9], n_groups=2, gamma=2)
    ref = P.DeviceState(w, device); ref.compress()
    st = P.DeviceState(w, device)
    call = W.CompressCall(st.problem, w.n_groups, w.gamma, st.q, None, st.k, st.v, st.k_out, st.v_out,
                          st.win_idx, st.tok_idx, st.n_keep, st.workspace)
    ms = call.profiled()
    torch.cuda.synchronize()
    assert len(ms) == W.WKV_N_STAGES == len(W.STAGE_NAMES)
    assert all(0.0 < x < 50.0 for x in ms), ms
    for a, b in zip((st.win_idx, st.tok_idx, st.n_keep, *st.k_out, *st.v_out),
                    (ref.win_idx, ref.tok_idx, ref.n_keep, *ref.k_out, *ref.v_out)):
        assert torch.equal(a, b)
    # with the normalisers handed over there is no statistics pass: its slot reads 0
    lse = [st.oracle_lse(g) for g in range(w.n_groups)]
    call = W.CompressCall(st.problem, w.n_groups, w.gamma, st.q, lse, st.k, st.v, st.k_out, st.v_out,
                          st.win_idx, st.tok_idx, st.n_keep, st.workspace)
    ms = call.profiled()
    assert ms[0] < 0.02 and ms[1] > 0.0, ms


def test_graph_capture_and_replay(device):
    # The batched call is plain kernel launches on the caller's stream (no allocation, no host
    # synchronisation, no memset nodes), so it can be captured into a HIP graph.  Replays with the
    # inputs changed in place must match eager calls on the same inputs, every time.
    w = _mini(seq_len=[1500, 700], win=[8, 16], top_p=[8, 5], k_windows=[40, 9], n_groups=2, gamma=2)
    st = P.DeviceState(w, device)
    call = W.CompressCall(st.problem, w.n_groups, w.gamma, st.q, None, st.k, st.v, st.k_out, st.v_out,
                          st.win_idx, st.tok_idx, st.n_keep, st.workspace)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(side.cuda_stream)                       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        # new inputs, same buffers: permute the tokens of the scored layers and of one value layer
        perm = torch.randperm(w.max_seq_len, device=device, generator=torch.Generator(device=device).manual_seed(rep))
        for g in range(w.n_groups):
            st.k[g * w.gamma].copy_(st.k[g * w.gamma][:, :, perm])
        st.v[1].copy_(st.v[1][:, :, perm])
        for o in st.k_out + st.v_out:
            o.fill_(3.0)
        st.tok_idx.fill_(-9); st.win_idx.fill_(-9); st.n_keep.fill_(-9)
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (st.win_idx, st.tok_idx, st.n_keep, *st.k_out, *st.v_out)]
        for o in st.k_out + st.v_out:
            o.fill_(5.0)
        st.tok_idx.fill_(-8); st.win_idx.fill_(-8); st.n_keep.fill_(-8)
        call()                                       # eager, default stream
        torch.cuda.synchronize()
        want = (st.win_idx, st.tok_idx, st.n_keep, *st.k_out, *st.v_out)
        for a, b_ in zip(got, want):
            assert torch.equal(a, b_), f"replay {rep} differs from the eager call"


def test_per_layer_selection_and_index_similarity(device):
    # Section 3.2: every layer selects on its own (gamma = 1); the Jaccard similarity of the retained
    # positions of every pair of layers.  Layers 1..3 are made to resemble layer 0 to different
    # degrees (a mix of its keys and queries with their own: plain tensor arithmetic on the inputs).
    n_layers = 4
    w = _mini(seq_len=[2000, 900], win=[8, 16], top_p=[8, 5], k_windows=[30, 10], n_groups=n_layers, gamma=1)
    st = P.DeviceState(w, device)
    for l, rho in ((1, 0.95), (2, 0.7), (3, 0.0)):
        a, b_ = rho, (1.0 - rho * rho) ** 0.5
        st.k[l].copy_((a * st.k[0].float() + b_ * st.k[l].float()).to(st.k[l].dtype))
        st.q[l].copy_((a * st.q[0].float() + b_ * st.q[l].float()).to(st.q[l].dtype))
    st.compress()
    B, H = w.batch, w.n_kv_heads
    out = torch.full((n_layers, n_layers, B, H), -1.0, dtype=torch.float32, device=device)
    W.wkv_index_jaccard(st.problem, n_layers, st.tok_idx, st.n_keep, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    tok = st.tok_idx.cpu().numpy(); nk = st.n_keep.cpu().numpy()
    for i, j, b, h in itertools.product(range(n_layers), range(n_layers), range(B), range(H)):
        want = O.jaccard(tok[i, b, h, : nk[i, b, h]], tok[j, b, h, : nk[j, b, h]])
        assert got[i, j, b, h] == pytest.approx(want, rel=1e-6), f"jaccard layers {i},{j} b{b} h{h}"
    # every layer's own selection is what the oracle selects for that layer alone
    for l, b, h in itertools.product(range(n_layers), range(B), range(H)):
        t, s, sel, idx = P.oracle_problem(w, st.q[l], st.k[l], b, h)
        P.check_selection(s, sel, st.win_idx.cpu().numpy()[l, b, h, : w.k_windows[b]], w.k_windows[b], f"layer {l} b{b} h{h}")
    mean = got.mean(axis=(2, 3))
    assert np.allclose(np.diag(mean), 1.0) and mean[0, 1] > mean[0, 2] > mean[0, 3], f"similarity should fall with the mixing weight: {mean[0]}"
