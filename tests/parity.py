"""Helpers of the GPU parity tests: run the HIP path through the C ABI, run the CPU oracle on the
same seeded inputs, and compare to the stated bar:

  * token scores t and window scores s: 2e-3 relative (bf16/fp32 inputs, fp32 accumulation)
  * window indices, token indices, gathered K/V: bit-exact, except that windows whose oracle
    score lies within 1e-4 relative of the oracle's k-th score may be swapped among themselves
    (fp32 versus fp64 can order such near-ties differently); the count must still be k and the
    gather must be exact for the indices the GPU chose.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2503_17922_amd as W
import wkv_synth as S
from oracle import wkv_oracle as O

RTOL_SCORE = 2e-3
ATOL_SCORE = 1e-12
TIE_BAND = 1e-4


def make_problem(w: S.Workload, **kw) -> W.Problem:
    return W.Problem(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, w_obs=w.w_obs,
                     seq_len=w.seq_len, win=w.win, top_p=w.top_p, k_windows=w.k_windows,
                     dtype=W.WKV_F32 if w.dtype == "f32" else W.WKV_BF16, max_seq_len=w.max_seq_len, **kw)


class DeviceState:
    """All device tensors of one workload plus the outputs of one wkv_compress_groups call."""

    def __init__(self, w: S.Workload, device, layers=True, flags=0):
        self.w = w
        self.device = device
        self.problem = make_problem(w, flags=flags)
        self.dims = W.wkv_get_dims(self.problem)
        self.q = [w.q_obs_torch(g, device) for g in range(w.n_groups)]
        self.k = [w.kv_torch(S.KIND_K, l, device) for l in range(w.n_layers)]
        self.v = [w.kv_torch(S.KIND_V, l, device) for l in range(w.n_layers)]
        B, H, d = w.batch, w.n_kv_heads, w.head_dim
        nk = self.dims.nkeep_max
        dt = self.k[0].dtype
        # outputs start from a non-zero pattern so that missing writes are visible
        self.k_out = [torch.full((B, H, nk, d), 7.0, dtype=dt, device=device) for _ in range(w.n_layers)]
        self.v_out = [torch.full((B, H, nk, d), 7.0, dtype=dt, device=device) for _ in range(w.n_layers)]
        G = w.n_groups
        self.win_idx = torch.full((G, B, H, max(self.dims.k_max, 1)), -7, dtype=torch.int32, device=device)
        self.tok_idx = torch.full((G, B, H, nk), -7, dtype=torch.int32, device=device)
        self.n_keep = torch.full((G, B, H), -7, dtype=torch.int32, device=device)
        self.ws_bytes = W.wkv_workspace_bytes(self.problem, G)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)

    def compress(self, lse=None, k_groups=None):
        """``lse``: None, or one float32 [B, Hq, w_obs] device tensor per group (normaliser hand-over).
        ``k_groups``: None, or [n_groups][batch] windows to keep per group."""
        w = self.w
        W.wkv_compress_groups(self.problem, w.n_groups, w.gamma, self.q, lse, self.k, self.v, self.k_out, self.v_out,
                              self.win_idx, self.tok_idx, self.n_keep, self.workspace, k_windows_groups=k_groups)
        torch.cuda.synchronize()

    def oracle_lse(self, g: int) -> torch.Tensor:
        """The oracle's ln-sum-exp of every observation row of group g, as the float32 device tensor
        [B, Hq, w_obs] a prefill attention kernel would hand over."""
        w = self.w
        G = w.q_per_kv
        out = np.zeros((w.batch, w.n_q_heads, w.w_obs), dtype=np.float64)
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                k = host_f64(w, self.k[g * w.gamma][b, h, : w.seq_len[b]])
                for gq in range(G):
                    out[b, h * G + gq] = O.softmax_lse(host_f64(w, self.q[g][b, h * G + gq]), k)
        return torch.from_numpy(out.astype(np.float32)).to(self.device)

    def stages(self, g: int, lse=None):
        """The four stage calls on group g; returns (t, s, win_idx, tok_idx, n_keep) tensors."""
        w, d = self.w, self.dims
        B, H = w.batch, w.n_kv_heads
        dev = self.device
        t = torch.full((B, H, max(d.t_stride, 1)), -3.0, dtype=torch.float32, device=dev)
        s = torch.full((B, H, max(d.nw_max, 1)), -3.0, dtype=torch.float32, device=dev)
        wi = torch.full((B, H, max(d.k_max, 1)), -7, dtype=torch.int32, device=dev)
        ti = torch.full((B, H, d.nkeep_max), -7, dtype=torch.int32, device=dev)
        nk = torch.full((B, H), -7, dtype=torch.int32, device=dev)
        ws = torch.empty(W.wkv_workspace_bytes(self.problem, 1), dtype=torch.uint8, device=dev)
        W.wkv_score(self.problem, self.q[g], self.k[g * w.gamma], lse, t, ws)
        W.wkv_window_pool(self.problem, t, s)
        W.wkv_topk_windows(self.problem, s, wi, ti, nk)
        torch.cuda.synchronize()
        return t, s, wi, ti, nk


def host_f64(w: S.Workload, x: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of a device/host tensor in the workload dtype."""
    return x.detach().to("cpu").to(torch.float64).numpy()


def oracle_problem(w: S.Workload, q_dev: torch.Tensor, k_dev: torch.Tensor, b: int, h: int):
    """Oracle results for (sequence b, KV head h) of the group whose first-layer tensors are
    q_dev [B,Hq,w_obs,d] and k_dev [B,Hkv,Lmax,d] (as produced by the shared generator)."""
    G, L = w.q_per_kv, w.seq_len[b]
    q = host_f64(w, q_dev[b, h * G:(h + 1) * G])
    k = host_f64(w, k_dev[b, h, :L])
    return O.select_indices(q, k, w.win[b], w.top_p[b], w.k_windows[b])


def check_generator_matches(w: S.Workload, kind: int, layer: int, dev_tensor: torch.Tensor, b: int, h: int,
                            rows=(0, 1, 17)):
    """The device tensor (torch form of the generator) equals the numpy form on sampled rows."""
    rows = np.array([r for r in rows if r < w.seq_len[b]] + [w.seq_len[b] - 1])
    want = w.kv_np(kind, layer, b, h, rows)
    got = dev_tensor[b, h, torch.from_numpy(rows).to(dev_tensor.device)].cpu()
    got = got.numpy() if w.dtype == "f32" else got.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want), "device generator differs from host generator"


def assert_scores_close(got: np.ndarray, want: np.ndarray, what: str):
    err = np.abs(got - want)
    tol = RTOL_SCORE * np.abs(want) + ATOL_SCORE
    if not np.all(err <= tol):
        i = int(np.argmax(err - tol))
        raise AssertionError(f"{what}: element {i}: got {got[i]!r}, oracle {want[i]!r}, "
                             f"rel err {err[i] / max(abs(want[i]), 1e-300):.3e}")


def check_selection(s_oracle: np.ndarray, sel_oracle: np.ndarray, sel_gpu: np.ndarray, k: int, what: str) -> bool:
    """Tie-aware comparison of the selected windows.  Returns True when the sets are identical."""
    sel_gpu = np.asarray(sel_gpu, dtype=np.int64)
    assert len(sel_gpu) == k, f"{what}: {len(sel_gpu)} windows selected, budget says {k}"
    if k == 0:
        return True
    assert np.all(np.diff(sel_gpu) > 0), f"{what}: window indices not strictly ascending"
    assert sel_gpu[0] >= 0 and sel_gpu[-1] < len(s_oracle), f"{what}: window index out of range"
    if np.array_equal(sel_gpu, sel_oracle):
        return True
    kth = np.sort(s_oracle)[::-1][k - 1]
    band = np.abs(s_oracle - kth) <= TIE_BAND * abs(kth)
    a = set(int(x) for x in sel_gpu if not band[x])
    o = set(int(x) for x in sel_oracle if not band[x])
    assert a == o, (f"{what}: selections differ outside the tie band: gpu-only {sorted(a - o)[:8]}, "
                    f"oracle-only {sorted(o - a)[:8]}")
    return False


def check_indices_structure(w: S.Workload, b: int, win_row, tok_row, n_keep: int, k_max: int, nkeep_max: int, what: str):
    """win_idx / tok_idx / n_keep of one (b, h) are consistent with each other and padded."""
    k, L = w.k_windows[b], w.seq_len[b]
    win_row = np.asarray(win_row); tok_row = np.asarray(tok_row)
    sel = win_row[:k]
    assert np.all(win_row[k:] == -1), f"{what}: win_idx padding"
    want_tok = O.token_indices(sel, w.win[b], L, w.w_obs)
    assert n_keep == len(want_tok), f"{what}: n_keep {n_keep} != {len(want_tok)}"
    assert np.array_equal(tok_row[:n_keep], want_tok), f"{what}: tok_idx is not the expansion of win_idx"
    assert np.all(tok_row[n_keep:] == -1), f"{what}: tok_idx padding"
    return sel
