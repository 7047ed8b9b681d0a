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
from paper_2503_17922_amd import synthetic as _synthetic
from paper_2503_17922_amd.synthetic import make_problem, host_f64   # re-exported for the tests

RTOL_SCORE = 2e-3
ATOL_SCORE = 1e-12
TIE_BAND = 1e-4


class DeviceState(_synthetic.DeviceState):
    """The shared device state plus what only the tests need: the oracle's normalisers."""

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
