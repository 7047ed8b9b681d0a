"""Device-side state of a synthetic workload: the tensors of every layer, the output buffers and
the workspace of one ``wkv_compress_groups`` call.  Shared by the benchmark and the GPU tests;
no arithmetic of the method lives here (inputs come from the seeded generator ``wkv_synth``,
results from the HIP library)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2503_17922_amd as W
import wkv_synth as S


def make_problem(w: S.Workload, **kw) -> W.Problem:
    kw.setdefault("dtype", {"f32": W.WKV_F32, "bf16": W.WKV_BF16, "f16": W.WKV_F16}[w.dtype])
    return W.Problem(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, w_obs=w.w_obs,
                     seq_len=w.seq_len, win=w.win, top_p=w.top_p, k_windows=w.k_windows,
                     max_seq_len=w.max_seq_len, **kw)


def _exact_half(t: torch.Tensor) -> torch.Tensor:
    """The same values as IEEE half; refuses a tensor that half cannot hold exactly."""
    h = t.to(torch.float16)
    assert torch.equal(h.to(torch.float32), t.to(torch.float32)), "values are not representable in fp16"
    return h


class DeviceState:
    """All device tensors of one workload plus the outputs of one wkv_compress_groups call."""

    def __init__(self, w: S.Workload, device, layers=True, flags=0, as_f16=False):
        """``as_f16``: a bf16 workload handed to the library as IEEE half tensors.  Every value the
        generator makes in bf16 is exactly representable in fp16, so the inputs (and what the
        oracle computes from them) are the same numbers in another storage format."""
        self.w = w
        self.device = device
        self.as_f16 = as_f16
        kw = dict(dtype=W.WKV_F16) if as_f16 else {}
        self.problem = make_problem(w, flags=flags, **kw)
        self.dims = W.wkv_get_dims(self.problem)
        self.q = [w.q_obs_torch(g, device) for g in range(w.n_groups)]
        self.k = [w.kv_torch(S.KIND_K, l, device) for l in range(w.n_layers)]
        self.v = [w.kv_torch(S.KIND_V, l, device) for l in range(w.n_layers)]
        if as_f16:
            assert w.dtype == "bf16"
            self.q = [_exact_half(t) for t in self.q]
            self.k = [_exact_half(t) for t in self.k]
            self.v = [_exact_half(t) for t in self.v]
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
