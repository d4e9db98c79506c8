"""Device-side container for one verification batch: uploads the numpy arrays of a batch
(any object with the fields of ssv_inputs.VerifyCase) into HBM through PyTorch, owns the output,
index and workspace buffers, and calls the C ABI.  PyTorch is used for memory and streams only.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _to_device(arr: np.ndarray, dtype: str, device) -> torch.Tensor:
    if dtype == "bf16" and arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


class DeviceCase:
    def __init__(self, case, device="cuda:0", mode=B.SSV_REFRESH, group_size=0, scale=0.0, exec=B.SSV_EXEC_FUSED,
                 topn_home=B.SSV_TOPN_AUTO, max_slice_tiles=0, imp_rows=0, strided_q_out=False, scan_kernel=B.SSV_SCAN_AUTO, avg_seq_len=None):
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceCase needs a GPU: the NSA verification path has no CPU fallback")
        B.load_library()
        self.case = case
        self.device = torch.device(device)
        nsa = case.nsa
        dt = case.dtype
        self.q = _to_device(case.q, dt, self.device)
        tdt = torch.bfloat16 if dt == "bf16" else torch.float32
        q_stride = out_stride = (0, 0, 0)
        if strided_q_out:
            # q and out as views into wider buffers (a fused QKV projection's output, a padded output): head-major
            # [B, H, T, d + 8] storage addressed through (batch, query, head) strides
            qbuf = torch.zeros((case.B, case.H, case.T, case.d_k + 8), dtype=tdt, device=self.device)
            qbuf[..., :case.d_k] = self.q.permute(0, 2, 1, 3)
            self.q = qbuf.permute(0, 2, 1, 3)[..., :case.d_k]
            q_stride = self.q.stride()[:3]
        self.k = _to_device(case.k, dt, self.device)
        self.v = _to_device(case.v, dt, self.device)
        self.k_cmp = _to_device(case.k_cmp, dt, self.device)
        self.v_cmp = _to_device(case.v_cmp, dt, self.device)
        self.gates = torch.from_numpy(np.ascontiguousarray(case.gates, np.float32)).to(self.device)
        self.seq_lens = torch.from_numpy(np.ascontiguousarray(case.seq_lens, np.int32)).to(self.device)
        self.n_cmp = torch.from_numpy(np.ascontiguousarray(case.n_cmp, np.int32)).to(self.device)
        self.n_query = torch.from_numpy(np.ascontiguousarray(case.n_query, np.int32)).to(self.device)
        self.parents = None if case.parents is None else \
            torch.from_numpy(np.ascontiguousarray(case.parents, np.int32)).to(self.device)
        self.out = torch.zeros((case.B, case.T, case.H, case.d_v), dtype=tdt, device=self.device)
        if strided_q_out:
            obuf = torch.full((case.B, case.H, case.T, case.d_v + 8), 7.0, dtype=tdt, device=self.device)
            self.out_buf = obuf
            self.out = obuf.permute(0, 2, 1, 3)[..., :case.d_v]
            out_stride = self.out.stride()[:3]
        self.sel_idx = torch.full((case.B, case.T, case.H_kv, nsa.n_sel), -1, dtype=torch.int32, device=self.device)
        self.params = B.make_params(
            B=case.B, T=case.T, H=case.H, H_kv=case.H_kv, d_k=case.d_k, d_v=case.d_v, l=nsa.l, d=nsa.d,
            l_sel=nsa.l_sel, n_sel=nsa.n_sel, w=nsa.w, n_init=nsa.n_init, n_local=nsa.n_local,
            dtype=B.SSV_BF16 if dt == "bf16" else B.SSV_F32, mode=mode, group_size=group_size, scale=scale,
            max_seq_len=int(case.seq_lens.max()), max_n_cmp=int(case.n_cmp.max()),
            avg_seq_len=int(case.seq_lens.mean()) if avg_seq_len is None else avg_seq_len,
            k_stride=self.k.stride()[:3], v_stride=self.v.stride()[:3],
            kc_stride=self.k_cmp.stride()[:3], vc_stride=self.v_cmp.stride()[:3], q_stride=q_stride, out_stride=out_stride,
            exec=exec, topn_home=topn_home, max_slice_tiles=max_slice_tiles, imp_rows=imp_rows, scan_kernel=scan_kernel)
        self.workspace_bytes = 0
        self.workspace = None
        self.set_group_size(group_size, mode)

    def set_group_size(self, group_size: int, mode=None, scan_group_size: int = 0) -> None:
        """Change C (verifier queries per workgroup) and the group size of the scan launch; the workspace grows if
        the new plan needs more."""
        self.params.group_size = group_size
        self.params.scan_group_size = scan_group_size
        mode = self.params.mode if mode is None else mode
        # the split plan (and with it the scratch size) depends on the mode: size the workspace for all of them
        need = 0
        modes = (B.SSV_REFRESH, B.SSV_REUSE) if self.params.exec == B.SSV_EXEC_UNFUSED else \
            (B.SSV_REFRESH, B.SSV_REUSE, B.SSV_REFRESH_SHARED)
        for m in modes:
            self.params.mode = m
            need = max(need, B.ssv_nsa_workspace_bytes(self.params))
        if need > self.workspace_bytes:
            self.workspace_bytes = need
            # (a byte pattern, not zeros: a call must not depend on what the scratch held before; 0x55.. reads as a large
            # positive float, so a partial state that a call reads without having written it shows in the output)
            self.workspace = torch.full((need,), 0x55, dtype=torch.uint8, device=self.device)
        self.set_mode(mode)

    def set_mode(self, mode: int) -> None:
        self.params.mode = mode
        self.plan = B.ssv_nsa_plan_query(self.params)

    def set_exec(self, exec: int, mode=None) -> None:
        """Fused (grouped, merged schedule) or unfused (per query, one launch per branch) execution."""
        self.params.exec = exec
        self.set_group_size(0, mode)

    def set_queries(self, q: np.ndarray) -> None:
        """Replace the verifier queries (same shape), keeping the caches."""
        self.q.copy_(_to_device(q, self.case.dtype, self.device))

    def set_sel_idx(self, sel: np.ndarray) -> None:
        self.sel_idx.copy_(torch.from_numpy(np.ascontiguousarray(sel, np.int32)).to(self.device))

    def run(self, kernel_ms=None, repeats: int = 1) -> None:
        """Enqueue one call on torch's current stream."""
        stream = torch.cuda.current_stream(self.device).cuda_stream
        B.ssv_nsa_verify(self.q, self.k, self.v, self.k_cmp, self.v_cmp, self.gates, self.seq_lens, self.n_cmp,
                         self.n_query, self.parents, self.params, self.out, self.sel_idx, self.workspace,
                         self.workspace_bytes, stream, kernel_ms=kernel_ms, repeats=repeats)

    def results(self):
        torch.cuda.synchronize(self.device)
        return self.out.float().cpu().numpy().astype(np.float64), self.sel_idx.cpu().numpy()
