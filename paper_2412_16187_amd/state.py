"""Device buffers of a fixed-budget HashEvict cache.

Allocation and argument plumbing only: torch supplies device memory and the stream, all
computation happens inside ``liblshe.so`` through ``binding``.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def to_device(x: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """float32 host array -> device tensor of the workload dtype (bf16: round-to-nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch_dtype(dtype)).to(device)


class DeviceCache:
    """K/V/code slot arrays, slot_pos, n_valid, projection and workspace for one config."""

    def __init__(self, batch, n_layers, n_kv_heads, gqa_group, head_dim, hash_bits, budget,
                 dtype="bf16", n_sink=0, n_recent=0, n_prompt_max=0, device="cuda:0",
                 policy="hash"):
        self.cfg = B.make_config(head_dim, hash_bits, n_kv_heads, gqa_group, n_layers, batch,
                                 budget, dtype, n_sink, n_recent, policy)
        self.policy = policy
        rc = B.lshe_check_config(self.cfg)
        if rc != B.LSHE_OK:
            raise B.LsheError(rc, "lshe_check_config")
        self.B, self.L, self.H, self.G = batch, n_layers, n_kv_heads, gqa_group
        self.d, self.r, self.C = head_dim, hash_bits, budget
        self.W = (hash_bits + 31) // 32 if policy == "hash" else 1
        self.Wr = (hash_bits + 31) // 32          # words per hyperplane code (layout of R_dev)
        self.dtype = dtype
        self.device = torch.device(device)
        self.units = batch * n_layers * n_kv_heads
        td = torch_dtype(dtype)
        dev = self.device
        U, Cn, d, W = self.units, budget, head_dim, self.W
        self.K = torch.zeros((U, Cn, d), dtype=td, device=dev)
        self.V = torch.zeros((U, Cn, d), dtype=td, device=dev)
        self.code = torch.zeros((U, Cn, W), dtype=torch.int32, device=dev)
        self.slot_pos = torch.full((U, Cn), -1, dtype=torch.int32, device=dev)
        self.n_valid = torch.zeros((U,), dtype=torch.int32, device=dev)
        self.out = torch.zeros((U, gqa_group, d), dtype=td, device=dev)
        self.evicted = torch.zeros((U,), dtype=torch.int32, device=dev)
        self.R_dev = torch.zeros((B.lshe_projection_bytes(self.cfg),), dtype=torch.uint8, device=dev)
        self.ws_bytes = B.lshe_workspace_bytes(self.cfg, n_prompt_max)
        self.workspace = torch.empty((max(self.ws_bytes, 256),), dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.workspace[:256].zero_()      # the status word starts clear

    # -- projection ------------------------------------------------------------------------
    def init_projection(self, R_host=None, seed=0):
        if R_host is not None:
            R_host = np.ascontiguousarray(R_host, dtype=np.float32)
            assert R_host.shape == (self.d, self.r)
        B.lshe_init_projection(self.cfg, seed, R_host, self.R_dev)

    def projection_host(self) -> np.ndarray:
        """The [d][r] float32 values the device actually uses (read back from R_dev)."""
        td = torch_dtype(self.dtype)
        R = self.R_dev.view(td).view(32 * self.Wr, self.d)[: self.r].float().cpu().numpy()
        return np.ascontiguousarray(R.T)

    # -- entry points ------------------------------------------------------------------------
    def hash_keys(self, X: torch.Tensor) -> torch.Tensor:
        n = X.numel() // self.d
        codes = torch.empty((n, self.Wr), dtype=torch.int32, device=self.device)
        B.lshe_hash_keys(self.cfg, self.R_dev, X, n, codes)
        return codes

    def key_norms(self, X: torch.Tensor) -> torch.Tensor:
        n = X.numel() // self.d
        norm2 = torch.empty((n,), dtype=torch.float32, device=self.device)
        B.lshe_key_norms(self.cfg, X, n, norm2)
        return norm2

    def prefill(self, Kp, Vp, Qp, n_prompt, evict_log=None):
        need = B.lshe_workspace_bytes(self.cfg, n_prompt)
        if need > self.workspace.numel():
            self.workspace = torch.empty((need,), dtype=torch.uint8, device=self.device)
            self.workspace[:256].zero_()
        B.lshe_prefill_compress(self.cfg, self.R_dev, Kp, Vp, Qp, n_prompt, self.K, self.V,
                                self.code, self.slot_pos, self.n_valid, evict_log, self.workspace)

    def decode_step(self, q, k, v, pos, scores_dbg=None, codes_dbg=None, out=None, evicted=None,
                    evicted_mass=None):
        B.lshe_decode_step(self.cfg, self.R_dev, q, k, v, pos, self.K, self.V, self.code,
                           self.slot_pos, self.n_valid, self.out if out is None else out,
                           self.evicted if evicted is None else evicted, scores_dbg, codes_dbg,
                           evicted_mass, self.workspace)

    def status(self) -> int:
        """The workspace's status word (synchronises)."""
        return int(self.workspace[:4].view(torch.int32).item())

    def snapshot(self):
        return tuple(t.clone() for t in (self.K, self.V, self.code, self.slot_pos, self.n_valid))

    def restore(self, snap):
        for dst, src in zip((self.K, self.V, self.code, self.slot_pos, self.n_valid), snap):
            dst.copy_(src)


def upload_workload(w, threads=8, device="cuda:0"):
    """Generate every unit of a synthetic workload on the host (threaded, one unit at a time in
    memory) and copy it to the device.  Returns (Kp, Vp, Qp, kd, vd, qd): the prompt tensors
    [U][N][d], [U][N][d], [U][G][N][d] and the decode-step tensors [T][U][d], [T][U][d],
    [T][U][G][d] in the workload dtype."""
    from concurrent.futures import ThreadPoolExecutor

    from . import synth
    U, N, T, G, d = w.n_units, w.n_prompt, w.n_decode, w.gqa_group, w.head_dim
    td = torch_dtype(w.dtype)
    dev = torch.device(device)
    Kp = torch.empty((U, N, d), dtype=td, device=dev)
    Vp = torch.empty((U, N, d), dtype=td, device=dev)
    Qp = torch.empty((U, G, N, d), dtype=td, device=dev)
    kd = torch.empty((T, U, d), dtype=td, device=dev)
    vd = torch.empty((T, U, d), dtype=td, device=dev)
    qd = torch.empty((T, U, G, d), dtype=td, device=dev)

    def gen(u):
        x = synth.gen_unit(w, u)
        return u, x["K"], x["V"], x["Q"]

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for u, K, V, Q in ex.map(gen, range(U)):
            Kp[u].copy_(torch.from_numpy(K[:N]).to(td))
            Vp[u].copy_(torch.from_numpy(V[:N]).to(td))
            Qp[u].copy_(torch.from_numpy(Q[:, :N]).to(td))
            if T:
                kd[:, u].copy_(torch.from_numpy(K[N:]).to(td))
                vd[:, u].copy_(torch.from_numpy(V[N:]).to(td))
                qd[:, u].copy_(torch.from_numpy(np.ascontiguousarray(Q[:, N:].transpose(1, 0, 2))).to(td))
    return Kp, Vp, Qp, kd, vd, qd
