"""Helpers for the GPU parity tests: move a synthetic DecodeCase to the device, run the C-ABI
entry points through the binding, and compute the oracle's answers for the same inputs."""

import numpy as np
import torch

import oracle
import paper_2510_18413_amd as A

SM_SCALE = 1.0 / np.sqrt(128.0)
ATTN_TOL = 2e-3   # max relative error of the attention output against the oracle


def dev_bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def host_dist(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).astype(np.int32)


class DeviceCase:
    """Device copies of a DecodeCase plus config, workspace and output buffers."""

    def __init__(self, case, k, encode=True, variant=0, code_bits=0, thresholds=None):
        self.case, self.k = case, k
        self.thresholds = case.thresholds if thresholds is None else thresholds
        self.head_dim = int(case.q.shape[-1])
        self.cfg = A.Config.make(case.Hq, case.Hkv, case.pool_tokens, thr_k=self.thresholds,
                                 variant=variant, code_bits=code_bits, head_dim=self.head_dim)
        self.q = dev_bf16(case.q)
        self.K = dev_bf16(case.K)
        self.V = dev_bf16(case.V)
        self.k_new = None if case.k_new is None else dev_bf16(case.k_new)
        self.v_new = None if case.v_new is None else dev_bf16(case.v_new)
        self.seq_start = torch.from_numpy(case.seq_start).cuda()
        self.seq_len = torch.from_numpy(case.seq_len).cuda()
        self.max_len = max(case.max_seq_len, 1)
        self.codes = torch.zeros(case.Hkv, case.pool_tokens, self.cfg.code_row_bytes,
                                 dtype=torch.uint8, device="cuda")
        nbytes = A.adamas_workspace_bytes(self.cfg, case.B, self.max_len, k)
        assert nbytes > 0
        # poison the workspace: the library must not rely on its contents
        self.workspace = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
        self.out = torch.full((case.B, case.Hq, self.head_dim), float("nan"), device="cuda")
        self.idx = torch.full((case.B, case.Hq, k), -7, dtype=torch.int32, device="cuda")
        if encode:
            A.adamas_encode_keys(self.cfg, self.K, self.codes, 0, case.pool_tokens)

    def decode_step(self, with_idx=True):
        A.adamas_decode_step(self.cfg, self.q, self.K, self.V, self.codes, self.seq_start,
                             self.seq_len, self.k, self.out, self.max_len, self.workspace,
                             k_new=self.k_new, v_new=self.v_new,
                             idx_out=self.idx if with_idx else None)
        torch.cuda.synchronize()
        return self.out.cpu().numpy(), self.idx.cpu().numpy()


def oracle_step(case, k, want_dist=True, variant=0):
    """The oracle's answer for the whole step.  Returns dict(out, idx, dist, K, V, rows).
    variant: the library's ADAMAS_VARIANT_* flags, mapped onto the oracle's two switches."""
    hadamard = not (variant & A.VARIANT_NO_HADAMARD)
    squared = bool(variant & A.VARIANT_L2)
    K, V = case.K.copy(), case.V.copy()
    d = int(case.q.shape[-1])
    with oracle.head_dim(d):
        _, rows = oracle.encode(K, case.thresholds, hadamard=hadamard)
        out, idx, dist = oracle.decode_step(case.q, K, V, rows, case.seq_start, case.seq_len, k,
                                            case.thresholds, case.thresholds, 1.0 / np.sqrt(d),
                                            k_new=case.k_new, v_new=case.v_new,
                                            want_dist=want_dist, hadamard=hadamard,
                                            squared=squared)
    return dict(out=out, idx=idx, dist=dist, K=K, V=V, rows=rows)


def attn_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, 1e-3 * max_j |ref_j|), worst over (b, head)."""
    got = got.reshape(-1, got.shape[-1]).astype(np.float64)
    ref = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    worst = 0.0
    for g, r in zip(got, ref):
        floor = 1e-3 * np.abs(r).max()
        if floor == 0.0:
            assert np.all(g == 0.0)
            continue
        worst = max(worst, float(np.max(np.abs(g - r) / np.maximum(np.abs(r), floor))))
    return worst
