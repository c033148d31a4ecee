"""Upload a synthetic case to the GPU and call the library through its C ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2601_22716_amd as L


def bf16_tensor(bits_u16: np.ndarray) -> torch.Tensor:
    return L.bf16_from_bits(bits_u16)


class DeviceCase:
    def __init__(self, cs):
        self.cs = cs
        self.codes = torch.from_numpy(cs.codes.copy()).cuda()
        self.codebook = torch.from_numpy(cs.codebook.copy()).cuda()
        if cs.B_bf16 is not None:
            self.B, self.A = bf16_tensor(cs.B_bf16), bf16_tensor(cs.A_bf16)
        else:
            self.B, self.A = torch.from_numpy(cs.B_f32.copy()).cuda(), torch.from_numpy(cs.A_f32.copy()).cuda()
        self.X = bf16_tensor(cs.X_bf16)
        self.N, self.K, self.r, self.bits, self.M = cs.N, cs.K, cs.r, cs.bits, cs.M

    def unpack(self) -> np.ndarray:
        idx = torch.full((self.N, self.K), 255, dtype=torch.uint8, device="cuda")
        L.lords_unpack(self.codes, idx, self.N, self.K, self.bits)
        torch.cuda.synchronize()
        return idx.cpu().numpy()

    def dequant(self, dtype=torch.float32) -> np.ndarray:
        W = torch.full((self.N, self.K), float("nan"), dtype=dtype, device="cuda")
        L.lords_dequant(self.codes, self.codebook, self.B, self.A, W, self.N, self.K, self.r, self.bits)
        torch.cuda.synchronize()
        return W.float().cpu().numpy()

    def matmul(self, path=L.LORDS_PATH_AUTO, dtype=torch.float32, X=None, M=None) -> np.ndarray:
        X = self.X if X is None else X
        M = self.M if M is None else M
        Y = torch.full((M, self.N), float("nan"), dtype=dtype, device="cuda")
        L.lords_matmul_ex(X, self.codes, self.codebook, self.B, self.A, Y, M, self.N, self.K, self.r, self.bits, path)
        torch.cuda.synchronize()
        return Y.float().cpu().numpy()
