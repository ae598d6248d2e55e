"""Runs workloads through libppll.so on cuda:0 and returns host copies for comparison.
PyTorch only provides device memory and streams."""
import numpy as np
import torch

from paper_2411_12780_amd import binding as P
from paper_2411_12780_amd import synth

DEV = "cuda:0"


def to_device(x: np.ndarray, wl: dict) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if wl["precision"] == synth.BF16:
        t = t.to(torch.bfloat16)          # inputs are already bf16-representable
    return t.to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


class GpuBlock:
    """One ppll block with its workspace and output buffer."""

    def __init__(self, wl: dict, flat_params: np.ndarray):
        self.wl = wl
        self.cfg = P.make_config(wl)
        self.ws_bytes = P.ppll_block_workspace_bytes(self.cfg)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=DEV)
        self.dtype = torch.bfloat16 if wl["precision"] == synth.BF16 else torch.float32
        self.x_out = torch.empty(synth.output_shape(wl), dtype=self.dtype, device=DEV)
        self.loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        self.h = P.ppll_block_init(self.cfg, self.ws, self.ws_bytes, flat_params, None)
        self.names = [P.ppll_block_tensor_info(self.h, P.T_PARAM, i)[0]
                      for i in range(P.ppll_block_tensor_count(self.h, P.T_PARAM))]

    def step(self, x: np.ndarray, y: np.ndarray, lr: float):
        self.x_in = to_device(x, self.wl)
        self.y = torch.from_numpy(y.astype(np.int32)).to(DEV)
        stream = torch.cuda.current_stream().cuda_stream
        P.ppll_block_step(self.h, self.x_in, self.y, lr, self.x_out, self.loss, stream)
        loss = P.ppll_block_sync(self.h)
        assert abs(loss - float(self.loss.item())) == 0.0
        return to_host(self.x_out), loss

    def tensors(self, kind=P.T_PARAM) -> dict:
        return {n: P.ppll_block_read_tensor(self.h, kind, i).astype(np.float64) for i, n in enumerate(self.names)}

    def bn(self, kind) -> dict:
        n = P.ppll_block_tensor_count(self.h, kind)
        return {P.ppll_block_tensor_info(self.h, kind, i)[0]: P.ppll_block_read_tensor(self.h, kind, i).astype(np.float64)
                for i in range(n)}

    def close(self):
        P.ppll_block_destroy(self.h)
