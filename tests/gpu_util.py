"""Host<->device plumbing for the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

from paper_2601_09093_amd import workloads as wl

DEV = "cuda:0"


def dev_bits(a):
    """numpy uint16 (bf16 bit patterns) -> int16 device tensor with the same bytes."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host_bits(t):
    """device bf16/int16 tensor -> numpy uint16 bit patterns."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def host_f32_of_bf16(t):
    return wl.bf16_bits_to_f32(host_bits(t))


def new_status():
    return torch.zeros(1, dtype=torch.int32, device=DEV)
