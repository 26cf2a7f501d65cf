"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import pytest
import torch


def to_dev(a, device="cuda"):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(device)
    torch.cuda.synchronize()
    return t


def to_host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


@pytest.fixture(scope="module")
def ctx():
    from paper_2504_08378_amd import binding as B
    c = B.Context(0)
    yield c
    c.close()
