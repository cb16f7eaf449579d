"""Helpers for the GPU parity tests: numpy <-> device marshalling around the C-ABI binding."""
import numpy as np


def to_dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def pack(d, group):
    """d: workload dict with qweight/s/z -> PackedW4 (device)."""
    import paper_2508_15601_amd as tm
    K, N = d["q"].shape
    return tm.tm_pack_w4(to_dev(d["qweight"]), to_dev(d["s"]), to_dev(d["z"]), K, N, group)


def gemm(packed, X, M=None):
    """X numpy float16 [M,K] -> Y numpy float16 [M,N] through tm_gemm_w4a16."""
    import torch
    import paper_2508_15601_amd as tm
    Xd = to_dev(X)
    Y = torch.full((X.shape[0], packed.N), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16(Xd, packed, Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy()
