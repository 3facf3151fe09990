"""Shared plumbing for the GPU parity tests: move seeded inputs to the device, call the C-ABI binding,
bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

import paper_2511_11248_amd as tman
import synth

TOL = 2e-3  # max relative error under the row-normalised metric (fp16 tables / weights, fp32 accumulation)


def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def rand_case(seed, M, K, N, bits, group, has_zero=True, zero_range=None):
    if zero_range is None:
        zero_range = (6.0, 9.0) if bits == 4 else (1.0, 2.0) if bits == 2 else (0.25, 0.75)
    q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
    s = synth.uniform_fp16(seed + 1, M * (K // group), 0.005, 0.02).reshape(M, -1)
    z = synth.uniform_fp16(seed + 2, M * (K // group), *zero_range).reshape(M, -1) if has_zero else None
    x = synth.normal_fp16(seed + 3, N * K).reshape(N, K)
    return q, s, z, x


def to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def pack(shape, q, s, z):
    """q/s/z numpy or torch -> packed blob (torch u8 on the device)."""
    qd = q if torch.is_tensor(q) else to_dev(q)
    sd = s if torch.is_tensor(s) else to_dev(s)
    zd = z if (z is None or torch.is_tensor(z)) else to_dev(z)
    blob = torch.empty(tman.tman_packed_bytes(shape), dtype=torch.uint8, device=dev())
    blob.fill_(0xA5)  # poison: the packer must define every byte
    tman.tman_pack_weights(shape, qd, sd, zd, blob)
    return blob


def build_lut(x, group):
    xd = x if torch.is_tensor(x) else to_dev(x)
    N, K = xd.shape
    lut = torch.empty(tman.tman_lut_bytes(N, K, group), dtype=torch.uint8, device=dev())
    lut.fill_(0x5A)
    tman.tman_build_lut(xd, N, K, group, lut)
    return lut


def gemv_workspace(shape, N):
    return torch.zeros(tman.tman_mpgemv_workspace_bytes(shape, N), dtype=torch.uint8, device=dev())


def mpgemv(shape, blob, x, workspace=None):
    xd = x if torch.is_tensor(x) else to_dev(x)
    N = xd.shape[0]
    lut = build_lut(xd, shape.group)
    ws = gemv_workspace(shape, N) if workspace is None else workspace
    y = torch.full((N, shape.M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemv(shape, blob, lut, N, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def mpgemv_x(shape, blob, x, workspace=None):
    """One token through the kernel that builds its tables itself; x numpy/torch fp16 [1][K] or [K]."""
    xd = x if torch.is_tensor(x) else to_dev(x)
    ws = gemv_workspace(shape, 1) if workspace is None else workspace
    y = torch.full((1, shape.M), float("nan"), dtype=torch.float16, device=dev())
    tman.tman_mpgemv_x(shape, blob, xd, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def mpgemm(shape, blob, x):
    xd = x if torch.is_tensor(x) else to_dev(x)
    N = xd.shape[0]
    y = torch.full((N, shape.M), float("nan"), dtype=torch.float16, device=dev())
    need = tman.tman_mpgemm_workspace_bytes(shape, N)
    ws = torch.zeros(need, dtype=torch.uint8, device=dev()) if need else None
    tman.tman_mpgemm(shape, blob, xd, N, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()
