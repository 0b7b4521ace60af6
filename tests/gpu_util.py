"""Helpers for the GPU parity tests: move a case to the device and call the C ABI."""
import numpy as np
import torch

import paper_2410_21271_amd as eora


def dev(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def run_linear_q(c, M=None, x=None, r=None, canary=True, ws=None):
    """Run eora_linear_q on case c; returns y as float16 numpy (M x d_out)."""
    M = c.M if M is None else M
    r = c.r if r is None else r
    x = c.x if x is None else x
    xd = dev(x)
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    A, B, As, Bs = (dev(c.A), dev(c.B), dev(c.As), dev(c.Bs)) if r > 0 else (None, None, None, None)
    ws = eora.new_workspace(M, c.d_in, c.d_out, r) if ws is None else ws
    pad = 64
    ybuf = torch.full((M * c.d_out + 2 * pad,), 777.0, dtype=torch.float16, device="cuda")
    y = ybuf[pad: pad + M * c.d_out]
    eora.linear_q(xd, qw, sc, qz, A, B, As, Bs, y, M, c.d_in, c.d_out, r, c.w_bits, c.group, c.ab_bits, ws)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    if canary:
        assert np.all(out[:pad] == 777.0) and np.all(out[pad + M * c.d_out:] == 777.0), "write outside y"
    return out[pad: pad + M * c.d_out].reshape(M, c.d_out)


def run_linear_q_group(cases, x, r=None, ws=None):
    """Run eora_linear_q_group on cases that share d_in, r and formats, all fed the activations x
    (M x d_in fp16 numpy); returns the list of y (M x d_out fp16 numpy)."""
    c0 = cases[0]
    M = x.shape[0]
    r = c0.r if r is None else r
    xd = dev(x)
    keep, members, ys = [], [], []
    for c in cases:
        t = [dev(c.qw), dev(c.sc), dev(c.qz)] + ([dev(c.A), dev(c.B), dev(c.As), dev(c.Bs)] if r > 0 else [None] * 4)
        y = torch.full((M * c.d_out,), 777.0, dtype=torch.float16, device="cuda")
        keep.append(t)
        ys.append(y)
        members.append(tuple(t) + (y, c.d_out))
    ws = eora.new_workspace(M, c0.d_in, max(c.d_out for c in cases), r, n_members=len(cases)) if ws is None else ws
    eora.linear_q_group(xd, members, M, c0.d_in, r, c0.w_bits, c0.group, c0.ab_bits, ws)
    torch.cuda.synchronize()
    return [y.cpu().numpy().reshape(M, c.d_out) for y, c in zip(ys, cases)]


def run_linear_sp24(c, M=None, x=None, r=None, ws=None):
    """Run eora_linear_sp24 on case c; returns y as float16 numpy (M x d_out)."""
    M = c.M if M is None else M
    r = c.r if r is None else r
    x = c.x if x is None else x
    xd, values, indices = dev(x), dev(c.values), dev(c.indices)
    A, B = (dev(c.A), dev(c.B)) if r > 0 else (None, None)
    ws = eora.new_workspace(M, c.d_in, c.d_out, r) if ws is None else ws
    pad = 64
    ybuf = torch.full((M * c.d_out + 2 * pad,), 777.0, dtype=torch.float16, device="cuda")
    y = ybuf[pad: pad + M * c.d_out]
    eora.linear_sp24(xd, values, indices, A, B, y, M, c.d_in, c.d_out, r, ws)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    assert np.all(out[:pad] == 777.0) and np.all(out[pad + M * c.d_out:] == 777.0), "write outside y"
    return out[pad: pad + M * c.d_out].reshape(M, c.d_out)


def run_linear_sp24q4(c, ws=None):
    """Run eora_linear_sp24q4 on case c; returns y as float16 numpy (M x d_out)."""
    xd = dev(c.x)
    t = [dev(c.tiles), dev(c.meta)]
    A, B = (dev(c.A), dev(c.B)) if c.r > 0 else (None, None)
    y = torch.full((c.M * c.d_out,), 777.0, dtype=torch.float16, device="cuda")
    ws = eora.new_workspace(c.M, c.d_in, c.d_out, c.r) if ws is None else ws
    eora.linear_sp24q4(xd, t[0], t[1], A, B, y, c.M, c.d_in, c.d_out, c.r, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy().reshape(c.M, c.d_out)


def run_linear_q_multi(c, sel, r_per, ws=None):
    """Run eora_linear_q_multi on case c, whose factors of rank c.r are c.r / r_per adapters side by side;
    sel: int32 numpy, one adapter index (or -1) per token row.  Returns y as float16 numpy (M x d_out)."""
    n = c.r // r_per
    xd = dev(c.x)
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    A, B, As, Bs = dev(c.A), dev(c.B), dev(c.As), dev(c.Bs)
    seld = torch.from_numpy(np.ascontiguousarray(sel, dtype=np.int32)).cuda()
    ws = eora.new_workspace(c.M, c.d_in, c.d_out, c.r) if ws is None else ws
    pad = 64
    ybuf = torch.full((c.M * c.d_out + 2 * pad,), 777.0, dtype=torch.float16, device="cuda")
    y = ybuf[pad: pad + c.M * c.d_out]
    eora.linear_q_multi(xd, qw, sc, qz, A, B, As, Bs, seld, y, c.M, c.d_in, c.d_out, r_per, n, c.w_bits, c.group,
                        c.ab_bits, ws)
    torch.cuda.synchronize()
    assert eora.workspace_error(ws) == 0
    out = ybuf.cpu().numpy()
    assert np.all(out[:pad] == 777.0) and np.all(out[pad + c.M * c.d_out:] == 777.0), "write outside y"
    return out[pad: pad + c.M * c.d_out].reshape(c.M, c.d_out)


def run_linear_sp24_group(cases, ws=None):
    """Run eora_linear_sp24_group on 2:4 cases (all SparseCase or all SparseQCase) that share M, d_in, r and the
    activations of the first case; returns the list of y (M x d_out fp16 numpy)."""
    c0 = cases[0]
    xd = dev(c0.x)
    mem, ys = [], []
    for c in cases:
        y = torch.full((c0.M * c.d_out,), 777.0, dtype=torch.float16, device="cuda")
        A, B = (dev(c.A), dev(c.B)) if c0.r > 0 else (None, None)
        if hasattr(c, "tiles"):
            mem.append((None, None, dev(c.tiles), dev(c.meta), A, B, y, c.d_out))
        else:
            mem.append((dev(c.values), dev(c.indices), None, None, A, B, y, c.d_out))
        ys.append(y)
    ws = eora.new_workspace(c0.M, c0.d_in, max(c.d_out for c in cases), c0.r) if ws is None else ws
    eora.linear_sp24_group(xd, mem, c0.M, c0.d_in, c0.r, ws)
    torch.cuda.synchronize()
    assert eora.workspace_error(ws) == 0
    return [y.cpu().numpy().reshape(c0.M, c.d_out) for y, c in zip(ys, cases)]
