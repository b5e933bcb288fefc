"""Helpers shared by the GPU parity tests: move numpy inputs to the device, call the C ABI
through the binding, bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

import paper_2208_05631_amd as qa

DEV = torch.device("cuda:0")


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def workspace(nbytes):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV) if nbytes else None


def gpu_quantize_pack(g, bucket, thr_coef=0.75, thresholds=None, code_stride=None,
                      scale_stride=None, g_stride=None, exact=False):
    """g: numpy f32 [M, d] -> (codes u32 [M, cs], scales [M, ss], thresholds [M, ss]) as numpy."""
    M, d = g.shape
    L = qa.Layout.make(d, M, bucket, thr_coef, code_stride, scale_stride)
    gs = g_stride or ((d + 3) // 4) * 4
    gp = np.zeros((M, gs), np.float32)
    gp[:, :d] = g
    gd = dev(gp)
    codes = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
    scales = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    th = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    flags = 0
    if thresholds is not None:
        th[:, :L.n_buckets] = dev(np.asarray(thresholds, np.float32).reshape(M, -1))
        flags = qa.QA_THRESH_GIVEN
    if exact:
        flags = qa.QA_THRESH_EXACT
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE))
    qa.qa_quantize_pack(L, gd, gs, codes, scales, th, flags, ws)
    torch.cuda.synchronize()
    return host(codes).view(np.uint32), host(scales), host(th), L


class GpuState:
    """x, G, z on the device plus the layout's codes/scales, for stepping through the C ABI."""

    def __init__(self, L, codes, scales, x, G, z):
        self.L = L
        self.codes = dev(np.ascontiguousarray(codes).view(np.int32))
        self.scales = dev(scales)
        self.x, self.G, self.z = dev(x), dev(G), dev(z)
        self.ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP))

    def qcmd(self, eta, lam, delta, requant=0, track_z=True):
        qa.qa_step_qcmd(self.L, self.codes, self.scales, self.x, self.G,
                        self.z if track_z else None, eta, lam, delta, requant, self.ws)

    def qrda(self, t, eta, lam, delta, requant=0):
        qa.qa_step_qrda(self.L, self.codes, self.scales, self.x, self.G, self.z, t, eta, lam, delta,
                        requant, self.ws)

    def get(self):
        torch.cuda.synchronize()
        return host(self.x), host(self.G), host(self.z)
