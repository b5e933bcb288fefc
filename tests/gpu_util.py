"""Helpers shared by the GPU parity tests: move numpy inputs to the device, call the C ABI
through the binding, bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

import oracle
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
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE_EXACT if exact else qa.QA_OP_QUANTIZE))
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


def ulp_distance(a, b):
    """Distance in units in the last place between two float32 arrays (finite values)."""
    def ordered(v):
        i = np.ascontiguousarray(v, np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    return np.abs(ordered(a) - ordered(b))


def quantizer_parity(g, bucket, codes, scales, thresholds, what="", thr_coef=0.75):
    """The GPU quantizer's message (codes u32 [M, >=W], scales / thresholds f32 [M, >=nb]) for the
    gradient g (f32 [M, d]) against the oracle's for the same g.

    What the arithmetic guarantees: a bucket's sums are formed in binary64 in a different order on
    the two sides and rounded once, so a threshold or a scale may differ by one binary32 ulp (about
    once in 2^29 sums); codes are exact given the threshold.  Bit-identical messages return 0.
    Otherwise every threshold and scale must lie within 1 ulp, and the codes must equal, bit for
    bit, the oracle's codes for the GPU's own thresholds; the number of (worker, bucket) pairs
    that were not bit-identical is returned so that the caller can report it."""
    M, d = g.shape
    W, nb = oracle.n_words(d), oracle.n_buckets(d, bucket)
    oc, osc, oth = oracle.quantize_pack(g, bucket=bucket, thr_coef=thr_coef)
    gt = np.ascontiguousarray(thresholds[:, :nb], np.float32)
    gs = np.ascontiguousarray(scales[:, :nb], np.float32)
    same = (gt.view(np.uint32) == oth[:, :nb].view(np.uint32)) & \
           (gs.view(np.uint32) == osc[:, :nb].view(np.uint32))
    if same.all():
        assert np.array_equal(codes[:, :W], oc[:, :W]), f"codes differ with identical thresholds {what}"
        return 0
    assert int(ulp_distance(gt, oth[:, :nb]).max()) <= 1, f"threshold off by more than 1 ulp {what}"
    oc2, osc2, _ = oracle.quantize_pack(g, bucket=bucket, thr_coef=thr_coef, thresholds=gt)
    assert np.array_equal(codes[:, :W], oc2[:, :W]), f"codes differ for the same thresholds {what}"
    assert int(ulp_distance(gs, osc2[:, :nb]).max()) <= 1, f"scale off by more than 1 ulp {what}"
    return int((~same).sum())
