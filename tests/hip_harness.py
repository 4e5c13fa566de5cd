"""Shared helpers of the GPU parity tests: upload a workload, run the HIP path
through the C ABI, fetch maps and C.  No arithmetic of the method lives here."""
import numpy as np
import torch

import mmm_synth as synth
import paper_2402_14118_amd as mm

# fp32 inputs: the stated bound.  bf16 inputs: the stated bound.  IEEE half inputs: no bound is stated; the product of
# two halves is exact in float and the sums are float sums, so the fp32 bound applies unchanged.
# Double inputs: none is stated either; products are accumulated by double FMAs over at most a few thousand terms
# (error below terms * 2^-53 * |A||B|, i.e. 1e-12 leaves two decimal digits of room), and the absolute slack scales
# with the precision.
TOL_REL = {synth.DT_F32: 1e-5, synth.DT_BF16: 1e-2, synth.DT_F16: 1e-5, synth.DT_F64: 1e-12}
TOL_ABS = {synth.DT_F32: 1e-6, synth.DT_BF16: 1e-6, synth.DT_F16: 1e-6, synth.DT_F64: 1e-15}


def _dev(a, ld=None):
    """Upload a 2-D host array; with ld > cols the device rows are padded to ld."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if ld is not None and ld != a.shape[1]:
        buf = torch.full((a.shape[0], ld), -7, dtype=t.dtype)     # junk in the padding
        buf[:, : a.shape[1]] = t
        return buf.cuda()[:, : a.shape[1]]
    return t.cuda()


def _bits_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


class HipRun:
    """Device-resident copy of a workload plus its MaskedMatmul engine."""

    def __init__(self, w, ldx=None, ldy=None, ldc=None):
        self.w = w
        if w.dtype == synth.DT_F64:
            self.X = _dev(np.asarray(w.X, dtype=np.float64), ldx)
            self.Y = _dev(np.asarray(w.Y, dtype=np.float64), ldy)
        elif w.dtype != synth.DT_F32:
            self.X = _dev(w.X_bits.view(np.int16), ldx)
            self.Y = _dev(w.Y_bits.view(np.int16), ldy)
        else:
            self.X = _dev(w.X, ldx)
            self.Y = _dev(w.Y, ldy)
        self.keep_a = _bits_dev(w.keep_a)
        self.keep_rows = _bits_dev(w.keep_rows)
        self.keep_blocks = _bits_dev(w.keep_blocks)
        ldc = ldc or w.N
        self.Cbuf = torch.full((w.M, ldc), float("nan"), device="cuda",
                               dtype=torch.float64 if w.dtype == synth.DT_F64 else torch.float32)
        self.C = self.Cbuf[:, : w.N]
        self.eng = mm.MaskedMatmul(w.M, w.K, w.N, w.bw, w.dtype)

    def build(self, a=True, b=True):
        self.eng.build_maps(self.X if a else None, self.Y if b else None, self.w.pred, self.w.threshold,
                            self.keep_a, self.keep_rows, self.keep_blocks)

    def matmul(self, accumulate=False):
        self.eng.matmul(self.X, self.Y, self.C, accumulate)

    def run(self, accumulate=False):
        self.build()
        self.matmul(accumulate)
        torch.cuda.synchronize()
        return self.maps_host() + (self.C.cpu().numpy(),)

    def maps_host(self):
        torch.cuda.synchronize()
        return (self.eng.a_bits().cpu().numpy().view(np.uint64), self.eng.b_bits().cpu().numpy().view(np.uint64))

    def derived_host(self):
        torch.cuda.synchronize()
        return (self.eng.a_colany().cpu().numpy().view(np.uint64), self.eng.bt_bits().cpu().numpy().view(np.uint64))

    def lists_host(self):
        """(counts [blocks_m, blocks_k], list of per-block uint64 entry arrays up to the padded count)"""
        torch.cuda.synchronize()
        counts, entries = self.eng.a_lists()
        counts = counts.cpu().numpy()
        padded = (counts.reshape(-1).astype(np.int64) + 63) // 64 * 64
        return counts, [entries[b, : int(n)].cpu().numpy().view(np.uint64) for b, n in enumerate(padded)]


def assert_close(C, C_ref, mag, dtype, what=""):
    err = np.abs(C.astype(np.float64) - C_ref.astype(np.float64))
    bound = TOL_REL[dtype] * mag + TOL_ABS[dtype]
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements out of tolerance; worst at {i}: "
                             f"got {C[i]!r} want {C_ref[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")
    return float((err / (mag + 1e-30)).max())
