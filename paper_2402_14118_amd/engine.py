"""Convenience holder for one MMM problem on the current CUDA/HIP device.

Owns the workspace tensor and the maps handle and forwards to the C ABI; it does
no arithmetic of its own.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class MaskedMatmul:
    def __init__(self, M: int, K: int, N: int, block_width: int, dtype: int = B.MMM_F32, device="cuda:0"):
        self.M, self.K, self.N, self.bw, self.dtype = M, K, N, block_width, dtype
        self.device = torch.device(device)
        nbytes = B.mmm_maps_workspace_bytes(M, K, N, block_width)
        # torch's caching allocator hands out >= 512-byte aligned blocks
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        self.maps = B.mmm_maps_init(self.workspace, nbytes, M, K, N, block_width)
        self._keep = []

    def close(self) -> None:
        if self.maps is not None:
            B.mmm_maps_release(self.maps)
            self.maps = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def build_maps(self, X: Optional[torch.Tensor], Y: Optional[torch.Tensor], pred: int = B.MMM_PRED_NONZERO,
                   threshold: float = 0.0, keep_a: Optional[torch.Tensor] = None,
                   keep_rows: Optional[torch.Tensor] = None, keep_blocks: Optional[torch.Tensor] = None,
                   stream=None) -> None:
        ma = mb = None
        if X is not None:
            ma = B.MaskA(pred, threshold, B._ptr(keep_a))
        if Y is not None:
            mb = B.MaskB(self.bw, B._ptr(keep_rows), B._ptr(keep_blocks))
        B.mmm_build_maps(self.maps, self.dtype, X, X.stride(0) if X is not None else 0, ma,
                         Y, Y.stride(0) if Y is not None else 0, mb, stream)

    def matmul(self, X: torch.Tensor, Y: torch.Tensor, C: torch.Tensor, accumulate: bool = False, stream=None) -> None:
        B.mmm_matmul(self.maps, self.dtype, X, X.stride(0), Y, Y.stride(0), C, C.stride(0), int(accumulate), stream)

    def matmul_static_scratch(self, X: torch.Tensor, Y: torch.Tensor, C: torch.Tensor, accumulate: bool = False,
                              stream=None) -> None:
        B.mmm_matmul_static_scratch(self.maps, self.dtype, X, X.stride(0), Y, Y.stride(0), C, C.stride(0),
                                    int(accumulate), stream)

    def matmul_fused(self, X: torch.Tensor, Y: torch.Tensor, C: torch.Tensor, pred: int = B.MMM_PRED_NONZERO,
                     threshold: float = 0.0, keep_a: Optional[torch.Tensor] = None, accumulate: bool = False,
                     stream=None) -> None:
        """C (+)= M(X) x B with M evaluated inside the multiplication; only the B side of the maps is used."""
        ma = B.MaskA(pred, threshold, B._ptr(keep_a))
        B.mmm_matmul_fused(self.maps, self.dtype, X, X.stride(0), ma, Y, Y.stride(0), C, C.stride(0), int(accumulate),
                           stream)

    def set_path(self, path: int = -1) -> None:
        B.mmm_maps_set_path(self.maps, path)

    def path(self) -> int:
        return B.mmm_matmul_path(self.maps)

    def stats(self, stream=None):
        return B.mmm_maps_stats(self.maps, stream)

    def plan(self):
        return B.mmm_matmul_plan(self.maps, self.dtype)

    def set_plan(self, variant: int = -1, split_k: int = 0) -> None:
        B.mmm_maps_set_plan(self.maps, variant, split_k)

    def autotune(self, X: torch.Tensor, Y: torch.Tensor, C: torch.Tensor, splits=(0,), reps: int = 20):
        """Time every tile variant (and the given K splits) on the maps as built, with the caller's operands, and fix
        the fastest as this handle's plan.  Returns [(microseconds, variant, split_k)] sorted by time.  C is
        overwritten."""
        results = []
        for v in range(B.mmm_matmul_variant_count()):
            for sp in splits:
                self.set_plan(v, sp)
                pv, ps, _ = self.plan()
                if pv != v or any(r[1] == pv and r[2] == ps for r in results):
                    continue   # not usable for this shape, or the same plan as one already timed
                for _ in range(3):
                    self.matmul(X, Y, C)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    self.matmul(X, Y, C)
                e1.record()
                torch.cuda.synchronize()
                results.append((e0.elapsed_time(e1) * 1e3 / reps, pv, ps))
        results.sort()
        self.set_plan(results[0][1], results[0][2])
        return results

    def _bits_tensor(self, addr: int, rows: int, words: int) -> torch.Tensor:
        off = addr - self.workspace.data_ptr()
        assert 0 <= off and off + rows * words * 8 <= self.workspace.numel()
        return self.workspace[off: off + rows * words * 8].view(torch.int64).view(rows, words)

    def a_bits(self) -> torch.Tensor:
        a, aw, _, _ = B.mmm_maps_view(self.maps)
        return self._bits_tensor(a, self.M, aw)

    def b_bits(self) -> torch.Tensor:
        _, _, b, bw = B.mmm_maps_view(self.maps)
        return self._bits_tensor(b, self.K, bw)

    def a_colany(self) -> torch.Tensor:
        a, _, kw = B.mmm_maps_view_derived(self.maps)
        return self._bits_tensor(a, (self.M + 31) // 32, kw)

    def bt_bits(self) -> torch.Tensor:
        _, b, kw = B.mmm_maps_view_derived(self.maps)
        return self._bits_tensor(b, self.N // self.bw, kw)

    def compacted(self):
        """None unless the B side was built with keep_rows; else (live_count int32 [1], kmap int32 [K], a_colany_c int64
        [ceil(M/32), ceil(K/64)], btc_bits int64 [NB, ceil(K/64)]) as views of the workspace."""
        on, kc, km, ca, bt = B.mmm_maps_view_compacted(self.maps)
        if not on:
            return None
        base = self.workspace.data_ptr()
        wa = (self.K + 63) // 64

        def view(addr, nbytes, dt):
            assert 0 <= addr - base and addr - base + nbytes <= self.workspace.numel()
            return self.workspace[addr - base: addr - base + nbytes].view(dt)

        return (view(kc, 4, torch.int32), view(km, self.K * 4, torch.int32),
                view(ca, ((self.M + 31) // 32) * wa * 8, torch.int64).view(-1, wa),
                view(bt, (self.N // self.bw) * wa * 8, torch.int64).view(-1, wa))

    def k_lists(self) -> torch.Tensor:
        """The matrix kernel's per-tile active-k lists as uint8 [row tiles, column groups, steps, 132] (4-byte count,
        then the list bytes); see mmm_debug_k_lists."""
        need = B.mmm_debug_k_lists(self.maps)
        out = torch.zeros(need, dtype=torch.uint8, device=self.device)
        B.mmm_debug_k_lists(self.maps, out, need)
        tm, groups, steps = (self.M + 63) // 64, 16 * ((self.N + 255) // 256), (self.K + 127) // 128
        return out.view(tm, groups, steps, 132)

    def a_lists(self):
        """(counts int32 [blocks_m, blocks_k], entries int64 [blocks_m * blocks_k, capacity]) as views of the workspace."""
        c, e, bm, bk, cap = B.mmm_maps_view_lists(self.maps)
        base = self.workspace.data_ptr()
        assert 0 <= c - base and c - base + bm * bk * 4 <= self.workspace.numel()
        assert 0 <= e - base and e - base + bm * bk * cap * 8 <= self.workspace.numel()
        counts = self.workspace[c - base: c - base + bm * bk * 4].view(torch.int32).view(bm, bk)
        entries = self.workspace[e - base: e - base + bm * bk * cap * 8].view(torch.int64).view(bm * bk, cap)
        return counts, entries
