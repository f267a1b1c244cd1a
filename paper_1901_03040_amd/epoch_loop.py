"""Host-side driver of the QESGD epoch loop (Alg. 2 / Alg. 3) on top of the C-ABI binding.

It owns the device buffers of one parameter vector (snapshot w_t, deviation z, working point
u = w_t + z, running sum of the z iterates) and sequences the library calls; all arithmetic runs
in the library's kernels.  Gradients are the caller's: each round the caller hands in the
workers' candidate deviations z_hat_k = z - eta * g_k (compress-on-push form) or the server's
z_hat = z - (eta / B) * sum_k g_k (Alg. 3 as written).
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class QesgdEpochLoop:
    def __init__(self, w0: torch.Tensor, K: int, seed: int, *, s: int = 256, bucket: int = 512,
                 fixed_bits: Optional[int] = None):
        """w0: fp32 CUDA vector (copied).  K workers.  Bucketed quantiser (s, bucket) for the
        push form; fixed_bits selects the paper's fixed-grid quantiser for the server form."""
        assert w0.is_cuda and w0.dtype == torch.float32 and w0.dim() == 1
        self.d, self.K, self.seed = w0.numel(), K, seed
        self.s, self.bucket, self.fixed_bits = s, bucket, fixed_bits
        dev = w0.device
        self.w = w0.clone()
        self.z = torch.zeros_like(w0)
        self.u = w0.clone()
        self.zsum = torch.zeros_like(w0)
        self.step = torch.zeros_like(w0)   # mean of the workers' quantised steps (gradient_round)
        self.round_id = 0          # global round counter: a new set of variates every round
        self.steps_in_epoch = 0
        self.lay = B.qesgd_layout_query(self.d, s, bucket)
        self.packed = B.alloc_packed(self.lay, K, dev)
        if fixed_bits is not None:
            self.codes = torch.empty((self.d * fixed_bits + 31) // 32, dtype=torch.int32, device=dev)
        wsb = B.qesgd_workspace_bytes(self.d, s, bucket, K)
        self.ws = torch.empty(wsb // 4, dtype=torch.float32, device=dev) if wsb else None

    def begin_epoch(self):
        """z_{t,0} = 0, u_{t,0} = w_t (first step of Alg. 2 / Alg. 3)."""
        self.z.zero_()
        self.zsum.zero_()
        self.u.copy_(self.w)
        self.steps_in_epoch = 0

    def _zsum_arg(self, last: bool):
        # The epoch mean runs over the iterates k = 0 .. K_t - 1 (Alg. 2): z_{t,0} = 0 needs no
        # add, z_{t,k} is added when step k produces it, and the iterate of the last step stays out.
        return None if last else self.zsum

    def push_round(self, z_hat_slab: torch.Tensor, last: bool = False) -> torch.Tensor:
        """Compress-on-push round: row k of z_hat_slab is worker k's z - eta * g_k.
        z <- (1/K) sum_k Q(z_hat_k), u <- w_t + z.  Returns u."""
        assert z_hat_slab.shape[0] == self.K and z_hat_slab.stride(0) % 4 == 0
        # both halves of the round in one call (one launch for power-of-two buckets)
        B.qesgd_round(z_hat_slab, z_hat_slab.stride(0), None, self.d, self.s, self.bucket, B.NORM_L2, self.seed,
                      self.round_id, self.K, self.packed, self.packed.stride(0), self.w, self.z, self.u,
                      self._zsum_arg(last), workspace=self.ws)
        self.round_id += 1
        self.steps_in_epoch += 1
        return self.u

    def gradient_round(self, step_slab: torch.Tensor, last: bool = False) -> torch.Tensor:
        """Gradient-compression baseline (QSGD as compared in Sec. 5): row k of step_slab is worker
        k's -eta * g_k, quantised with the scale of what is sent (per bucket, or one scale over the
        whole vector when bucket >= d).  z <- z + (1/K) sum_k Q(-eta g_k), u <- w_t + z.  Returns u."""
        assert step_slab.shape[0] == self.K and step_slab.stride(0) % 4 == 0
        B.qesgd_quantize_pack_batched(step_slab, step_slab.stride(0), None, self.d, self.s, self.bucket,
                                      B.NORM_L2, self.seed, self.round_id, self.K, self.packed,
                                      self.packed.stride(0), self.ws)
        B.qesgd_unpack_aggregate(self.packed, self.packed.stride(0), self.K, self.d, self.s, self.bucket, self.step)
        B.qesgd_apply_update(self.z, self.step, self.z, None, self.d)              # z += mean step
        B.qesgd_apply_update(self.w, self.z, self.u, self._zsum_arg(last), self.d)  # u = w_t + z, zsum += z
        self.round_id += 1
        self.steps_in_epoch += 1
        return self.u

    def server_round(self, z_hat: torch.Tensor, delta: float, last: bool = False) -> torch.Tensor:
        """Alg. 3, server task: z <- Q_{delta,b}(z_hat) on the fixed grid, u <- w_t + z.  Returns u."""
        assert self.fixed_bits is not None
        B.qesgd_quantize_fixed(z_hat, None, self.d, delta, self.fixed_bits, self.seed, self.round_id, 0, self.codes)
        B.qesgd_dequantize_fixed_update(self.codes, self.d, delta, self.fixed_bits, self.w, self.z, self.u,
                                        self._zsum_arg(last))
        self.round_id += 1
        self.steps_in_epoch += 1
        return self.u

    def end_epoch(self) -> torch.Tensor:
        """w_{t+1} = w_t + (1/K_t) sum_{k<K_t} z_{t,k} (last step of Alg. 3).  Returns w_{t+1}."""
        assert self.steps_in_epoch > 0
        B.qesgd_epoch_commit(self.w, self.zsum, self.steps_in_epoch, self.d)
        return self.w
