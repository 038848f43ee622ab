"""Run a workloads.Problem through libtcx on the GPU (torch supplies device memory and the
stream only)."""
from __future__ import annotations

import sys

import numpy as np

import workloads as W

DT = {"f32": 0, "f64": 1, "c64": 2, "c128": 3, "f16": 4, "bf16": 5}


def say(msg: str):
    sys.stdout.write("[gpu] %s\n" % msg)
    sys.stdout.flush()


class GpuProduct:
    """Plan for one Problem: tensor infos + product + executor on torch's current stream."""

    def __init__(self, p: W.Problem, force_path=None, variant=None, split_k=None, precision=0):
        import torch
        import paper_2601_07827_amd as T
        self.T, self.p = T, p
        self.dtype = DT[p.dtype]
        ids = W.label_ids(p)
        self.h = T.tcx_create_handle()
        assert T.tcx_handle_has_device(self.h), "no gfx950 device bound"
        self.ex = T.tcx_create_executor(self.h, torch.cuda.current_stream().cuda_stream)
        ia = T.tcx_create_tensor_info(self.h, self.dtype, p.A.extents, p.A.strides)
        ib = T.tcx_create_tensor_info(self.h, self.dtype, p.B.extents, p.B.strides)
        idd = T.tcx_create_tensor_info(self.h, self.dtype, p.D.extents, p.D.strides)
        la, lb, ld = ([ids[l] for l in t.labels] for t in (p.A, p.B, p.D))
        self.prod = T.tcx_create_product(self.h, p.opA, ia, la, p.opB, ib, lb, p.opC, idd, ld, 0, idd, ld, precision)
        for i in (ia, ib, idd):
            T.tcx_destroy_tensor_info(i)       # the plan keeps its own copy
        if force_path is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_FORCE_PATH, force_path)
        if variant is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_VARIANT, variant)
        if split_k is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_SPLIT_K, split_k)

    def get(self, key):
        return self.T.tcx_product_get(self.prod, key)

    def execute(self, dA, dB, dC, dD, alpha=None, beta=None):
        """dX: torch device tensors (1-D buffers).  dC may be dD (in place) or None."""
        p, T = self.p, self.T
        item = dD.element_size()
        al = p.alpha if alpha is None else alpha
        be = p.beta if beta is None else beta
        st = T.tcx_execute_product(self.prod, self.ex, self.dtype, al,
                                   dA.data_ptr() + p.A.base * item, dB.data_ptr() + p.B.base * item, be,
                                   0 if dC is None else dC.data_ptr() + p.D.base * item,
                                   dD.data_ptr() + p.D.base * item, want_status=True)
        self.last_path = T.tcx_status_get(st, T.TCX_KEY_PATH)
        self.last_variant = T.tcx_status_get(st, T.TCX_KEY_VARIANT)
        self.last_gather_width = T.tcx_status_get(st, T.TCX_KEY_GATHER_WIDTH)
        assert T.tcx_status_get(st, T.TCX_KEY_HIP_ERROR) == 0
        assert T.tcx_destroy_status(st) == 0

    def close(self):
        self.T.tcx_destroy_product(self.prod)
        self.T.tcx_destroy_executor(self.ex)
        self.T.tcx_destroy_handle(self.h)


def run_gpu(p: W.Problem, bufA, bufB, bufC, force_path=None, variant=None, alpha=None, beta=None, c_null=False,
            split_k=None, precision=0):
    """D buffer (numpy) after D := alpha op(A) op(B) + beta op(C), computed in place over a copy of bufC."""
    import torch
    gp = GpuProduct(p, force_path, variant, split_k, precision)
    try:
        dA, dB = torch.from_numpy(bufA).cuda(), torch.from_numpy(bufB).cuda()
        dD = torch.from_numpy(bufC.copy()).cuda()
        gp.execute(dA, dB, None if c_null else dD, dD, alpha, beta)
        torch.cuda.synchronize()
        if force_path is not None and (alpha is None or alpha != 0):
            assert gp.last_path == force_path, "the forced path did not run"
        if variant is not None and force_path != 2:
            assert gp.last_variant == variant
        return dD.cpu().numpy()
    finally:
        gp.close()
