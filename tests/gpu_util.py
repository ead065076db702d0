"""Helpers for the GPU parity tests: move seeded inputs to the device, call the library through
its binding, bring results back as float64 numpy."""
import numpy as np
import torch

import paper_2511_00413_amd as T


def dev(x):
    return x.to("cuda") if isinstance(x, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(x)).to("cuda")


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def gpu_attention(meta, q, k, v, d_o=None, *, k_prefix=None, v_prefix=None, scale=None,
                  reference_kernels=False, prefix_acc=None):
    """meta: TreeMeta from tree_build_meta (with n_prefix matching k_prefix).  CPU tensors in,
    dict of float64 numpy out (o, lse, dq, dk, dv, dk_prefix, dv_prefix)."""
    qd, kd, vd = dev(q), dev(k), dev(v)
    kend, kmin, kmax = dev(meta.kend), dev(meta.ktile_kend_min), dev(meta.ktile_kend_max)
    kp = None if k_prefix is None else dev(k_prefix)
    vp = None if v_prefix is None else dev(v_prefix)
    o, lse = T.tree_attn_fwd(qd, kd, vd, kend, kmin, kmax, k_prefix=kp, v_prefix=vp, scale=scale,
                             reference_kernels=reference_kernels)
    out = dict(o=f64(o), lse=f64(lse), o_dev=o, lse_dev=lse)
    if d_o is not None:
        dod = dev(d_o)
        dkp = dvp = None
        if kp is not None:
            if prefix_acc is None:
                dkp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
                dvp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
            else:
                dkp, dvp = prefix_acc
        dq, dk, dv = T.tree_attn_bwd(qd, kd, vd, kend, kmin, kmax, o, dod, lse, k_prefix=kp, v_prefix=vp,
                                     dk_prefix_acc=dkp, dv_prefix_acc=dvp, scale=scale,
                                     reference_kernels=reference_kernels)
        out.update(dq=f64(dq), dk=f64(dk), dv=f64(dv), dq_dev=dq, dk_dev=dk, dv_dev=dv)
        if kp is not None:
            out.update(dk_prefix=f64(dkp), dv_prefix=f64(dvp))
    torch.cuda.synchronize()
    return out
