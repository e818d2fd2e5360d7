"""Detection on a few small batches of every configuration shape, under a set of the library's diagnostic flags.

Used by the GPU test that compares a plain run with a run under QRM_DIAG_POISON_WORKSPACE (every new workspace is
filled with 0xFF bytes, NaN as bf16 and as fp32: a kernel that reads workspace bytes which no kernel wrote would
show up as a difference, or as NaN) or QRM_DIAG_NO_FUSED_PAIRS (one launch per block).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

CASES = [("C1", 16, 0), ("C2", 40, 16), ("C2", 7, 0), ("C4", 5, 2), ("C3", 2, 1)]   # configuration, images, micro-batch


def run_cases(diag_flags=0):
    import torch
    import synth
    import paper_2509_02447_amd as q

    out = {}
    for name, N, mb in CASES:
        cfg = synth.CONFIGS[name]
        ctx = q.Context(weights=synth.config_weights(cfg),
                        rs=dict(m=cfg.m, prim_poly=cfg.prim_poly, n=cfg.n, k=cfg.k, fcr=cfg.fcr))
        ctx.qrm_diag_set_flags(diag_flags)
        if mb:
            ctx.qrm_set_micro_batch(mb)
        imgs = torch.from_numpy(synth.images(cfg, 7, N)).cuda()
        off = torch.from_numpy(synth.offsets(cfg, 7, N)).cuda()
        logits = torch.empty((N, cfg.n_bits), dtype=torch.float32, device="cuda")
        msg = torch.empty((N, cfg.k), dtype=torch.uint8, device="cuda")
        nerr = torch.empty((N,), dtype=torch.int8, device="cuda")
        for rep in range(2):    # the second call reuses the workspace the first one left
            ctx.qrm_detect(imgs, N, cfg.H, cfg.W, off, cfg.tile, logits, None, msg, None, nerr)
            torch.cuda.synchronize()
            out[f"{name}_{N}_{rep}_logits"] = logits.cpu().numpy()
            out[f"{name}_{N}_{rep}_msg"] = msg.cpu().numpy()
        ctx.close()
    return out
