"""Helpers shared by the GPU parity tests: build the HIP model and the oracle model from the
same seeded weights, fill both caches the same way."""
import numpy as np
import torch

import csd_inputs as I


def tol_ok(got, ref, rtol, atol):
    err = np.abs(got - ref)
    return bool((err <= atol + rtol * np.abs(ref)).all()), float(err.max())


def make_pair(shape, seed, max_batch, max_seq, max_block, std=0.02):
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    w = I.make_weights(shape, seed, device="cuda", std=std)
    gm = P.Model(shape, w, max_batch=max_batch, max_seq=max_seq, max_block=max_block)
    om = O.Model(shape, [x.cpu() for x in w], max_batch=max_batch, max_seq=max_seq, max_block=max_block)
    return gm, om


def prefill_both(gm, om, tokens_2d, chunk):
    """Run both models over tokens [B][t] from an empty cache, `chunk` rows at a time."""
    B, t = tokens_2d.shape
    for pos in range(0, t, chunk):
        blk = tokens_2d[:, pos:pos + chunk].contiguous()
        cl = torch.full((B,), pos, dtype=torch.int32)
        gm.verify_block(blk.cuda(), cl.cuda())
        om.verify_block(blk.numpy(), cl.numpy())


def import_synthetic_kv(gm, om, shape, n_rows, seed, B=1, std=1.0):
    """Fill rows [0, n_rows) of every layer's cache of both models with the same seeded values."""
    for l in range(shape.n_layers):
        for b in range(B):
            K, V = I.synthetic_kv(shape, n_rows, seed, l, b, device="cuda", std=std)
            gm.kv_write(l, b, 0, K.contiguous(), V.contiguous())
            if om is not None:
                om.kv_write(l, b, 0, K.cpu().numpy(), V.cpu().numpy())
    torch.cuda.synchronize()
