"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import oracle
from paper_2601_07048_amd import datagen


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def random_data(n, d, dtype, seed):
    rng = np.random.default_rng(seed)
    if dtype == np.uint8:
        c = rng.integers(40, 216, (8, d))
        x = c[rng.integers(0, 8, n)] + rng.normal(0, 25, (n, d))
        return np.clip(np.rint(x), 0, 255).astype(np.uint8)
    c = rng.standard_normal((8, d))
    return (c[rng.integers(0, 8, n)] + 0.5 * rng.standard_normal((n, d))).astype(np.float32)


def oracle_index(x, R, L_build, alpha=1.2):
    ix = oracle.Index(x.shape[1], x.dtype, R, L_build, alpha, len(x))
    ix.insert(x)
    return ix


def jx_dtype(jx, x):
    return {np.dtype(np.uint8): jx.U8, np.dtype(np.float32): jx.F32, np.dtype(np.float16): jx.F16}[x.dtype]


def gpu_index_from_oracle(jx, x, ix, R, L_build, quant_bits=0, capacity=None):
    adj, deg = ix.graph()
    g = jx.Index(x.shape[1], jx_dtype(jx, x), R, L_build, 1.2,
                 capacity=capacity or len(x), max_batch=max(1024, len(x)), quant_bits=quant_bits)
    g.import_graph(dev(x), dev(adj), ix.entry)
    return g
