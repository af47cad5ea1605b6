"""jx_bruteforce_static (the entry point for callers that cannot allocate device memory) against jx_bruteforce,
through the C ABI: identical ids and distances, on two calls in a row of which the second is smaller (the scratch
array keeps the first call's contents), for every storage type; sizes beyond the static scratch are refused before
anything is launched."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2601_07048_amd import jx  # noqa: E402

from gpu_common import dev, random_data, u32  # noqa: E402


def _index(x, dtype):
    g = jx.Index(x.shape[1], dtype, 8, 16, 1.2, capacity=len(x), max_batch=max(1024, len(x)))
    # brute force only reads the vector store: install the vectors with an empty graph
    adj = np.full((len(x), 8), 0xFFFFFFFF, np.uint32)
    g.import_graph(dev(x), dev(adj), 0)
    return g


@pytest.mark.parametrize("kind", ["u8", "f32", "f16"])
def test_static_scratch_bruteforce_equals_arena_bruteforce(kind):
    d = {"u8": 128, "f32": 100, "f16": 104}[kind]
    x = random_data(6000 + 37, d, np.uint8 if kind == "u8" else np.float32, 11)
    q = random_data(700 + 5, d, np.uint8 if kind == "u8" else np.float32, 12)
    if kind == "f16":
        x, q = x.astype(np.float16), q.astype(np.float16)
    dt = {"u8": jx.U8, "f32": jx.F32, "f16": jx.F16}[kind]
    dx, dq = dev(x), dev(q)
    # the first call on a GPU resolves the scratch symbol, which makes the runtime load the code object that holds
    # the array; from then on a call leaves the amount of free device memory alone
    jx.bruteforce_static(dx[:64], dq[:1], 1)
    # first call: the larger one (705 queries, k = 20, 6037 base vectors); second: fewer queries, fewer base
    # vectors, smaller k, so most of the scratch still holds the first call's lists
    for n, nq, k in ((len(x), len(q), 20), (1500 + 3, 130, 7)):
        g = _index(x[:n], dt)
        want_ids, want_dist = g.bruteforce(dq[:nq], k)
        out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        ids, dist = jx.bruteforce_static(dx[:n], dq[:nq], k, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0, "the call changed the amount of free device memory"
        assert np.array_equal(u32(ids), u32(want_ids)), (kind, n, nq, k)
        assert np.array_equal(dist.cpu().numpy().view(np.uint32), want_dist.cpu().numpy().view(np.uint32)), (kind, n, nq, k)
        # and against the definition, on a sample (exact integers for uint8)
        if kind == "u8":
            xs, qs = x[:n].astype(np.int64), q[:16].astype(np.int64)
            dd = ((qs[:, None, :] - xs[None, :, :]) ** 2).sum(-1)
            order = np.lexsort((np.broadcast_to(np.arange(n), dd.shape), dd), axis=1)[:, :k]
            assert np.array_equal(u32(ids)[:16], order.astype(np.uint32))


def test_static_scratch_limit_is_enforced():
    x = dev(random_data(4096, 32, np.uint8, 3))
    # 40,000 queries at k = 128: nsplit = 4, 40,000 * 4 * 128 * 8 = 164 MB of partial lists > 16 MiB
    q = dev(random_data(40000, 32, np.uint8, 4))
    with pytest.raises(jx.JxError) as e:
        jx.bruteforce_static(x, q, 128)
    assert e.value.code == -2 and "static scratch" in str(e.value)
    # the largest k still fits for a small batch
    ids, _ = jx.bruteforce_static(x, q[:200], 128)
    torch.cuda.synchronize()
    assert int(ids.min()) >= 0 and int(ids.max()) < 4096
