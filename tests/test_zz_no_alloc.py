"""csd_verify_accept_static (scratch in the library's static device array, no allocation) against
csd_verify_accept (scratch in the model) through the C ABI: logits and probabilities element by element,
accepted lengths and emitted tokens bit for bit, on two calls in a row of which the second is smaller."""
import numpy as np
import pytest
import torch

import csd_inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    P.lib()


def _one_call(gm, block, cache_len, q, onehot, seed, static):
    B, m = block.shape
    k = m - 1
    V = gm.shape.vocab
    u_acc = I.uniforms(B * max(k, 1), seed, 7).reshape(B, -1)[:, :max(k, 1)].contiguous().cuda()
    u_s = I.uniforms(B, seed, 8).cuda()
    logits = torch.full((B, m, V), float("nan"), dtype=torch.float32, device="cuda")
    probs = torch.full((B, m, V), float("nan"), dtype=torch.float32, device="cuda")
    n, x = gm.verify_accept(block, cache_len, u_acc, u_s, q=q, q_onehot=onehot, logits=logits, probs=probs,
                            static=static)
    torch.cuda.synchronize()
    return logits.cpu().numpy(), probs.cpu().numpy(), n.cpu().numpy(), x.cpu().numpy()


def test_static_scratch_entry_point_equals_the_allocating_one():
    import paper_2312_11462_amd as P
    shape = I.ModelShape("noalloc", 0, "bf16", 3, 256, 4, 64, 704, 1024)
    seed = 0x5C2A
    w = I.make_weights(shape, seed, device="cuda", std=0.05)
    gm = P.Model(shape, w, max_batch=7, max_seq=160, max_block=8)
    assert gm.path(7, 8) == 0 and gm.path(1, 3) == 1     # the two calls below take the two forwards
    toks = I.token_ids(7 * 120, shape.vocab, seed, 1).reshape(7, 120).cuda()
    # prefill 96 rows per sequence through the ordinary entry point
    for pos in range(0, 96, 8):
        gm.verify_block(toks[:, pos:pos + 8].contiguous(), torch.full((7,), pos, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    kv0 = gm.kv.clone()
    V = shape.vocab
    # call 1: 7 sequences x 8 rows, dense draft distributions; call 2: 1 sequence x 3 rows, deterministic drafts
    calls = [(toks[:, 96:104].contiguous(), torch.tensor([96, 90, 77, 96, 81, 64, 95], dtype=torch.int32, device="cuda"), True),
             (toks[:1, 100:103].contiguous(), torch.tensor([41], dtype=torch.int32, device="cuda"), False)]
    results = {}
    for static in (False, True):
        gm.kv.copy_(kv0)
        out = []
        for j, (block, cl, dense) in enumerate(calls):
            B, m = block.shape
            q = None
            if dense:
                q = torch.softmax(I.normal((B, m - 1, V), 2.0, seed, 50 + j, device="cuda"), dim=-1).contiguous()
            out.append(_one_call(gm, block, cl, q, None, seed + j, static))
        results[static] = (out, gm.kv.clone())
    for j in range(len(calls)):
        a, b = results[False][0][j], results[True][0][j]
        assert not np.isnan(b[0]).any() and not np.isnan(b[1]).any()
        # same kernels, same launch shapes, same order of every sum: the two must agree to the bit
        assert np.array_equal(a[0], b[0]), f"call {j}: logits differ, max {np.abs(a[0] - b[0]).max()}"
        assert np.array_equal(a[1], b[1]), f"call {j}: probabilities differ"
        assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3]), f"call {j}: accept differs"
    assert torch.equal(results[False][1], results[True][1]), "cache rows written differ"


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2312_11462_amd as P
    from paper_2312_11462_amd.binding import CsdError
    # scratch grows with max_batch * max_block * vocab: 64 rows x 32768 logits x 4 B alone exceed 8 MiB
    shape = I.ModelShape("toolarge", 0, "bf16", 1, 128, 2, 64, 256, 32768)
    w = I.make_weights(shape, 3, device="cuda")
    gm = P.Model(shape, w, max_batch=8, max_seq=64, max_block=8)
    block = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    cl = torch.zeros(1, dtype=torch.int32, device="cuda")
    u = torch.zeros((1, 1), dtype=torch.float32, device="cuda")
    with pytest.raises(CsdError) as e:
        gm.verify_accept(block, cl, u, u[0], static=True)
    assert e.value.status == -2
    gm.verify_accept(block, cl, u, u[0])          # the allocating entry point still takes it
    torch.cuda.synchronize()
