"""ecoserve_attn_decode_noalloc (the decode call for callers that cannot allocate) against
ecoserve_attn_decode on the same inputs: two calls in a row, the second with a smaller batch, so that
what the first call left in the shared scratch array would show if the second relied on it."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2504_18154_amd import binding
from paper_2504_18154_amd import workloads as wl
from tests.parity_util import Layer, compare, compare_lse, dev_i32, say

pytestmark = pytest.mark.gpu


def _decode_both_ways(model, ctx_len, seed):
    pb = wl.prefill_batch(model, ctx_len, seed)
    layer = Layer(model, pb.num_blocks, max_batch=pb.B, max_blocks_per_seq=pb.block_table.shape[1])
    k = wl.randn((pb.T, model.Hkv, model.D), model.dtype, seed + 1)
    v = wl.randn((pb.T, model.Hkv, model.D), model.dtype, seed + 2)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    q = wl.randn((pb.B, model.Hq, model.D), model.dtype, seed + 3)
    lens = np.asarray(ctx_len, dtype=np.int32)
    want, want_lse = layer.decode_gpu(q, pb.block_table, lens)            # the existing entry point
    ref, ref_lse = layer.decode_oracle(q, pb.block_table, lens)
    qd = q.cuda()
    got = torch.full_like(qd, float("nan"))
    got_lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
    st = binding.attn_decode_noalloc(layer.ctx.layout, qd, layer.kc, layer.vc, dev_i32(pb.block_table), dev_i32(lens),
                                     got, int(lens.max()), got_lse)
    assert st == binding.OK, binding.strerror(st)
    torch.cuda.synchronize()
    # to the bar of the parity tests against the existing entry point's output ...
    compare("noalloc vs ecoserve_attn_decode", got, want.double().cpu().numpy(), "bf16")
    compare_lse("noalloc vs ecoserve_attn_decode", got_lse, want_lse.double().cpu().numpy(), "bf16")
    # ... and against the oracle; the two calls launch the same kernels over the same chunks, so the bits agree too
    compare("noalloc vs oracle", got, ref, "bf16")
    compare_lse("noalloc vs oracle", got_lse, ref_lse, "bf16")
    assert torch.equal(got.view(torch.int16), want.view(torch.int16)), "outputs differ in bits"
    assert torch.equal(got_lse, want_lse), "log-sum-exps differ in bits"
    layer.close()


def test_noalloc_decode_matches_the_context_call_twice_in_a_row():
    model = wl.ModelShape("30B-heads", 40, 8, 128, 1, "bf16")
    rng = np.random.default_rng(2024)
    say("noalloc decode: 96 sequences, contexts 1..3000 (most (sequence, head)s cut between wavefronts)")
    _decode_both_ways(model, np.r_[1, 15, 16, 17, 2049, rng.integers(1, 3000, size=91)].astype(np.int32), 901)
    say("noalloc decode: 5 sequences right after it (the scratch array still holds the larger call's states)")
    _decode_both_ways(model, np.array([700, 3, 64, 1, 129], dtype=np.int32), 902)
    say("noalloc decode: group size 8, one long sequence cut into hundreds of pieces")
    _decode_both_ways(wl.ModelShape("70B-heads", 64, 8, 128, 1, "bf16"), np.array([8000, 40], dtype=np.int32), 903)


def test_noalloc_decode_rejects_what_it_cannot_hold():
    lay = binding.make_layout(40, 8, 128, 64, "bf16")
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    bt = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    f = binding._lib.ecoserve_attn_decode_noalloc
    vp = lambda x: ctypes.c_void_p(x.data_ptr())
    args = lambda B, mcl: (0, ctypes.byref(lay), vp(t), vp(t), vp(t), vp(bt), 4, vp(t), vp(t), None, B, mcl, None)
    assert f(*args(4097, 16)) == binding.EINVAL          # more sequences than the scratch array is sized for
    assert f(*args(1, 65)) == binding.EINVAL             # max_ctx_len beyond the block table
    assert f(*args(0, 16)) == binding.OK                 # empty batch: nothing to do
    lay32 = binding.make_layout(4, 2, 64, 64, "f32")
    assert f(0, ctypes.byref(lay32), vp(t), vp(t), vp(t), vp(bt), 4, vp(t), vp(t), None, 1, 16, None) == binding.EUNSUPPORTED
    assert f(64, ctypes.byref(lay), vp(t), vp(t), vp(t), vp(bt), 4, vp(t), vp(t), None, 1, 16, None) == binding.EINVAL
