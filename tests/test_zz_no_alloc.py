"""GPU: vf_score_static (the entry point that allocates nothing) against vf_score."""
import numpy as np
import pytest

from paper_2011_14486_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vf():
    import paper_2011_14486_amd as pkg
    return pkg.load()


def raw(F, M, seed):
    rng = np.random.default_rng(seed)
    return np.floor(np.exp2(rng.random((F, M)) * 20.0)).astype(np.int32)


@pytest.mark.parametrize("dims", [[256, 1024, 1024, 1024, 1], [256, 512, 512, 1], [64, 96, 32, 1]])
def test_static_scratch_mlp_equals_vf_score(vf, ovf, dims):
    """Two calls in a row through the C ABI, the second with a smaller input (the array keeps the
    first call's minima behind the part the second one uses): scores, group winners and their
    values must be bit-identical to vf_score's, and that in turn is checked against the checker."""
    import torch
    from tests.util import TOL, score_err
    w = I.mlp_weights(dims, seed=11, bias_std=0.1)
    model = I.model_record(I.MLP, dims, I.BF16)
    ctx = vf.vf_create(0)
    vf.vf_set_model(ctx, model, w)
    assert vf.vf_score_static_max(ctx) == (64 if max(dims) > 512 else 128) * 65536
    for M, group in ((20000, 4096), (1500, 256)):
        x = raw(dims[0], M, seed=M)
        xd = torch.from_numpy(x).cuda()
        out = (ctx.empty((M,), torch.float32), ctx.empty(((M + group - 1) // group,), torch.int32),
               ctx.empty(((M + group - 1) // group,), torch.float32))
        s1, i1, v1 = vf.vf_score_static(ctx, xd, vf.VF_X_RAW_I32, group=group, out=out)
        s1, i1, v1 = s1.clone(), i1.clone(), v1.clone()
        s0, i0, v0 = vf.vf_score(ctx, xd, vf.VF_X_RAW_I32, group=group)
        torch.cuda.synchronize()
        assert torch.equal(s0, s1) and torch.equal(i0, i1) and torch.equal(v0, v1)
        # again, now that the kernels' code is loaded: the call takes no device memory
        for t in out:
            t.zero_()
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        s2, i2, v2 = vf.vf_score_static(ctx, xd, vf.VF_X_RAW_I32, group=group, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0
        assert torch.equal(s0, s2) and torch.equal(i0, i2) and torch.equal(v0, v2)
        ref = ovf.score_mlp(model, w, x[:, :2048].copy())
        assert score_err(s1.cpu().numpy()[:2048], ref) <= TOL[1]
    vf.vf_destroy(ctx)


def test_static_scratch_lstm_and_limits(vf, ovf):
    import torch
    F, H, T = 64, 96, 5
    w = I.lstm_weights(F, H, seed=3, bias_std=0.1)
    ctx = vf.vf_create(0)
    vf.vf_set_model(ctx, I.model_record(I.LSTM, [F, H, 1], I.BF16), w)
    for B in (700, 130):
        xb = I.feature_sequences(0, 768, T=T, F=F, seed=9)[:B]
        xd = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        s1, i1, v1 = vf.vf_score_static(ctx, xd, vf.VF_X_SEQ_BF16)
        s0, i0, v0 = vf.vf_score(ctx, xd, vf.VF_X_SEQ_BF16)
        torch.cuda.synchronize()
        assert torch.equal(s0, s1) and torch.equal(i0, i1) and torch.equal(v0, v1)
    # beyond the array: refused, nothing launched
    lim = vf.vf_score_static_max(ctx)
    assert lim == 64 * 65536
    dummy = torch.zeros((1, T, F), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(vf.VfError) as e:
        vf.vf_score_static(ctx, dummy, vf.VF_X_SEQ_BF16, M=lim + 1, out=(None, ctx.empty((1,), torch.int32),
                                                                            ctx.empty((1,), torch.float32)))
    assert e.value.code == vf.VF_EINVAL
    # fp32 models keep activation matrices in scratch: refused
    d = [64, 32, 1]
    vf.vf_set_model(ctx, I.model_record(I.MLP, d, I.FP32), I.mlp_weights(d, 1))
    assert vf.vf_score_static_max(ctx) == 0
    with pytest.raises(vf.VfError) as e:
        vf.vf_score_static(ctx, torch.zeros((64, 8), dtype=torch.int32, device="cuda"))
    assert e.value.code == vf.VF_EINVAL
    vf.vf_destroy(ctx)
