"""The entry point that allocates nothing (sushi_infer_static: activations in the library's static device
array) against sushi_infer in exec mode 0, the entry point it is a variant of: same kernels, same order, so the
logits must agree bit for bit; also within the usual tolerance of the CPU oracle.  Two calls in a row, the
second on a smaller input, and a request beyond the array's size."""
import numpy as np
import pytest
import torch

from tests.common import make_problem, oracle_logits, rel_l2
from workloads import arch as A
from workloads import tensors as T

pytestmark = pytest.mark.gpu


def _pair(ctx, cfg, x, n_classes):
    a = torch.full((x.shape[0], n_classes), float("nan"), device="cuda")
    b = torch.full((x.shape[0], n_classes), float("nan"), device="cuda")
    ctx.sushi_infer(cfg, x, a)
    ctx.sushi_infer_static(cfg, x, b)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


@pytest.mark.parametrize("fam,bf16", [("mbv3", True), ("resnet", True), ("tiny", False)])
def test_static_scratch_entry_point_matches_sushi_infer(fam, bf16):
    import paper_2306_17266_amd as S
    arch = {"tiny": A.tiny_arch, "resnet": A.small_resnet_arch, "mbv3": A.small_mbv3_arch}[fam]()
    blob, wts = make_problem(arch, 13, bf16)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16 if bf16 else S.FP32)
    big, small = max(arch.res_choices), min(arch.res_choices)
    # first the largest SubNet on a batch of 3 at the larger resolution, then the smallest SubNet on one image
    # at the smaller resolution (its buffers are cut differently out of the same array), then the first again
    calls = [(A.max_cfg(arch, big), 3), (A.min_cfg(arch, small), 1), (A.max_cfg(arch, big), 3)]
    for t, (cfg, batch) in enumerate(calls):
        print(fam, "call", t, "batch", batch, "resolution", cfg.resolution, flush=True)
        x_np = T.make_input(13, t, batch, cfg.resolution, 3, bf16)
        x = torch.from_numpy(x_np).cuda()
        x = (x.to(torch.bfloat16) if bf16 else x).contiguous()
        want, got = _pair(ctx, cfg, x, arch.n_classes)
        assert np.isfinite(got).all()
        np.testing.assert_array_equal(got, want)
        if t < 2 and not (fam == "mbv3" and t == 0):   # (the shrunken MobileNetV3-shaped net's largest SubNet sits at the
            #                                             bf16 storage floor: see the resident-slab test)
            assert rel_l2(got, oracle_logits(arch, wts, cfg, x_np)) <= (1e-2 if bf16 else 1e-4)
    ctx.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import paper_2306_17266_amd as S
    arch = A.small_resnet_arch()
    blob, _ = make_problem(arch, 13, True)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16)
    cfg = A.max_cfg(arch, 96)
    x = torch.zeros(64, 96, 96, 3, device="cuda", dtype=torch.bfloat16)     # 64 images: ~30 MB of activations
    y = torch.full((64, arch.n_classes), float("nan"), device="cuda")
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_infer_static(cfg, x, y)
    assert e.value.code == -2 and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(y).all()                                           # nothing was enqueued
    ctx.close()
