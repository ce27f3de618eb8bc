"""The five benchmark configurations as plain data: which SuperNet, batch size, query stream,
window Q and SubGraph budget.  Shared by bench.py and the tests so that both run the same streams;
nothing here computes anything of the method (SubNet slices, vectors and SubGraph candidates are
derived by each side with its own encoder).

  tiny_uniform        config 1  Tiny SuperNet, fp32, 8 uniformly random SubNets
  resnet_bs1_sticky   config 2  ResNet50-shaped, batch 1, 1000 queries, next SubNet repeats with p = 0.8
  mbv3_bs1_zipf       config 3  MobileNetV3-shaped, batch 1, 1000 queries, Zipf(1.2) over a pool of 32
  resnet_bs16_levels  config 4  ResNet50-shaped, batch 16, 2000 queries, a latency target drawn from 5
                                levels per query picks the SubNet (Algorithm 1, STRICT_LATENCY), 64 MiB
  mbv3_bs1_regimes    config 5  MobileNetV3-shaped, batch 1, 10000 queries, resolution drawn per query
                                from {160, 192, 224}, Zipf popularity re-drawn every 500 queries;
                                budgets 4 / 32 / 256 MiB
"""
from . import arch as A
from . import streams

NAMES = ["resnet_bs1_sticky", "mbv3_bs1_zipf", "resnet_bs16_levels", "mbv3_bs1_regimes", "tiny_uniform"]


def build(name, budget_mib=None):
    """dict(arch, batch, bf16, cfgs or (pool, levels), Q, budget, policy, desc)."""
    if name == "tiny_uniform":
        arch = A.tiny_arch()
        return dict(name=name, arch=arch, batch=1, bf16=False, cfgs=streams.stream_uniform(arch, 8, 1), Q=4,
                    budget=(budget_mib or 1) << 20,
                    desc="Tiny SuperNet, fp32, batch 1, 32x32, 8 uniformly random SubNets")
    if name == "resnet_bs1_sticky":
        arch = A.resnet_arch()
        b = budget_mib or 16
        return dict(name=name, arch=arch, batch=1, bf16=True, cfgs=streams.stream_sticky(arch, 1000, 2, 0.8, 224),
                    Q=8, budget=b << 20,
                    desc="ResNet50-shaped SuperNet, bf16, batch 1, 224x224, 1000-query stream, next SubNet repeats "
                         "with p=0.8 else uniform, cache re-chosen every 8 queries, budget %d MiB" % b)
    if name == "mbv3_bs1_zipf":
        arch = A.mbv3_arch()
        pool = streams.subnet_pool(arch, 32, 3, 224)
        cfgs = [pool[i] for i, _ in streams.stream_zipf(32, 1000, 3, 1.2)]
        b = budget_mib or 4
        return dict(name=name, arch=arch, batch=1, bf16=True, cfgs=cfgs, Q=10, budget=b << 20,
                    desc="MobileNetV3-shaped SuperNet, bf16, batch 1, 224x224, 1000-query stream, Zipf(1.2) over a "
                         "pool of 32 SubNets, cache re-chosen every 10 queries, budget %d MiB" % b)
    if name == "resnet_bs16_levels":
        arch = A.resnet_arch()
        pool = streams.subnet_pool(arch, 16, 4, 224)
        b = budget_mib or 64
        return dict(name=name, arch=arch, batch=16, bf16=True, cfgs=None, pool=pool,
                    levels=streams.stream_levels(5, 2000, 4), n_levels=5, Q=8, budget=b << 20,
                    desc="ResNet50-shaped SuperNet, bf16, batch 16, 224x224, 2000-query stream, SubNet chosen per "
                         "query by Algorithm 1 (strict latency) for a latency target drawn from 5 levels, serving "
                         "pool of 16 SubNets, budget %d MiB" % b)
    if name == "mbv3_bs1_regimes":
        arch = A.mbv3_arch()
        pool = streams.subnet_pool(arch, 32, 3, 224)
        picks = streams.stream_zipf(32, 10000, 5, 1.2, regime=500, resolutions=[160, 192, 224])
        cfgs = [streams.with_resolution(pool[i], r) for i, r in picks]
        b = budget_mib or 4
        return dict(name=name, arch=arch, batch=1, bf16=True, cfgs=cfgs, Q=10, budget=b << 20,
                    desc="MobileNetV3-shaped SuperNet, bf16, batch 1, resolution per query from {160,192,224}, "
                         "10000-query stream, Zipf(1.2) popularity re-drawn every 500 queries, cache re-chosen "
                         "every 10 queries, budget %d MiB" % b)
    raise ValueError("unknown workload %r" % (name,))
