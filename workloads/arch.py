"""Plain-data descriptions of the synthetic SuperNets and of one SubNet choice.

These are inputs only: which family, the base channel counts, the lists of
elastic choices, and (for a SubNet) which choice was picked where.  How a
choice turns into channel counts, layers and weight slices is the method's
business and lives on each side separately (the CPU evaluator and the GPU
library each derive it on their own).

The three families stand in for the paper's workloads (Section 5.1: weight
shared ResNet50 and MobileNetV3 SuperNets) plus a tiny net for fast checks;
only their shapes and sizes are taken, no trained weights exist here.
"""
from dataclasses import dataclass, field
from typing import List

FAMILY_TINY = 0
FAMILY_RESNET = 1
FAMILY_MBV3 = 2

ACT_NONE = 0
ACT_RELU = 1
ACT_HSWISH = 2

MAX_STAGES = 8
MAX_CHOICES = 4
MAX_BLOCKS = 32


@dataclass
class Arch:
    family: int
    n_classes: int
    in_channels: int
    stage_base_out: List[int]          # channels of a stage at width multiplier 1
    stage_stride: List[int]
    stage_max_depth: List[int]
    stage_act: List[int]
    stage_se: List[int]
    depth_drop_choices: List[int]      # a stage may run max_depth - d blocks, d in this list
    width_choices: List[float]         # channel multipliers (per stage and stem)
    expand_choices: List[float]        # per block
    kernel_choices: List[int]          # per block (depthwise kernel size)
    res_choices: List[int]             # input resolutions accepted
    stem_mid: int = 0                  # base channels of the stem convs
    stem_out: int = 0
    head_mid: int = 0                  # MBV3: 1x1 after the last stage
    head_feat: int = 0                 # MBV3: feature-mix FC before the classifier

    @property
    def n_stages(self):
        return len(self.stage_base_out)

    @property
    def n_block_slots(self):
        return sum(self.stage_max_depth)

    def slot(self, stage, j):
        return sum(self.stage_max_depth[:stage]) + j


@dataclass
class SubnetCfg:
    resolution: int
    depth: List[int]                   # active blocks per stage (TINY: depth[0] = active layers)
    width_idx: List[int]               # [0] stem, [1+s] stage s
    expand_idx: List[int]              # per block slot
    kernel_idx: List[int]              # per block slot

    def key(self):
        return (self.resolution, tuple(self.depth), tuple(self.width_idx),
                tuple(self.expand_idx), tuple(self.kernel_idx))


def tiny_arch():
    """Config 1: four conv3x3+ReLU layers, widths {16,24,32}, depth {2,3,4}."""
    return Arch(family=FAMILY_TINY, n_classes=10, in_channels=3,
                stage_base_out=[32, 32, 32, 32], stage_stride=[1, 1, 1, 1],
                stage_max_depth=[1, 1, 1, 1], stage_act=[ACT_RELU] * 4, stage_se=[0] * 4,
                depth_drop_choices=[0, 1, 2], width_choices=[0.5, 0.75, 1.0],
                expand_choices=[1.0], kernel_choices=[3], res_choices=[32])


def resnet_arch():
    """Configs 2 and 4: ResNet50-shaped bottleneck SuperNet."""
    return Arch(family=FAMILY_RESNET, n_classes=1000, in_channels=3,
                stage_base_out=[256, 512, 1024, 2048], stage_stride=[1, 2, 2, 2],
                stage_max_depth=[4, 4, 6, 4], stage_act=[ACT_RELU] * 4, stage_se=[0] * 4,
                depth_drop_choices=[0, 1, 2], width_choices=[0.65, 0.8, 1.0],
                expand_choices=[0.2, 0.25, 0.35], kernel_choices=[3], res_choices=[224],
                stem_mid=32, stem_out=64)


def mbv3_arch():
    """Configs 3 and 5: MobileNetV3-shaped inverted-residual SuperNet."""
    return Arch(family=FAMILY_MBV3, n_classes=1000, in_channels=3,
                stage_base_out=[24, 40, 80, 112, 160], stage_stride=[2, 2, 2, 1, 2],
                stage_max_depth=[4] * 5,
                stage_act=[ACT_RELU, ACT_RELU, ACT_HSWISH, ACT_HSWISH, ACT_HSWISH],
                stage_se=[0, 1, 0, 1, 1],
                depth_drop_choices=[0, 1, 2], width_choices=[1.0],
                expand_choices=[3.0, 4.0, 6.0], kernel_choices=[3, 5, 7],
                res_choices=[160, 192, 224],
                stem_out=16, head_mid=960, head_feat=1280)


def small_resnet_arch():
    """A shrunken bottleneck SuperNet (same structure, 1/8 of the channels, 2 stages fewer
    blocks) that the CPU evaluator finishes in well under a second; for parity cases that
    need many queries."""
    return Arch(family=FAMILY_RESNET, n_classes=40, in_channels=3,
                stage_base_out=[32, 64, 128, 256], stage_stride=[1, 2, 2, 2],
                stage_max_depth=[3, 3, 4, 3], stage_act=[ACT_RELU] * 4, stage_se=[0] * 4,
                depth_drop_choices=[0, 1, 2], width_choices=[0.65, 0.8, 1.0],
                expand_choices=[0.2, 0.25, 0.35], kernel_choices=[3], res_choices=[64, 96],
                stem_mid=16, stem_out=24)


def small_mbv3_arch():
    """A shrunken inverted-residual SuperNet for fast parity cases."""
    return Arch(family=FAMILY_MBV3, n_classes=24, in_channels=3,
                stage_base_out=[16, 24, 40, 48, 64], stage_stride=[2, 2, 2, 1, 2],
                stage_max_depth=[3] * 5,
                stage_act=[ACT_RELU, ACT_RELU, ACT_HSWISH, ACT_HSWISH, ACT_HSWISH],
                stage_se=[0, 1, 0, 1, 1],
                depth_drop_choices=[0, 1], width_choices=[1.0],
                expand_choices=[3.0, 4.0, 6.0], kernel_choices=[3, 5, 7],
                res_choices=[64, 96],
                stem_out=16, head_mid=192, head_feat=256)


def max_cfg(arch, resolution=None):
    nb = arch.n_block_slots
    return SubnetCfg(resolution=resolution or max(arch.res_choices),
                     depth=([arch.n_stages] if arch.family == FAMILY_TINY else list(arch.stage_max_depth)),
                     width_idx=[len(arch.width_choices) - 1] * (arch.n_stages + 1),
                     expand_idx=[len(arch.expand_choices) - 1] * nb,
                     kernel_idx=[len(arch.kernel_choices) - 1] * nb)


def min_cfg(arch, resolution=None):
    nb = arch.n_block_slots
    drop = max(arch.depth_drop_choices)
    return SubnetCfg(resolution=resolution or max(arch.res_choices),
                     depth=([arch.n_stages - drop] if arch.family == FAMILY_TINY
                            else [m - drop for m in arch.stage_max_depth]),
                     width_idx=[0] * (arch.n_stages + 1),
                     expand_idx=[0] * nb, kernel_idx=[0] * nb)
