"""Workload descriptions: the five benchmark configurations plus small test flows.

A FlowConfig fixes the image shape, the flow's macro structure (levels, couplings
per level, factor-out, prior heads) and the family of the coupling network t().
Nothing here computes anything; it is the shape vocabulary shared by the input
generators, the tests and the benchmark.
"""
from dataclasses import dataclass, replace

PLAIN, RESNET, DENSE = 0, 1, 2
FAMILY_NAMES = {PLAIN: "plain", RESNET: "resnet", DENSE: "dense"}


@dataclass(frozen=True)
class FlowConfig:
    name: str
    H: int
    W: int
    batch: int
    levels: int
    couplings: int          # per level
    family: int
    width: int
    depth: int              # residual blocks (resnet) / dense layers (dense); 0 for plain
    heads: bool             # prior-parameter heads at every factor-out
    keep: float = 1.0       # fraction of filters kept by the binary gates
    image_kind: str = "filtered"   # "filtered" | "uniform"
    seed_id: int = 0
    block_k2: int = 1       # resnet family: kernel of a block's second conv (the paper's own blocks use 3)
    keep_levels: tuple = () # per-level keep fractions (level 1 first); empty = `keep` everywhere
    act_unsigned: bool = False   # post-ReLU activations are unsigned 8-bit codes 0..255 (the paper's own format)

    def keep_at(self, level):
        return self.keep_levels[level - 1] if self.keep_levels else self.keep

    def level_channels(self, level):
        """Channels of the flow state at 1-based `level` (after its squeeze)."""
        return 12 * (2 ** (level - 1))

    def level_hw(self, level):
        return self.H >> level, self.W >> level

    def z_chunk_channels(self, level):
        c = self.level_channels(level)
        return c if level == self.levels else c // 2

    @property
    def d(self):
        return 3 * self.H * self.W

    @property
    def d_codes(self):
        if not self.heads:
            return 0
        n = 0
        for lv in range(1, self.levels):
            h, w = self.level_hw(lv)
            n += 2 * self.z_chunk_channels(lv) * h * w
        return n

    def with_batch(self, b):
        return replace(self, batch=b)


def net_layers(family, c_in, c_out, width, depth, k2=1):
    """Layer list of one network: tuples (C_out, C_in, k, relu, shortcut, gated).

    plain : conv3x3 -> ReLU -> conv3x3
    resnet: conv_in, depth x [conv3x3 ReLU, conv k2 x k2 + shortcut ReLU], conv_out
    dense : conv_in, depth x [conv1x1 over all features so far, conv3x3], conv_out
            over the concatenation of all features
    Only convolutions that produce hidden features carry gates.
    """
    L = []
    if family == PLAIN:
        L.append((width, c_in, 3, True, False, True))
        L.append((c_out, width, 3, False, False, False))
    elif family == RESNET:
        L.append((width, c_in, 3, True, False, True))
        for _ in range(depth):
            L.append((width, width, 3, True, False, True))
            L.append((width, width, k2, True, True, True))
        L.append((c_out, width, 3, False, False, False))
    elif family == DENSE:
        L.append((width, c_in, 3, True, False, True))
        for l in range(1, depth + 1):
            L.append((width, l * width, 1, True, False, True))
            L.append((width, width, 3, True, False, True))
        L.append((c_out, (depth + 1) * width, 3, False, False, False))
    else:
        raise ValueError("unknown family %r" % (family,))
    return L


def flow_networks(cfg):
    """Networks of a flow in blob order: (kind, level, C_level, C_in, C_out).

    kind 0 = coupling network t(), kind 1 = prior head. Level l holds its K
    couplings, then its head when the level factors out and heads are on.
    """
    nets = []
    for lv in range(1, cfg.levels + 1):
        c = cfg.level_channels(lv)
        for _ in range(cfg.couplings):
            nets.append((0, lv, c, c // 2, c - c // 2))
        if cfg.heads and lv < cfg.levels:
            nets.append((1, lv, c, c // 2, 2 * (c - c // 2)))
    return nets


def macs_per_image(cfg, with_heads=True, kept_only=True):
    """Multiply-accumulates of one forward pass for one image, at true channel counts."""
    total = 0
    for kind, lv, c, c_in, c_out in flow_networks(cfg):
        if kind == 1 and not with_heads:
            continue
        h, w = cfg.level_hw(lv)
        wk = max(1, int(round(cfg.width * cfg.keep_at(lv)))) if kept_only and cfg.keep_at(lv) < 1.0 else cfg.width
        for i, (co, ci, k, relu, sc, gated) in enumerate(
                net_layers(cfg.family, c_in, c_out, cfg.width, cfg.depth, cfg.block_k2)):
            co_k = wk if gated else co
            ci_k = ci if i == 0 else (ci // cfg.width) * wk
            total += co_k * ci_k * k * k * h * w
    return total


CONFIGS = {
    # 1: tiny flow the oracle finishes instantly
    "cfg1": FlowConfig("cfg1", 8, 8, 1, 1, 2, PLAIN, 32, 0, False, image_kind="uniform", seed_id=1),
    # 2: 32x32, residual t() at width 128
    "cfg2": FlowConfig("cfg2", 32, 32, 64, 2, 4, RESNET, 128, 2, False, seed_id=2),
    # 3: ImageNet32-shaped, dense t() at width 512, prior heads
    "cfg3": FlowConfig("cfg3", 32, 32, 256, 3, 8, DENSE, 512, 8, True, seed_id=3),
    # 4: ImageNet64-shaped (the headline workload)
    "cfg4": FlowConfig("cfg4", 64, 64, 128, 4, 8, DENSE, 512, 8, True, seed_id=4),
    # 5: as 4 with half of the filters of every hidden conv gated off
    "cfg5": FlowConfig("cfg5", 64, 64, 1024, 4, 8, DENSE, 512, 8, True, keep=0.5, seed_id=5),
    # gated residual flow: exercises the scatter-add shortcut
    "cfg2g": FlowConfig("cfg2g", 32, 32, 4, 2, 4, RESNET, 128, 2, False, keep=0.5, seed_id=6),
    # small stand-ins with the same structure, for element-by-element parity
    "mini_dense": FlowConfig("mini_dense", 16, 16, 5, 2, 2, DENSE, 64, 3, True, seed_id=7),
    "mini_dense_g": FlowConfig("mini_dense_g", 16, 16, 3, 2, 2, DENSE, 64, 3, True, keep=0.5, seed_id=8),
    "mini_resnet": FlowConfig("mini_resnet", 16, 16, 3, 2, 2, RESNET, 32, 2, False, seed_id=9),
    "mini_resnet_g": FlowConfig("mini_resnet_g", 16, 16, 3, 2, 2, RESNET, 32, 2, False, keep=0.5, seed_id=10),
    "mid_dense": FlowConfig("mid_dense", 32, 32, 3, 3, 2, DENSE, 256, 4, True, seed_id=11),
    "odd_dense_g": FlowConfig("odd_dense_g", 16, 16, 2, 2, 2, DENSE, 72, 2, True, keep=0.625, seed_id=12),
    # image sides that are not powers of two and not square (levels 12x20 and 6x10); depth 3 gives the last
    # layer 256 input channels, the width from which the library tap-expands it
    "rect_dense": FlowConfig("rect_dense", 24, 40, 3, 2, 2, DENSE, 64, 3, True, seed_id=13),
    "rect_resnet_g": FlowConfig("rect_resnet_g", 24, 40, 2, 2, 2, RESNET, 32, 2, False, keep=0.5, seed_id=14),
    # six levels down to 1x1 maps: level 6 has 192 input channels per coupling network (whole 64-channel
    # planes, the first layer stays a 3x3 one) and single-pixel images
    "deep6": FlowConfig("deep6", 64, 64, 2, 6, 1, PLAIN, 32, 0, True, seed_id=22),
    # The paper's own coupling network (App. B.1): conv_in, 8 residual blocks of two 3x3 convolutions at
    # 128 channels, conv_out; L = 3 levels for 32x32 images, 4 for 64x64, 8 couplings per level; the pruned
    # variant keeps fewer filters the deeper the level (Sec. 5.1, the pruning figure).
    "paper_res32": FlowConfig("paper_res32", 32, 32, 512, 3, 8, RESNET, 128, 8, True, seed_id=15, block_k2=3),
    "paper_res64": FlowConfig("paper_res64", 64, 64, 256, 4, 8, RESNET, 128, 8, True, seed_id=16, block_k2=3),
    "paper_iodf64": FlowConfig("paper_iodf64", 64, 64, 256, 4, 8, RESNET, 128, 8, True, seed_id=17, block_k2=3,
                               keep=0.5, keep_levels=(0.75, 0.625, 0.375, 0.25)),
    # unsigned post-ReLU activations (Eq. 3): the three families, a gated one, and the paper's network
    "mini_dense_u": FlowConfig("mini_dense_u", 16, 16, 5, 2, 2, DENSE, 64, 3, True, seed_id=19, act_unsigned=True),
    "mini_resnet_gu": FlowConfig("mini_resnet_gu", 16, 16, 3, 2, 2, RESNET, 32, 2, True, keep=0.5, seed_id=20,
                                 act_unsigned=True),
    "cfg1_u": FlowConfig("cfg1_u", 8, 8, 1, 1, 2, PLAIN, 32, 0, False, image_kind="uniform", seed_id=21,
                         act_unsigned=True),
    "paper_iodf64_u": FlowConfig("paper_iodf64_u", 64, 64, 256, 4, 8, RESNET, 128, 8, True, seed_id=17, block_k2=3,
                                 keep=0.5, keep_levels=(0.75, 0.625, 0.375, 0.25), act_unsigned=True),
    # residual networks 256 wide over many pixels (800 tiles of 256x256 at level 1): shortcut layers of full
    # tile width with several tiles per CU, in both activation formats
    "wide_resnet": FlowConfig("wide_resnet", 64, 64, 200, 2, 2, RESNET, 256, 2, True, seed_id=23, block_k2=3),
    "wide_resnet_u": FlowConfig("wide_resnet_u", 64, 64, 200, 2, 2, RESNET, 256, 2, True, seed_id=24, block_k2=3,
                                act_unsigned=True),
    "mini_paper_g": FlowConfig("mini_paper_g", 16, 16, 3, 2, 2, RESNET, 32, 3, True, seed_id=18, block_k2=3,
                               keep=0.5, keep_levels=(0.75, 0.375)),
}
