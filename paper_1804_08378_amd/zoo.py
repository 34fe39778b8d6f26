"""Network architectures for the whole-network measurements (Sections 5.2-5.4 evaluate
torchvision's VGG, ResNet and DenseNet families).

Written here from the architectures' published descriptions, with hand-written `forward`
methods (residual additions as `+`, dense concatenations as `torch.cat`) and random weights:
what matters for the measurements is the layer structure and the tensor shapes, not trained
parameters.  `width` scales every channel count, `classes` the classifier, so that tests can
build small versions of the same structure.
"""
from __future__ import annotations

import torch
import torch.nn.functional as F
from torch import nn

__all__ = ["vgg_bn", "vgg", "resnet", "densenet", "alexnet", "squeezenet", "inception_v3", "randomize_batchnorm"]


def randomize_batchnorm(model: nn.Module, seed: int = 0) -> nn.Module:
    """Non-trivial running statistics and affine parameters for every BatchNorm2d (a freshly
    constructed one is the identity)."""
    g = torch.Generator().manual_seed(seed)
    with torch.no_grad():
        for m in model.modules():
            if isinstance(m, nn.BatchNorm2d):
                c = m.num_features
                m.running_mean.copy_(torch.randn(c, generator=g) * 0.1)
                m.running_var.copy_(torch.rand(c, generator=g) * 0.5 + 0.75)
                m.weight.copy_(torch.rand(c, generator=g) * 0.5 + 0.75)
                m.bias.copy_(torch.randn(c, generator=g) * 0.1)
    return model


# ------------------------------------------------------------------------------- VGG
class VGG(nn.Module):
    """Blocks of 3x3 convolutions, each followed by BatchNorm and ReLU, a 2x2 max pool after
    every block, three fully connected layers."""

    def __init__(self, blocks, width, classes, hidden, batch_norm=True):
        super().__init__()
        layers, cin = [], 3
        for n_conv, c in blocks:
            c = max(1, int(c * width))
            for _ in range(n_conv):
                layers += [nn.Conv2d(cin, c, 3, padding=1)] + ([nn.BatchNorm2d(c)] if batch_norm else []) + \
                          [nn.ReLU(inplace=True)]
                cin = c
            layers.append(nn.MaxPool2d(2, 2))
        self.features = nn.Sequential(*layers)
        self.avgpool = nn.AdaptiveAvgPool2d(7)
        self.classifier = nn.Sequential(nn.Linear(cin * 49, hidden), nn.ReLU(inplace=True), nn.Dropout(),
                                        nn.Linear(hidden, hidden), nn.ReLU(inplace=True), nn.Dropout(),
                                        nn.Linear(hidden, classes))

    def forward(self, x):
        x = self.avgpool(self.features(x))
        return self.classifier(torch.flatten(x, 1))


def vgg_bn(depth: int = 16, width: float = 1.0, classes: int = 1000, batch_norm: bool = True) -> nn.Module:
    convs = {11: (1, 1, 2, 2, 2), 13: (2, 2, 2, 2, 2), 16: (2, 2, 3, 3, 3), 19: (2, 2, 4, 4, 4)}[depth]
    blocks = list(zip(convs, (64, 128, 256, 512, 512)))
    return VGG(blocks, width, classes, max(8, int(4096 * width)), batch_norm)


def vgg(depth: int = 16, width: float = 1.0, classes: int = 1000) -> nn.Module:
    """The same networks without BatchNorm."""
    return vgg_bn(depth, width, classes, batch_norm=False)


# --------------------------------------------------------------------------- AlexNet
class AlexNet(nn.Module):
    """Five convolutions (11x11/4, 5x5, three 3x3) with ReLU, 3x3/2 max pools after the first,
    second and fifth, three fully connected layers with Dropout."""

    def __init__(self, width, classes):
        super().__init__()
        c = [max(1, int(v * width)) for v in (64, 192, 384, 256, 256)]
        self.features = nn.Sequential(
            nn.Conv2d(3, c[0], 11, 4, 2), nn.ReLU(inplace=True), nn.MaxPool2d(3, 2),
            nn.Conv2d(c[0], c[1], 5, padding=2), nn.ReLU(inplace=True), nn.MaxPool2d(3, 2),
            nn.Conv2d(c[1], c[2], 3, padding=1), nn.ReLU(inplace=True),
            nn.Conv2d(c[2], c[3], 3, padding=1), nn.ReLU(inplace=True),
            nn.Conv2d(c[3], c[4], 3, padding=1), nn.ReLU(inplace=True), nn.MaxPool2d(3, 2))
        self.avgpool = nn.AdaptiveAvgPool2d(6)
        hidden = max(8, int(4096 * width))
        self.classifier = nn.Sequential(nn.Dropout(), nn.Linear(c[4] * 36, hidden), nn.ReLU(inplace=True),
                                        nn.Dropout(), nn.Linear(hidden, hidden), nn.ReLU(inplace=True),
                                        nn.Linear(hidden, classes))

    def forward(self, x):
        x = self.avgpool(self.features(x))
        return self.classifier(torch.flatten(x, 1))


def alexnet(width: float = 1.0, classes: int = 1000) -> nn.Module:
    return AlexNet(width, classes)


# ------------------------------------------------------------------------ SqueezeNet
class Fire(nn.Module):
    """1x1 "squeeze" convolution, then a 1x1 and a 3x3 "expand" convolution side by side, each
    followed by ReLU; the two expand results are concatenated."""

    def __init__(self, cin, squeeze, expand):
        super().__init__()
        self.squeeze = nn.Conv2d(cin, squeeze, 1)
        self.expand1 = nn.Conv2d(squeeze, expand, 1)
        self.expand3 = nn.Conv2d(squeeze, expand, 3, padding=1)

    def forward(self, x):
        x = F.relu(self.squeeze(x))
        return torch.cat([F.relu(self.expand1(x)), F.relu(self.expand3(x))], 1)


class SqueezeNet(nn.Module):
    def __init__(self, version, width, classes):
        super().__init__()
        w = lambda v: max(1, int(v * width))
        fire = lambda cin, s, e: Fire(w(cin), w(s), w(e))
        pool = lambda: nn.MaxPool2d(3, 2, ceil_mode=True)
        if version == "1.0":
            self.features = nn.Sequential(
                nn.Conv2d(3, w(96), 7, 2), nn.ReLU(inplace=True), pool(),
                fire(96, 16, 64), fire(128, 16, 64), fire(128, 32, 128), pool(),
                fire(256, 32, 128), fire(256, 48, 192), fire(384, 48, 192), fire(384, 64, 256), pool(),
                fire(512, 64, 256))
        else:
            self.features = nn.Sequential(
                nn.Conv2d(3, w(64), 3, 2), nn.ReLU(inplace=True), pool(),
                fire(64, 16, 64), fire(128, 16, 64), pool(),
                fire(128, 32, 128), fire(256, 32, 128), pool(),
                fire(256, 48, 192), fire(384, 48, 192), fire(384, 64, 256), fire(512, 64, 256))
        self.classifier = nn.Sequential(nn.Dropout(), nn.Conv2d(w(512), classes, 1), nn.ReLU(inplace=True),
                                        nn.AdaptiveAvgPool2d(1))

    def forward(self, x):
        return torch.flatten(self.classifier(self.features(x)), 1)


def squeezenet(version: str = "1.0", width: float = 1.0, classes: int = 1000) -> nn.Module:
    return SqueezeNet(version, width, classes)


# ---------------------------------------------------------------------------- ResNet
class BasicBlock(nn.Module):
    expansion = 1

    def __init__(self, cin, c, stride):
        super().__init__()
        self.conv1 = nn.Conv2d(cin, c, 3, stride, 1, bias=False)
        self.bn1 = nn.BatchNorm2d(c)
        self.conv2 = nn.Conv2d(c, c, 3, 1, 1, bias=False)
        self.bn2 = nn.BatchNorm2d(c)
        self.down = None
        if stride != 1 or cin != c:
            self.down = nn.Sequential(nn.Conv2d(cin, c, 1, stride, bias=False), nn.BatchNorm2d(c))

    def forward(self, x):
        out = F.relu(self.bn1(self.conv1(x)))
        out = self.bn2(self.conv2(out))
        return F.relu(out + (x if self.down is None else self.down(x)))


class Bottleneck(nn.Module):
    expansion = 4

    def __init__(self, cin, c, stride):
        super().__init__()
        self.conv1 = nn.Conv2d(cin, c, 1, bias=False)
        self.bn1 = nn.BatchNorm2d(c)
        self.conv2 = nn.Conv2d(c, c, 3, stride, 1, bias=False)
        self.bn2 = nn.BatchNorm2d(c)
        self.conv3 = nn.Conv2d(c, 4 * c, 1, bias=False)
        self.bn3 = nn.BatchNorm2d(4 * c)
        self.down = None
        if stride != 1 or cin != 4 * c:
            self.down = nn.Sequential(nn.Conv2d(cin, 4 * c, 1, stride, bias=False), nn.BatchNorm2d(4 * c))

    def forward(self, x):
        out = F.relu(self.bn1(self.conv1(x)))
        out = F.relu(self.bn2(self.conv2(out)))
        out = self.bn3(self.conv3(out))
        out += x if self.down is None else self.down(x)
        return F.relu(out)


class ResNet(nn.Module):
    """7x7/2 convolution, BatchNorm, ReLU, 3x3/2 max pool, four stages of residual blocks,
    global average pool, one fully connected layer."""

    def __init__(self, block, counts, width, classes):
        super().__init__()
        c0 = max(1, int(64 * width))
        self.conv = nn.Conv2d(3, c0, 7, 2, 3, bias=False)
        self.bn = nn.BatchNorm2d(c0)
        self.pool = nn.MaxPool2d(3, 2, 1)
        blocks, cin = [], c0
        for stage, n in enumerate(counts):
            c = c0 * 2 ** stage
            for i in range(n):
                blocks.append(block(cin, c, 2 if (i == 0 and stage > 0) else 1))
                cin = c * block.expansion
        self.blocks = nn.Sequential(*blocks)
        self.fc = nn.Linear(cin, classes)

    def forward(self, x):
        x = self.blocks(self.pool(F.relu(self.bn(self.conv(x)))))
        return self.fc(torch.flatten(F.adaptive_avg_pool2d(x, 1), 1))


def resnet(depth: int = 18, width: float = 1.0, classes: int = 1000) -> nn.Module:
    block, counts = {18: (BasicBlock, (2, 2, 2, 2)), 34: (BasicBlock, (3, 4, 6, 3)), 50: (Bottleneck, (3, 4, 6, 3)),
                     101: (Bottleneck, (3, 4, 23, 3)), 152: (Bottleneck, (3, 8, 36, 3))}[depth]
    return ResNet(block, counts, width, classes)


# -------------------------------------------------------------------------- DenseNet
class DenseLayer(nn.Module):
    """BatchNorm, ReLU, 1x1 convolution to 4 * growth channels, BatchNorm, ReLU, 3x3 convolution
    to `growth` channels, on the concatenation of everything the block has produced so far."""

    def __init__(self, cin, growth):
        super().__init__()
        self.norm1 = nn.BatchNorm2d(cin)
        self.conv1 = nn.Conv2d(cin, 4 * growth, 1, bias=False)
        self.norm2 = nn.BatchNorm2d(4 * growth)
        self.conv2 = nn.Conv2d(4 * growth, growth, 3, padding=1, bias=False)

    def forward(self, feats):
        x = self.conv1(F.relu(self.norm1(torch.cat(feats, 1))))
        return self.conv2(F.relu(self.norm2(x)))


class DenseNet(nn.Module):
    def __init__(self, growth, counts, c0, classes):
        super().__init__()
        self.conv0 = nn.Conv2d(3, c0, 7, 2, 3, bias=False)
        self.norm0 = nn.BatchNorm2d(c0)
        self.pool0 = nn.MaxPool2d(3, 2, 1)
        self.blocks = nn.ModuleList()
        self.trans_norm, self.trans_conv = nn.ModuleList(), nn.ModuleList()
        c = c0
        for b, n in enumerate(counts):
            self.blocks.append(nn.ModuleList([DenseLayer(c + i * growth, growth) for i in range(n)]))
            c += n * growth
            if b + 1 < len(counts):
                self.trans_norm.append(nn.BatchNorm2d(c))
                self.trans_conv.append(nn.Conv2d(c, c // 2, 1, bias=False))
                c //= 2
        self.norm5 = nn.BatchNorm2d(c)
        self.fc = nn.Linear(c, classes)

    def forward(self, x):
        x = self.pool0(F.relu(self.norm0(self.conv0(x))))
        for b, block in enumerate(self.blocks):
            feats = [x]
            for layer in block:
                feats.append(layer(feats))
            x = torch.cat(feats, 1)
            if b < len(self.trans_norm):
                x = F.avg_pool2d(self.trans_conv[b](F.relu(self.trans_norm[b](x))), 2, 2)
        x = F.adaptive_avg_pool2d(F.relu(self.norm5(x)), 1)
        return self.fc(torch.flatten(x, 1))


def densenet(depth: int = 121, width: float = 1.0, classes: int = 1000) -> nn.Module:
    growth, counts, c0 = {121: (32, (6, 12, 24, 16), 64), 169: (32, (6, 12, 32, 32), 64),
                          201: (32, (6, 12, 48, 32), 64), 161: (48, (6, 12, 36, 24), 96)}[depth]
    return DenseNet(max(1, int(growth * width)), counts, max(2, int(c0 * width)), classes)


# ---------------------------------------------------------------------- Inception v3
class ConvBN(nn.Module):
    """Convolution without bias, BatchNorm (eps 0.001), ReLU: the unit every branch is made of."""

    def __init__(self, cin, cout, k, stride=1, padding=0):
        super().__init__()
        self.conv = nn.Conv2d(cin, cout, k, stride, padding, bias=False)
        self.bn = nn.BatchNorm2d(cout, eps=0.001)

    def forward(self, x):
        return F.relu(self.bn(self.conv(x)))


class InceptionA(nn.Module):  # 35 x 35 grid
    def __init__(self, cin, pool_features, w):
        super().__init__()
        self.b1 = ConvBN(cin, w(64), 1)
        self.b5 = nn.Sequential(ConvBN(cin, w(48), 1), ConvBN(w(48), w(64), 5, padding=2))
        self.b3 = nn.Sequential(ConvBN(cin, w(64), 1), ConvBN(w(64), w(96), 3, padding=1), ConvBN(w(96), w(96), 3, padding=1))
        self.bp = ConvBN(cin, w(pool_features), 1)

    def forward(self, x):
        return torch.cat([self.b1(x), self.b5(x), self.b3(x), self.bp(F.avg_pool2d(x, 3, 1, 1))], 1)


class InceptionB(nn.Module):  # 35 -> 17
    def __init__(self, cin, w):
        super().__init__()
        self.b3 = ConvBN(cin, w(384), 3, 2)
        self.bd = nn.Sequential(ConvBN(cin, w(64), 1), ConvBN(w(64), w(96), 3, padding=1), ConvBN(w(96), w(96), 3, 2))

    def forward(self, x):
        return torch.cat([self.b3(x), self.bd(x), F.max_pool2d(x, 3, 2)], 1)


class InceptionC(nn.Module):  # 17 x 17 grid, factorised 7 x 7 convolutions
    def __init__(self, cin, c7, w):
        super().__init__()
        c7 = w(c7)
        self.b1 = ConvBN(cin, w(192), 1)
        self.b7 = nn.Sequential(ConvBN(cin, c7, 1), ConvBN(c7, c7, (1, 7), padding=(0, 3)),
                                ConvBN(c7, w(192), (7, 1), padding=(3, 0)))
        self.bd = nn.Sequential(ConvBN(cin, c7, 1), ConvBN(c7, c7, (7, 1), padding=(3, 0)),
                                ConvBN(c7, c7, (1, 7), padding=(0, 3)), ConvBN(c7, c7, (7, 1), padding=(3, 0)),
                                ConvBN(c7, w(192), (1, 7), padding=(0, 3)))
        self.bp = ConvBN(cin, w(192), 1)

    def forward(self, x):
        return torch.cat([self.b1(x), self.b7(x), self.bd(x), self.bp(F.avg_pool2d(x, 3, 1, 1))], 1)


class InceptionD(nn.Module):  # 17 -> 8
    def __init__(self, cin, w):
        super().__init__()
        self.b3 = nn.Sequential(ConvBN(cin, w(192), 1), ConvBN(w(192), w(320), 3, 2))
        self.b7 = nn.Sequential(ConvBN(cin, w(192), 1), ConvBN(w(192), w(192), (1, 7), padding=(0, 3)),
                                ConvBN(w(192), w(192), (7, 1), padding=(3, 0)), ConvBN(w(192), w(192), 3, 2))

    def forward(self, x):
        return torch.cat([self.b3(x), self.b7(x), F.max_pool2d(x, 3, 2)], 1)


class InceptionE(nn.Module):  # 8 x 8 grid, branches that split once more
    def __init__(self, cin, w):
        super().__init__()
        self.b1 = ConvBN(cin, w(320), 1)
        self.b3 = ConvBN(cin, w(384), 1)
        self.b3a = ConvBN(w(384), w(384), (1, 3), padding=(0, 1))
        self.b3b = ConvBN(w(384), w(384), (3, 1), padding=(1, 0))
        self.bd = nn.Sequential(ConvBN(cin, w(448), 1), ConvBN(w(448), w(384), 3, padding=1))
        self.bda = ConvBN(w(384), w(384), (1, 3), padding=(0, 1))
        self.bdb = ConvBN(w(384), w(384), (3, 1), padding=(1, 0))
        self.bp = ConvBN(cin, w(192), 1)

    def forward(self, x):
        b3 = self.b3(x)
        bd = self.bd(x)
        return torch.cat([self.b1(x), torch.cat([self.b3a(b3), self.b3b(b3)], 1),
                          torch.cat([self.bda(bd), self.bdb(bd)], 1), self.bp(F.avg_pool2d(x, 3, 1, 1))], 1)


class InceptionV3(nn.Module):
    """299 x 299 input; five convolutions and two 3x3/2 max pools, three A, one B, four C, one D
    and two E modules, global average pool, Dropout, one fully connected layer (no auxiliary
    classifier)."""

    def __init__(self, width, classes):
        super().__init__()
        w = lambda v: max(1, int(v * width))
        self.stem1 = nn.Sequential(ConvBN(3, w(32), 3, 2), ConvBN(w(32), w(32), 3), ConvBN(w(32), w(64), 3, padding=1))
        self.stem2 = nn.Sequential(ConvBN(w(64), w(80), 1), ConvBN(w(80), w(192), 3))
        a1, a2, a3 = w(64) + w(64) + w(96) + w(32), w(64) + w(64) + w(96) + w(64), w(64) + w(64) + w(96) + w(64)
        b = w(384) + w(96) + a3
        d = w(320) + w(192) + 4 * w(192)
        e = w(320) + 4 * w(384) + w(192)
        self.mixed = nn.Sequential(
            InceptionA(w(192), 32, w), InceptionA(a1, 64, w), InceptionA(a2, 64, w), InceptionB(a3, w),
            InceptionC(b, 128, w), InceptionC(4 * w(192), 160, w), InceptionC(4 * w(192), 160, w),
            InceptionC(4 * w(192), 192, w), InceptionD(4 * w(192), w), InceptionE(d, w), InceptionE(e, w))
        self.dropout = nn.Dropout()
        self.fc = nn.Linear(e, classes)

    def forward(self, x):
        x = F.max_pool2d(self.stem1(x), 3, 2)
        x = F.max_pool2d(self.stem2(x), 3, 2)
        x = self.dropout(F.adaptive_avg_pool2d(self.mixed(x), 1))
        return self.fc(torch.flatten(x, 1))


def inception_v3(width: float = 1.0, classes: int = 1000) -> nn.Module:
    return InceptionV3(width, classes)
