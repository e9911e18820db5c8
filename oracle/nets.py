"""Op lists of the networks the oracle trains (TEST INFRASTRUCTURE, not the product).

Each op is a row (type, in0, in1, out, k, stride, pad, cout, bias); op i writes
tensor i+1 and tensor 0 is the input batch.  The paper (Sec. 4.1) trains
ResNet-18 and VGG-16 on 32x32 colour images; the two smaller nets are the
small-scale workloads.  Layer shapes are the published ones of those
architectures in their 32x32-input form.
"""
import numpy as np

CONV, DENSE, RELU, MAXPOOL, BN, ADD, GAP = range(7)


class _Builder:
    def __init__(self):
        self.ops = []

    def _push(self, typ, in0, in1=-1, k=0, stride=0, pad=0, cout=0, bias=0):
        out = len(self.ops) + 1
        self.ops.append((typ, in0, in1, out, k, stride, pad, cout, bias))
        return out

    def conv(self, x, cout, k=3, stride=1, pad=1, bias=True):
        return self._push(CONV, x, k=k, stride=stride, pad=pad, cout=cout, bias=int(bias))

    def dense(self, x, cout, bias=True):
        return self._push(DENSE, x, cout=cout, bias=int(bias))

    def relu(self, x):
        return self._push(RELU, x)

    def maxpool(self, x):
        return self._push(MAXPOOL, x)

    def bn(self, x):
        return self._push(BN, x)

    def add(self, x, y):
        return self._push(ADD, x, in1=y)

    def gap(self, x):
        return self._push(GAP, x)

    def array(self):
        return np.asarray(self.ops, dtype=np.int32).reshape(-1, 9)


def mlp(hidden=128, n_classes=10):
    """784-128-10 perceptron: dense, ReLU, dense."""
    b = _Builder()
    t = b.relu(b.dense(0, hidden))
    b.dense(t, n_classes)
    return b.array()


def cnn2(n_classes=10):
    """conv3x3(3->32) ReLU pool conv3x3(32->64) ReLU pool FC(4096->10); padding 1 keeps 32x32 -> 8x8x64 = 4096."""
    b = _Builder()
    t = b.maxpool(b.relu(b.conv(0, 32)))
    t = b.maxpool(b.relu(b.conv(t, 64)))
    b.dense(t, n_classes)
    return b.array()


def resnet18(n_classes=10):
    """ResNet-18 for 32x32 inputs: 3x3 stem of 64, four stages of two basic blocks (64,128,256,512;
    strides 1,2,2,2), 1x1 stride-2 projection on the three down-sampling blocks, BN after every
    convolution (no conv bias), global average pool, FC 512->10."""
    b = _Builder()
    t = b.relu(b.bn(b.conv(0, 64, bias=False)))
    cin = 64
    for cout, stride in ((64, 1), (128, 2), (256, 2), (512, 2)):
        for blk in range(2):
            s = stride if blk == 0 else 1
            u = b.relu(b.bn(b.conv(t, cout, stride=s, bias=False)))
            u = b.bn(b.conv(u, cout, bias=False))
            if s != 1 or cin != cout:
                sc = b.bn(b.conv(t, cout, k=1, stride=s, pad=0, bias=False))
            else:
                sc = t
            t = b.relu(b.add(u, sc))
            cin = cout
    b.dense(b.gap(t), n_classes)
    return b.array()


def vgg16(n_classes=10):
    """VGG-16 for 32x32 inputs: 13 conv3x3 (with bias) each followed by BN and ReLU, max-pool after
    each of the five groups, FC 512->10."""
    b = _Builder()
    t = 0
    for width, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(reps):
            t = b.relu(b.bn(b.conv(t, width)))
        t = b.maxpool(t)
    b.dense(t, n_classes)
    return b.array()


NETS = {"mlp": (mlp, (1, 1, 784)), "cnn2": (cnn2, (32, 32, 3)),
        "resnet18": (resnet18, (32, 32, 3)), "vgg16": (vgg16, (32, 32, 3))}
