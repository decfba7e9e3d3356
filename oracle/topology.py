"""ResNet-18/50/152 as flat operator lists, for the CPU oracle (test infrastructure).

The paper names its models only by family ("resnet18", "resnet50", "resnet152",
Table 1) and gives their weight sizes; it does not spell the layers out.  The
operator lists here are the standard post-activation ResNets with every
BatchNorm folded into the preceding convolution (weights plus one bias vector):

* stem: 7x7 stride-2 pad-3 conv 3->64 + ReLU, 3x3 stride-2 pad-1 max pool;
* ResNet-18: BasicBlock (3x3, 3x3) x [2,2,2,2], widths 64/128/256/512;
* ResNet-50/152: Bottleneck (1x1 w, 3x3 w, 1x1 4w) x [3,4,6,3] / [3,8,36,3],
  the stride of a down-sampling block sits on its 3x3 convolution;
* a block's last conv adds the shortcut (block input, or a 1x1 stride-s
  projection of it, without ReLU, when shape changes) and then applies ReLU;
* global average pool, fully connected layer to 1000 classes, softmax.

Written independently of the HIP library's own topology builder; a test checks
that the two lists are identical field by field.
"""
from collections import namedtuple

CONV, MAXPOOL, GAVGPOOL, FC, SOFTMAX = 0, 1, 2, 3, 4

Op = namedtuple("Op", "op cin cout kh kw stride pad relu residual_from input_from")

_CFG = {
    18: ("basic", [2, 2, 2, 2]),
    50: ("bottleneck", [3, 4, 6, 3]),
    152: ("bottleneck", [3, 8, 36, 3]),
}
_WIDTHS = [64, 128, 256, 512]


def resnet(depth, num_classes=1000):
    """Operator list of a ResNet; op i reads the output of op ``input_from``
    (-1 = the network input) and, if ``residual_from`` >= 0, adds that op's
    output before its ReLU."""
    kind, blocks = _CFG[depth]
    ops = []

    def conv(cin, cout, k, stride, pad, relu, src, res=-1):
        ops.append(Op(CONV, cin, cout, k, k, stride, pad, int(relu), res, src))
        return len(ops) - 1

    cur = conv(3, 64, 7, 2, 3, True, -1)
    ops.append(Op(MAXPOOL, 64, 64, 3, 3, 2, 1, 0, -1, cur))
    cur = len(ops) - 1
    cin = 64
    for stage, (w, nblk) in enumerate(zip(_WIDTHS, blocks)):
        for b in range(nblk):
            stride = 2 if (b == 0 and stage > 0) else 1
            cout = w if kind == "basic" else 4 * w
            block_in = cur
            if kind == "basic":
                t = conv(cin, w, 3, stride, 1, True, block_in)
            else:
                t = conv(cin, w, 1, 1, 0, True, block_in)
                t = conv(w, w, 3, stride, 1, True, t)
            shortcut = block_in
            if stride != 1 or cin != cout:
                shortcut = conv(cin, cout, 1, stride, 0, False, block_in)
            if kind == "basic":
                cur = conv(w, cout, 3, 1, 1, True, t, res=shortcut)
            else:
                cur = conv(w, cout, 1, 1, 0, True, t, res=shortcut)
            cin = cout
    ops.append(Op(GAVGPOOL, cin, cin, 0, 0, 1, 0, 0, -1, cur))
    ops.append(Op(FC, cin, num_classes, 1, 1, 1, 0, 0, -1, len(ops) - 1))
    ops.append(Op(SOFTMAX, num_classes, num_classes, 0, 0, 1, 0, 0, -1, len(ops) - 1))
    return ops


def weight_shapes(ops):
    """(cout, cin, kh, kw) of every op that owns weights, in op order."""
    return [(o.cout, o.cin, o.kh, o.kw) for o in ops if o.op in (CONV, FC)]


def param_count(ops):
    return sum(k * c * r * s + k for (k, c, r, s) in weight_shapes(ops))


def out_hw(o, h, w):
    if o.op in (CONV, MAXPOOL):
        return ((h + 2 * o.pad - o.kh) // o.stride + 1,
                (w + 2 * o.pad - o.kw) // o.stride + 1)
    return (1, 1)


def shapes(ops, in_h, in_w):
    """(channels, height, width) of every op's output."""
    res = []
    for o in ops:
        h, w = (in_h, in_w) if o.input_from < 0 else res[o.input_from][1:]
        ho, wo = out_hw(o, h, w)
        res.append((o.cout, ho, wo))
    return res


def mac_count(ops, in_h, in_w):
    """Multiply-accumulates per image of the conv and FC ops."""
    total = 0
    for o, (c, h, w) in zip(ops, shapes(ops, in_h, in_w)):
        if o.op in (CONV, FC):
            total += c * h * w * o.cin * o.kh * o.kw
    return total
