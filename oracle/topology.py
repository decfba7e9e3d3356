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

CONV, MAXPOOL, GAVGPOOL, FC, SOFTMAX, CONCAT = 0, 1, 2, 3, 4, 5

# relu: activation after the (optional) shortcut addition: 0 none, 1 ReLU, 2 hard swish.
# pad: padding in both directions for a square filter; for kh != kw it is the padding in height and
# pad_w the padding in width.  groups: 0 or 1 = dense, cin = depthwise (cin == cout).
# CONCAT: channels of op input_from followed by those of op residual_from (cin = the first's, cout = both).
Op = namedtuple("Op", "op cin cout kh kw stride pad relu residual_from input_from pad_w groups",
                defaults=(0, 0))


def conv_geometry(o):
    """(pad_h, pad_w, groups) of a CONV op."""
    return o.pad, (o.pad if o.kh == o.kw else o.pad_w), max(1, o.groups)

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
    """(cout, cin / groups, kh, kw) of every op that owns weights, in op order."""
    return [(o.cout, o.cin // max(1, o.groups), o.kh, o.kw) for o in ops if o.op in (CONV, FC)]


def param_count(ops):
    return sum(k * c * r * s + k for (k, c, r, s) in weight_shapes(ops))


def out_hw(o, h, w):
    if o.op == CONV:
        ph, pw, _ = conv_geometry(o)
        return ((h + 2 * ph - o.kh) // o.stride + 1, (w + 2 * pw - o.kw) // o.stride + 1)
    if o.op == MAXPOOL:
        return ((h + 2 * o.pad - o.kh) // o.stride + 1,
                (w + 2 * o.pad - o.kw) // o.stride + 1)
    if o.op == CONCAT:
        return (h, w)
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
            total += c * h * w * (o.cin // max(1, o.groups)) * o.kh * o.kw
    return total


# ---- other model families of the paper's Table 1, as operator lists of the same kind ----------
def _tail(ops, cin, num_classes):
    ops.append(Op(GAVGPOOL, cin, cin, 0, 0, 1, 0, 0, -1, len(ops) - 1))
    ops.append(Op(FC, cin, num_classes, 1, 1, 1, 0, 0, -1, len(ops) - 1))
    ops.append(Op(SOFTMAX, num_classes, num_classes, 0, 0, 1, 0, 0, -1, len(ops) - 1))
    return ops


def mobilenet(num_classes=1000, hswish_from=7, residual=True):
    """Depthwise-separable network in the MobileNet style (the family of the paper's mobile pose
    model): 3x3 stride-2 stem 3->32, then 13 pairs of {3x3 depthwise, 1x1 pointwise} with widths
    64,128,128,256,256,512 x6,1024,1024 and strides 1,2,1,2,1,2,1,1,1,1,1,2,1; ReLU in the early
    pairs, hard swish (as in MobileNet-v3) from pair `hswish_from` on; where a pair keeps shape the
    pointwise convolution adds the pair's input before its activation (as the v2/v3 blocks do).
    Global average pool, FC, softmax.  Widths are multiples of 32 throughout."""
    cfg = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1), (512, 1),
           (512, 1), (512, 1), (1024, 2), (1024, 1)]
    ops = [Op(CONV, 3, 32, 3, 3, 2, 1, 1, -1, -1)]
    cin = 32
    for i, (cout, stride) in enumerate(cfg):
        act = 2 if i >= hswish_from else 1
        block_in = len(ops) - 1
        ops.append(Op(CONV, cin, cin, 3, 3, stride, 1, act, -1, block_in, 0, cin))
        res = block_in if (residual and stride == 1 and cin == cout) else -1
        ops.append(Op(CONV, cin, cout, 1, 1, 1, 0, act, res, len(ops) - 1))
        cin = cout
    return _tail(ops, cin, num_classes)


def dense_net(num_classes=1000, growth=32, layers=(6, 12), bottleneck=128, stem=64):
    """Densely connected network in the DenseNet style: 7x7 stride-2 stem and 3x3 max pool, then
    dense blocks in which every layer {1x1 to `bottleneck` channels, 3x3 to `growth` channels}
    reads the concatenation of the block input and all earlier layers' outputs; between blocks a
    1x1 convolution halves the channels and a 2x2 stride-2 max pool the resolution (the original
    averages there; this operator set has max pooling)."""
    ops = [Op(CONV, 3, stem, 7, 7, 2, 3, 1, -1, -1), Op(MAXPOOL, stem, stem, 3, 3, 2, 1, 0, -1, 0)]
    cin = stem
    for b, n in enumerate(layers):
        cur = len(ops) - 1
        for _ in range(n):
            ops.append(Op(CONV, cin, bottleneck, 1, 1, 1, 0, 1, -1, cur))
            ops.append(Op(CONV, bottleneck, growth, 3, 3, 1, 1, 1, -1, len(ops) - 1))
            ops.append(Op(CONCAT, cin, cin + growth, 0, 0, 1, 0, 0, len(ops) - 1, cur))
            cur = len(ops) - 1
            cin += growth
        if b + 1 < len(layers):
            ops.append(Op(CONV, cin, cin // 2, 1, 1, 1, 0, 1, -1, cur))
            cin //= 2
            ops.append(Op(MAXPOOL, cin, cin, 2, 2, 2, 0, 0, -1, len(ops) - 1))
    return _tail(ops, cin, num_classes)


def inception_net(num_classes=1000, width=256, blocks=2):
    """Network with the factorised 7x7 branches of Inception v3's 17x17 blocks: a 3x3 stride-2
    stem and a 3x3 stride-2 convolution, then blocks that concatenate a 1x1 branch with a
    {1x1, 1x7, 7x1} branch (both `width` channels wide) and mix the result with a 1x1."""
    ops = [Op(CONV, 3, 32, 3, 3, 2, 1, 1, -1, -1), Op(CONV, 32, width, 3, 3, 2, 1, 1, -1, 0)]
    for _ in range(blocks):
        x = len(ops) - 1
        ops.append(Op(CONV, width, width, 1, 1, 1, 0, 1, -1, x))                 # branch a
        a = len(ops) - 1
        ops.append(Op(CONV, width, width, 1, 1, 1, 0, 1, -1, x))                 # branch b
        ops.append(Op(CONV, width, width, 1, 7, 1, 0, 1, -1, len(ops) - 1, 3))   # 1x7, pad (0, 3)
        ops.append(Op(CONV, width, width, 7, 1, 1, 3, 1, -1, len(ops) - 1, 0))   # 7x1, pad (3, 0)
        ops.append(Op(CONCAT, width, 2 * width, 0, 0, 1, 0, 0, len(ops) - 1, a))
        ops.append(Op(CONV, 2 * width, width, 1, 1, 1, 0, 1, x, len(ops) - 1))   # mix + shortcut
    return _tail(ops, width, num_classes)
