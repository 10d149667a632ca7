"""Seeded synthetic inputs shared by the oracle-side tests and the GPU-side harness.

Holds no arithmetic of the method itself: only a counter-based random generator
(splitmix64 -> uniform / Box-Muller normal), the initialisers the workload list
prescribes (Xavier-uniform for the MLP, N(0, 0.02) for GPT weights) and random cost
records for planner tests.  Everything is produced on the host as numpy arrays and
handed to whichever side asks, so initialisation is never a parity variable.
"""
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(seed, n):
    """n 64-bit words of the splitmix64 stream that starts at `seed`."""
    with np.errstate(over="ignore"):
        idx = np.arange(1, n + 1, dtype=np.uint64)
        z = np.uint64(seed) + idx * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def uniform01(seed, n):
    """Doubles in [0, 1) from the top 53 bits."""
    return (splitmix64(seed, n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(seed, shape, std=1.0):
    n = int(np.prod(shape))
    m = (n + 1) // 2
    u1 = 1.0 - uniform01(seed, m)                      # (0, 1]
    u2 = uniform01(seed ^ 0x5DEECE66D, m)
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.concatenate([r * np.cos(2 * np.pi * u2), r * np.sin(2 * np.pi * u2)])[:n]
    return (z * std).reshape(shape)


def uniform(seed, shape, lo, hi):
    n = int(np.prod(shape))
    return (lo + (hi - lo) * uniform01(seed, n)).reshape(shape)


def randint(seed, shape, hi):
    n = int(np.prod(shape))
    return (splitmix64(seed, n) % np.uint64(hi)).astype(np.int64).reshape(shape)


# ------------------------------------------------------------------ workloads
def mlp_problem(seed=2008114201, n_layers=8, width=256, batch=32):
    """Config 1: Xavier-uniform weights [out, in], zero biases, N(0,1) inputs/targets."""
    bound = float(np.sqrt(6.0 / (width + width)))
    Ws = [uniform(seed + 11 * i + 1, (width, width), -bound, bound) for i in range(n_layers)]
    bs = [np.zeros(width) for _ in range(n_layers)]
    x = normal(seed + 1001, (batch, width))
    t = normal(seed + 1002, (batch, width))
    return Ws, bs, x, t


# Keys of one transformer block's parameter dict, in the order the library numbers a block's tensors.
GPT_BLOCK_TENSORS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def gpt_problem(seed=2008114202, n_layers=24, hidden=1024, ffn=4096, vocab=32000,
                seq=1024, batch=32, std=0.02, bias_std=0.0):
    """Configs 2/4/5: N(0, std) weights, LayerNorm gain 1 / shift 0, biases N(0,
    bias_std) (0 by default; tests use a non-zero value so that bias paths matter),
    token ids and labels uniform over the vocabulary."""
    def w(k, shape, s=std):
        return normal(seed + 7919 * k, shape, s)
    params = dict(wte=w(1, (vocab, hidden)), wpe=w(2, (seq, hidden)),
                  lnf_g=np.ones(hidden), lnf_b=np.zeros(hidden), blocks=[])
    for i in range(n_layers):
        k = 10 + 10 * i
        def bias(j, n):
            return w(k + j, (n,), bias_std) if bias_std else np.zeros(n)
        params["blocks"].append(dict(
            ln1_g=np.ones(hidden) + (w(k + 8, (hidden,), bias_std) if bias_std else 0),
            ln1_b=bias(9, hidden),
            wqkv=w(k, (3 * hidden, hidden)), bqkv=bias(4, 3 * hidden),
            wo=w(k + 1, (hidden, hidden)), bo=bias(5, hidden),
            ln2_g=np.ones(hidden) + (w(k + 8, (hidden,), bias_std)[::-1] if bias_std else 0),
            ln2_b=bias(9, hidden)[::-1].copy(),
            w1=w(k + 2, (ffn, hidden)), b1=bias(6, ffn),
            w2=w(k + 3, (hidden, ffn)), b2=bias(7, hidden)))
    ids = randint(seed + 3, (batch, seq), vocab)
    labels = randint(seed + 5, (batch, seq), vocab)
    return params, ids, labels


# ------------------------------------------------------------------ planner stacks
def random_stack(seed, n_layers, kind="homogeneous"):
    """Random integer cost records (tf, tb, trc, sav, out, ws) for planner tests.
    kinds: homogeneous | front_heavy (memory shrinks with depth, as in CNNs) |
    back_heavy | imbalanced (compute and memory uncorrelated)."""
    r = splitmix64(seed, 8 * n_layers + 8)
    rows = []
    for i in range(n_layers):
        a = [int(v) for v in r[8 * i:8 * i + 8]]
        if kind == "homogeneous":
            tf = 1000 + a[0] % 50
            sav = 4096 * (8 + a[1] % 2)
            out = 4096
        elif kind == "front_heavy":
            tf = 800 + a[0] % 400
            sav = 4096 * (2 + 30 * (n_layers - i) // n_layers + a[1] % 3)
            out = 1024 * (1 + 8 * (n_layers - i) // n_layers)
        elif kind == "back_heavy":
            tf = 800 + a[0] % 400
            sav = 4096 * (2 + 30 * (i + 1) // n_layers + a[1] % 3)
            out = 1024 * (1 + 8 * (i + 1) // n_layers)
        else:
            tf = 200 + a[0] % 3000
            sav = 1024 * (1 + a[1] % 64)
            out = 256 * (1 + a[2] % 32)
        tb = 2 * tf + a[3] % 100
        trc = tf - a[4] % (tf // 10 + 1)
        ws = 256 * (a[5] % 8)
        rows.append((tf, tb, trc, sav, out, ws))
    return rows


# ------------------------------------------------------------------ bottleneck CNN
# Keys of one bottleneck block's parameter dict, in the order the library numbers a block's tensors
# (wp, gp, bp: projection shortcut, present on the first block of a stage only).
BOTTLENECK_TENSORS = ("w1", "g1", "b1", "w2", "g2", "b2", "w3", "g3", "b3", "wp", "gp", "bp")


def cnn_problem(seed=2008114203, width=64, stage_blocks=(3, 24, 36, 3), image=224, batch=64, classes=1000,
                bn_jitter=0.0):
    """Config 3: bottleneck residual network.  Convolution weights N(0, sqrt(2 / (k*k*c_out)))
    (Kaiming-normal, fan-out), batch-norm gain 1 / shift 0 (plus N(0, bn_jitter) in tests so
    that both matter), fully connected layer N(0, 0.01) with zero bias, images N(0, 1),
    labels uniform over the classes.  Layout: weights [c_out][k][k][c_in], images NHWC."""
    k = [0]

    def nxt():
        k[0] += 1
        return seed + 7919 * k[0]

    def conv(co, r, ci):
        return normal(nxt(), (co, r, r, ci), (2.0 / (r * r * co)) ** 0.5)

    def bn(c):
        g, b = np.ones(c), np.zeros(c)
        if bn_jitter:
            g = g + normal(nxt(), (c,), bn_jitter)
            b = b + normal(nxt(), (c,), bn_jitter)
        return g, b

    g, b = bn(width)
    params = dict(stem=dict(w=conv(width, 7, 3), g=g, b=b), blocks=[], head=None)
    cin = width
    for st, nb in enumerate(stage_blocks):
        mid, cout = width << st, 4 * (width << st)
        for j in range(nb):
            p = dict(w1=conv(mid, 1, cin), w2=conv(mid, 3, mid), w3=conv(cout, 1, mid))
            p["g1"], p["b1"] = bn(mid)
            p["g2"], p["b2"] = bn(mid)
            p["g3"], p["b3"] = bn(cout)
            if j == 0:
                p["wp"] = conv(cout, 1, cin)
                p["gp"], p["bp"] = bn(cout)
            params["blocks"].append((p, 2 if (j == 0 and st > 0) else 1))
            cin = cout
    params["head"] = dict(w=normal(nxt(), (classes, cin), 0.01), b=np.zeros(classes))
    images = normal(nxt(), (batch, image, image, 3))
    labels = randint(nxt(), (batch,), classes)
    return params, images, labels


# ------------------------------------------------------------------ wide residual network
# Keys of one basic block's parameter dict, in the order the library numbers a block's tensors
# (ws: the shortcut convolution, present on blocks that change the shape only).
BASIC_TENSORS = ("g1", "b1", "w1", "g2", "b2", "w2", "ws")


def wrn_problem(seed=2008114204, width=160, group_blocks=(4, 4, 4), image=32, batch=128, classes=10, stem=16,
                bn_jitter=0.0):
    """WRN-28-10 shapes by default: a 3x3 convolution to `stem` channels, three groups of basic blocks of
    width, 2*width and 4*width channels (stride 2 at the start of the second and third), batch norm, ReLU,
    global average pooling, fully connected layer.  Weights as for the bottleneck network: Kaiming-normal
    (fan-out) convolutions, batch-norm gain 1 / shift 0 (plus N(0, bn_jitter) in tests), fully connected
    layer N(0, 0.01) with zero bias; images N(0, 1); labels uniform over the classes."""
    k = [0]

    def nxt():
        k[0] += 1
        return seed + 7919 * k[0]

    def conv(co, r, ci):
        return normal(nxt(), (co, r, r, ci), (2.0 / (r * r * co)) ** 0.5)

    def bn(c):
        g, b = np.ones(c), np.zeros(c)
        if bn_jitter:
            g = g + normal(nxt(), (c,), bn_jitter)
            b = b + normal(nxt(), (c,), bn_jitter)
        return g, b

    params = dict(stem=dict(w=conv(stem, 3, 3)), blocks=[], head=None)
    cin = stem
    for gi, nb in enumerate(group_blocks):
        cout = width << gi
        for j in range(nb):
            p = {}
            p["g1"], p["b1"] = bn(cin)
            p["w1"] = conv(cout, 3, cin)
            p["g2"], p["b2"] = bn(cout)
            p["w2"] = conv(cout, 3, cout)
            if cin != cout:
                p["ws"] = conv(cout, 1, cin)
            params["blocks"].append((p, 2 if (j == 0 and gi > 0) else 1))
            cin = cout
    g, b = bn(cin)
    params["head"] = dict(g=g, b=b, w=normal(nxt(), (classes, cin), 0.01), bias=np.zeros(classes))
    images = normal(nxt(), (batch, image, image, 3))
    labels = randint(nxt(), (batch,), classes)
    return params, images, labels


LEVEL_TENSORS = ("w1", "g1", "b1", "w2", "g2", "b2")
UP_TENSORS = ("wu",) + LEVEL_TENSORS


def unet_problem(seed=2008114205, width=64, depth=4, image=512, batch=4, classes=2, bn_jitter=0.0):
    """U-Net shapes by default (the ssTEM sections of Table III: 512x512, one channel, two classes): depth + 1
    contracting levels of two 3x3 convolutions with width << level channels, depth expansive levels (2x2
    up-convolution [c_in][2][2][c_out], then two 3x3 convolutions, the first reading the contracting
    output's channels followed by the up-convolution's), 1x1 classifier.  Kaiming-normal (fan-out)
    convolutions, batch-norm gain 1 / shift 0 (plus N(0, bn_jitter) in tests), classifier N(0, 0.01) with zero
    bias; images N(0, 1); labels per pixel, smooth blobs: the sign pattern of a coarse random field, so that
    neighbouring pixels mostly agree as they do in a segmentation mask."""
    k = [0]

    def nxt():
        k[0] += 1
        return seed + 7919 * k[0]

    def conv(co, r, ci):
        return normal(nxt(), (co, r, r, ci), (2.0 / (r * r * co)) ** 0.5)

    def bn(c):
        g, b = np.ones(c), np.zeros(c)
        if bn_jitter:
            g = g + normal(nxt(), (c,), bn_jitter)
            b = b + normal(nxt(), (c,), bn_jitter)
        return g, b

    def level(cin, c):
        p = {}
        p["w1"] = conv(c, 3, cin)
        p["g1"], p["b1"] = bn(c)
        p["w2"] = conv(c, 3, c)
        p["g2"], p["b2"] = bn(c)
        return p

    params = dict(down=[], up=[], head=None)
    cin = 1
    for l in range(depth + 1):
        params["down"].append(level(cin, width << l))
        cin = width << l
    for j in range(depth):
        c = width << (depth - 1 - j)
        p = level(2 * c, c)
        p["wu"] = normal(nxt(), (2 * c, 2, 2, c), (2.0 / (4 * c)) ** 0.5)
        params["up"].append(p)
    params["head"] = dict(w=normal(nxt(), (classes, width), 0.01), bias=np.zeros(classes))
    images = normal(nxt(), (batch, image, image, 1))
    coarse = max(1, image // 8)
    field = randint(nxt(), (batch, (image + coarse - 1) // coarse, (image + coarse - 1) // coarse), classes)
    labels = np.repeat(np.repeat(field, coarse, axis=1), coarse, axis=2)[:, :image, :image]
    return params, images, np.ascontiguousarray(labels)
