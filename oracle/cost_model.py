"""Analytic cost model oracle (TEST INFRASTRUCTURE ONLY).

KARMA Sec. III-C takes the number of arithmetic operations of a block as the proxy of its
computational cost and projects it on the device's throughput; this file counts those
operations per block of the three model families, in plain Python integers, and turns them
into times.  Only tests may import it; the library's own counter (csrc/cost_model.cpp) shares
no code with it.

Operation counts per sample, as the paper lists them (one multiply-add = one operation):
  convolution      |Y| * K * K * C_in
  ReLU             |Y|
  pooling          |Y| * K * K * c, c = 1 for both pooling types here (global average pooling: one
                   operation per input element)
  batch norm       3 |B| + 4 |X| + 2 |Y|, with |B| = |X| = |Y| (the mini-batch mean and variance run
                   over the same elements): 9 |X|
  fully connected  |X| * |Y|
  softmax          2 |X|
  element-wise, tensor add (inferred, Sec. III-C "Other"): one operation per output element

Readings where the paper gives nothing usable:
  self-attention   the printed count has no sequence-length term; here: per head S*S*d multiply-adds
                   for Q K^T, S*S*d for P V, and a softmax over S*S scores (2 S*S); the causal mask is
                   not discounted
  layer norm       not listed; counted like batch normalisation (9 per element)
  GELU             element-wise: one per element
  embedding        one per output element (gather + positional add)
  cross entropy    the softmax count, 2 per logit
  backward         twice the forward count (one pass for the input gradient, one for the weight
                   gradient); recompute = forward
Matrix operations (convolution, fully connected, attention products) and all others are kept apart
because the device runs them at different rates:
  t_ns = ceil(matrix_ops * 1e9 / matrix_ops_per_s) + ceil(other_ops * 1e9 / other_ops_per_s)
"""


def ceil_div(a, b):
    return -(-a // b)


def time_ns(ops, rates):
    matrix, other = ops
    return ceil_div(matrix * 10**9, rates[0]) + ceil_div(other * 10**9, rates[1])


def conv_out(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


# ------------------------------------------------------------------ per-family counters
def mlp_blocks(width, n_layers, batch):
    """Linear(width -> width) + ReLU per block; loss: mean squared error (one op per element)."""
    blocks = [(batch * width * width, batch * width) for _ in range(n_layers)]
    loss = (0, batch * width)
    return blocks, loss


def gpt_blocks(n_layers, hidden, heads, ffn, vocab, seq, batch, split=False):
    """Block 0: embedding.  Blocks 1..n: LN, QKV projection, attention, output projection, residual
    add, LN, FC1, GELU, FC2, residual add.  Loss: final LN, tied LM head, softmax cross entropy.
    split: each transformer block as two entries, its attention half (up to the first residual add) and
    its feed-forward half."""
    T = batch * seq
    d = hidden // heads
    blocks = [(0, T * hidden)]
    attn_mm = batch * heads * 2 * seq * seq * d
    attn_softmax = batch * heads * 2 * seq * seq
    attention = (T * (hidden * 3 * hidden + hidden * hidden) + attn_mm, 9 * T * hidden + attn_softmax + T * hidden)
    feed_forward = (T * 2 * hidden * ffn, 9 * T * hidden + T * ffn + T * hidden)
    for _ in range(n_layers):
        if split:
            blocks += [attention, feed_forward]
        else:
            blocks.append((attention[0] + feed_forward[0], attention[1] + feed_forward[1]))
    loss = (T * hidden * vocab, 9 * T * hidden + 2 * T * vocab)
    return blocks, loss


def cnn_blocks(width, stage_blocks, image, batch, classes):
    """Block 0: stem (7x7 stride-2 convolution, batch norm, ReLU, 3x3 stride-2 max pooling).  Then the
    bottleneck blocks.  Loss: global average pooling, fully connected layer, softmax cross entropy."""
    h1 = conv_out(image, 7, 2, 3)
    h2 = conv_out(h1, 3, 2, 1)
    y_stem = batch * h1 * h1 * width
    blocks = [(y_stem * 7 * 7 * 3, 9 * y_stem + y_stem + batch * h2 * h2 * width * 9)]
    hw, cin = h2, width
    for st in range(4):
        mid, cout = width << st, 4 * (width << st)
        for k in range(stage_blocks[st]):
            stride = 2 if (k == 0 and st > 0) else 1
            ho = conv_out(hw, 3, stride, 1)
            p_in, p_out = batch * hw * hw, batch * ho * ho
            matrix = p_in * mid * cin + p_out * mid * 9 * mid + p_out * cout * mid
            other = 9 * p_in * mid + p_in * mid          # BN + ReLU after the 1x1
            other += 9 * p_out * mid + p_out * mid       # BN + ReLU after the 3x3
            other += 9 * p_out * cout                    # BN after the last 1x1
            if k == 0:                                   # projection shortcut: 1x1 (strided) + BN
                matrix += p_out * cout * cin
                other += 9 * p_out * cout
            other += 2 * p_out * cout                    # residual add + ReLU
            blocks.append((matrix, other))
            hw, cin = ho, cout
    loss = (batch * cin * classes, batch * hw * hw * cin + 2 * batch * classes)
    return blocks, loss


def wrn_blocks(width, group_blocks, image, batch, classes, stem=16):
    """Block 0: the first 3x3 convolution (3 -> stem channels).  Then the pre-activated basic blocks: batch
    norm + ReLU on the input, 3x3 convolution carrying the stride, batch norm + ReLU, 3x3 convolution,
    residual add, and a 1x1 shortcut convolution where the shape changes.  Loss: batch norm, ReLU, global
    average pooling, fully connected layer, softmax cross entropy."""
    hw, cin = image, stem
    blocks = [(batch * hw * hw * stem * 3 * 3 * 3, 0)]
    for gi in range(3):
        cout = width << gi
        for k in range(group_blocks[gi]):
            stride = 2 if (k == 0 and gi > 0) else 1
            ho = conv_out(hw, 3, stride, 1)
            p_in, p_out = batch * hw * hw, batch * ho * ho
            matrix = p_out * cout * 9 * cin + p_out * cout * 9 * cout
            if cin != cout:
                matrix += p_out * cout * cin
            other = 9 * p_in * cin + p_in * cin         # BN + ReLU on the input
            other += 9 * p_out * cout + p_out * cout    # BN + ReLU between the convolutions
            other += p_out * cout                       # residual add
            blocks.append((matrix, other))
            hw, cin = ho, cout
    pix = batch * hw * hw
    loss = (batch * cin * classes, 9 * pix * cin + pix * cin + pix * cin + 2 * batch * classes)
    return blocks, loss


def unet_blocks(width, depth, image, batch, classes):
    """Contracting levels 0..depth (level l >= 1: 2x2 max pooling of the level above, |Y| K K; then two 3x3
    convolutions, each with batch norm and ReLU), expansive levels depth-1..0 (2x2 stride-2 up-convolution: each
    output element takes one tap, |Y| C_in; then the two convolutions, the first over the concatenation of 2C
    channels).  Loss: 1x1 classifier over one image channel's worth of pixels, softmax cross entropy per pixel.
    The network reads one image channel."""
    blocks = []
    for l in range(depth + 1):
        p, c = batch * (image >> l) ** 2, width << l
        cin = (width << (l - 1)) if l else 1
        matrix = p * c * 9 * cin + p * c * 9 * c
        other = (p * cin * 2 * 2 if l else 0) + 2 * (9 * p * c + p * c)
        blocks.append((matrix, other))
    for l in range(depth - 1, -1, -1):
        p, c = batch * (image >> l) ** 2, width << l
        matrix = p * c * (width << (l + 1)) + p * c * 9 * (2 * c) + p * c * 9 * c
        blocks.append((matrix, 2 * (9 * p * c + p * c)))
    p0 = batch * image * image
    return blocks, (p0 * width * classes, 2 * p0 * classes)


def times(blocks, loss, rates):
    """Per block (t_fwd, t_bwd, t_recompute) in ns and the loss op's time (forward + gradient)."""
    out = []
    for ops in blocks:
        tf = time_ns(ops, rates)
        out.append((tf, 2 * tf, tf))
    return out, 3 * time_ns(loss, rates)
