"""Parameter shapes of the models whose gradients the benchmark configurations imitate.

The paper's experiments (Section 4.1 "Datasets and Tasks", Table "Model Characteristics")
train VGG16, BERT-LARGE, BERT-BASE, a Transformer and LSTM+AlexNet on datasets that are not
available here; the benchmark configurations name ResNet-50 and BERT shapes instead, and the
shapes are generated from the architecture numbers alone (no weights, no data).
"""


def resnet50_shapes():
    """[(name, shape)] in definition order; 161 tensors, 25,557,032 elements."""
    out = []

    def conv_bn(name, cin, cout, k):
        out.append((name + ".conv.weight", (cout, cin, k, k)))
        out.append((name + ".bn.weight", (cout,)))
        out.append((name + ".bn.bias", (cout,)))

    conv_bn("stem", 3, 64, 7)
    cin = 64
    for s, (blocks, width) in enumerate(zip((3, 4, 6, 3), (64, 128, 256, 512))):
        for b in range(blocks):
            p = "stage%d.block%d" % (s + 1, b)
            conv_bn(p + ".a", cin, width, 1)
            conv_bn(p + ".b", width, width, 3)
            conv_bn(p + ".c", width, width * 4, 1)
            if b == 0:
                conv_bn(p + ".down", cin, width * 4, 1)
            cin = width * 4
    out.append(("fc.weight", (1000, 2048)))
    out.append(("fc.bias", (1000,)))
    return out


def bert_shapes(layers, hidden, ffn, vocab=30522, positions=512, types=2):
    """[(name, shape)] of a BERT encoder with pooler, in definition order.

    bert_shapes(24, 1024, 4096) is the "BERT-large" configuration (about 335M elements),
    bert_shapes(12, 768, 3072) the "BERT-base" one (about 109.5M elements).
    """
    out = [("emb.word", (vocab, hidden)), ("emb.position", (positions, hidden)),
           ("emb.type", (types, hidden)), ("emb.ln.weight", (hidden,)), ("emb.ln.bias", (hidden,))]
    for l in range(layers):
        p = "layer%d" % l
        for proj in ("q", "k", "v", "o"):
            out.append(("%s.attn.%s.weight" % (p, proj), (hidden, hidden)))
            out.append(("%s.attn.%s.bias" % (p, proj), (hidden,)))
        out.append((p + ".attn.ln.weight", (hidden,)))
        out.append((p + ".attn.ln.bias", (hidden,)))
        out.append((p + ".ffn.in.weight", (ffn, hidden)))
        out.append((p + ".ffn.in.bias", (ffn,)))
        out.append((p + ".ffn.out.weight", (hidden, ffn)))
        out.append((p + ".ffn.out.bias", (hidden,)))
        out.append((p + ".ffn.ln.weight", (hidden,)))
        out.append((p + ".ffn.ln.bias", (hidden,)))
    out.append(("pooler.weight", (hidden, hidden)))
    out.append(("pooler.bias", (hidden,)))
    return out


def numel(shape):
    n = 1
    for d in shape:
        n *= d
    return n
