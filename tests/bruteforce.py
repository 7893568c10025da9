"""Nested-loop Python forward pass for toy sizes.

Written from the operator definitions, independently of the C oracle: plain
Python floats (fp64) and lists only.  Used to pin the oracle's whole forward.
"""


def forward(dense, tables, indices, lengths, bottom, top):
    B = len(dense)
    T = len(tables)
    D = len(tables[0][0])
    # bag boundaries, table-major
    starts, pos = [], 0
    for n in lengths:
        starts.append(pos)
        pos += n
    pooled = [[[0.0] * D for _ in range(T)] for _ in range(B)]
    for t in range(T):
        for b in range(B):
            s = starts[t * B + b]
            for k in range(s, s + lengths[t * B + b]):
                row = tables[t][indices[k]]
                for d in range(D):
                    pooled[b][t][d] += float(row[d])

    def layer(x, W, bias, relu):
        y = []
        for o in range(len(W)):
            acc = 0.0
            for i in range(len(x)):
                acc += float(W[o][i]) * x[i]
            acc += float(bias[o])
            y.append(max(acc, 0.0) if relu else acc)
        return y

    logits, inter_all, x0_all = [], [], []
    for b in range(B):
        h = [float(v) for v in dense[b]]
        for W, bias in bottom:
            h = layer(h, W, bias, True)
        x0_all.append(h)
        vecs = [h] + pooled[b]
        feat = list(h)
        for i in range(1, T + 1):
            for j in range(i):
                feat.append(sum(vecs[i][d] * vecs[j][d] for d in range(D)))
        inter_all.append(feat)
        z = feat
        for li, (W, bias) in enumerate(top):
            z = layer(z, W, bias, li + 1 < len(top))
        logits.append(z[0])
    return {"pooled": pooled, "bottom_out": x0_all, "interact": inter_all, "logits": logits}


def forward_towers(dense, tables, indices, lengths, bottom, towers):
    """Concatenation model: looked-up (pooled) vectors appended to the dense
    part, no interaction, one Predict-FC tower per task."""
    B, T, D = len(dense), len(tables), len(tables[0][0])
    logits, cat_all = [], []
    pos = [0]
    for n in lengths:
        pos.append(pos[-1] + n)
    for b in range(B):
        h = [float(v) for v in dense[b]]
        for W, bias in bottom:
            h = [max(sum(float(W[o][i]) * h[i] for i in range(len(h))) + float(bias[o]), 0.0)
                 for o in range(len(W))]
        feat = list(h)
        for t in range(T):
            vec = [0.0] * D
            for k in range(pos[t * B + b], pos[t * B + b + 1]):
                for d in range(D):
                    vec[d] += float(tables[t][indices[k]][d])
            feat += vec
        cat_all.append(feat)
        outs = []
        for tower in towers:
            z = feat
            for li, (W, bias) in enumerate(tower):
                y = [sum(float(W[o][i]) * z[i] for i in range(len(z))) + float(bias[o])
                     for o in range(len(W))]
                z = [max(v, 0.0) for v in y] if li + 1 < len(tower) else y
            outs.append(z[0])
        logits.append(outs)
    return {"concat": cat_all, "logits": logits}
