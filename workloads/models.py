"""Tensor lists (shapes + shard rules) of the synthetic parameter sets.

Shapes only: no arithmetic of the method lives here.  A tensor descriptor is a
dict ``{"name", "rows", "cols", "rule", "sections", "layer"}`` (layer: the decoder layer the
tensor belongs to, -1 for what stands in front of the layers, -2 for what stands behind them;
it matters to pipeline-parallel plans only); rules are the interface
values 0 replicated, 1 split rows (dim 0), 2 split cols (dim 1), 3 fused rows
(dim 0 is a stack of sections, each split).  The layouts are the usual
tensor-parallel ones for a dense decoder: QKV / gate / up are column-parallel
(split along the output dim = dim 0 of the stored [out, in] matrix), o / down
are row-parallel (dim 1), embedding and lm_head are split along the vocabulary,
norm weights are replicated.
"""

REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS = 0, 1, 2, 3


LAYER_FIRST, LAYER_LAST = -1, -2


def _t(name, rows, cols, rule, sections=None, layer=0):
    return {"name": name, "rows": int(rows), "cols": int(cols), "rule": rule,
            "sections": [int(s) for s in sections] if sections else None, "layer": int(layer)}


def decoder(layers, hidden, q_heads, kv_heads, head_dim, inter, vocab, fused=True):
    """Dense decoder parameter set, untied embedding / lm_head, RMSNorm weights."""
    q, kv = q_heads * head_dim, kv_heads * head_dim
    ts = [_t("embed", vocab, hidden, SPLIT_ROWS, layer=LAYER_FIRST)]
    for i in range(layers):
        p = "l%d." % i
        ts.append(_t(p + "input_norm", 1, hidden, REPLICATED, layer=i))
        if fused:
            ts.append(_t(p + "qkv", q + 2 * kv, hidden, FUSED_ROWS, [q, kv, kv], layer=i))
        else:
            ts.append(_t(p + "q", q, hidden, SPLIT_ROWS, layer=i))
            ts.append(_t(p + "k", kv, hidden, SPLIT_ROWS, layer=i))
            ts.append(_t(p + "v", kv, hidden, SPLIT_ROWS, layer=i))
        ts.append(_t(p + "o", hidden, q, SPLIT_COLS, layer=i))
        ts.append(_t(p + "post_norm", 1, hidden, REPLICATED, layer=i))
        if fused:
            ts.append(_t(p + "gate_up", 2 * inter, hidden, FUSED_ROWS, [inter, inter], layer=i))
        else:
            ts.append(_t(p + "gate", inter, hidden, SPLIT_ROWS, layer=i))
            ts.append(_t(p + "up", inter, hidden, SPLIT_ROWS, layer=i))
        ts.append(_t(p + "down", hidden, inter, SPLIT_COLS, layer=i))
    ts.append(_t("final_norm", 1, hidden, REPLICATED, layer=LAYER_LAST))
    ts.append(_t("lm_head", vocab, hidden, SPLIT_ROWS, layer=LAYER_LAST))
    return ts


def single_matrix(rows=4096, cols=4096):
    """One matrix, one destination shard."""
    return [_t("w", rows, cols, SPLIT_ROWS)]


def flat(numel=1 << 30):
    """One flat tensor, one destination shard."""
    return [_t("flat", 1, numel, REPLICATED)]


def decoder_7b(layers=32, fused=True):
    """7B-style MHA decoder (hidden 4096, 32 heads of 128, SwiGLU 11008, vocab 32000); TP=4."""
    return decoder(layers, 4096, 32, 32, 128, 11008, 32000, fused)


def decoder_32b(layers=64):
    """32B-style GQA decoder (hidden 5120, 40 query / 8 KV heads of 128, SwiGLU 27648,
    vocab 152064), fused QKV and gate_up; TP=8 puts 5 query heads + 1 KV head on a shard."""
    return decoder(layers, 5120, 40, 8, 128, 27648, 152064, True)


def decoder_8b(layers=36):
    """8B-style GQA decoder (hidden 4096, 32 query / 8 KV heads of 128, SwiGLU 12288, vocab 151936),
    the paper's smaller model (Sec. 5: TP=4 for training, TP=1 for rollout)."""
    return decoder(layers, 4096, 32, 8, 128, 12288, 151936, True)


def pp_stage(tensors, layers, pp, stage):
    """The tensors a pipeline stage holds (Sec. 4.2: the transfer engine supports TP and PP): layers
    are dealt to the pp stages in equal consecutive groups, the embedding goes with the first stage,
    final norm and lm_head with the last.  Returns (ordinal in `tensors`, descriptor) pairs, in order."""
    if layers % pp:
        raise ValueError("layers must divide evenly over the pipeline stages")
    per = layers // pp
    out = []
    for i, t in enumerate(tensors):
        n = t["name"]
        if n == "embed":
            s = 0
        elif n in ("final_norm", "lm_head"):
            s = pp - 1
        else:
            s = int(n[1:n.index(".")]) // per
        if s == stage:
            out.append((i, t))
    return out


def numel(tensors):
    return sum(t["rows"] * t["cols"] for t in tensors)
