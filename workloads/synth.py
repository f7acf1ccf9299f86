"""Seeded synthetic weight pairs (W_{t-1}, W_t) for tests and benchmarks.

Input recipes only: nothing here compares, compacts, maps to shards or applies.
They stand in for consecutive RL checkpoints (Sec. 4.2 reports > 95 % of the
delta's elements to be zero per layer, Sec. 6.3 about 99 % over training, with a
sweep of the non-zero fraction up to the 20 % crossover).

All generators run on the device they are given (``cpu`` for the small cases,
``cuda`` for full-size ones) from a ``torch.Generator`` seeded per tensor, so a
pair is reproducible from ``(seed, ordinal, shape, recipe, device type)``.
The caller copies the pair to the other side; it is never generated twice.
"""
import torch


def tensor_seed(base_seed, ordinal):
    return (int(base_seed) * 1000003 + int(ordinal) * 7919 + 12345) & 0x7FFFFFFF


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def gen_old(numel, g, device, std=0.02):
    """W_{t-1}: N(0, std^2) drawn in fp32, rounded to bf16 by torch's cast."""
    return (torch.randn(numel, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)


def ulp_shift(old, mask, steps):
    """Move the selected bf16 elements by ``steps`` (signed, non-zero) units in the last
    place, on the sign-magnitude number line (so a shift can cross zero).  Always
    changes the bit pattern of a selected element."""
    b = old.view(torch.int16).to(torch.int32) & 0xFFFF
    mag = b & 0x7FFF
    key = torch.where((b & 0x8000) != 0, -mag, mag)
    key2 = key + steps
    nb = torch.where(key2 < 0, 0x8000 | (-key2), key2)
    nb = torch.where(mask, nb, b)
    nb = ((nb + 0x8000) & 0xFFFF) - 0x8000          # to the int16 range
    return nb.to(torch.int16).view(torch.bfloat16)


def pair_bernoulli(numel, p, seed, device="cpu", chunk=1 << 28):
    """old ~ N(0, 0.02) bf16; new = old with an i.i.d. Bernoulli(p) set of elements moved
    by +-1..3 ulp (size and sign uniform).  Returns flat (old, new) bf16 tensors."""
    g = _gen(device, seed)
    old = torch.empty(numel, dtype=torch.bfloat16, device=device)
    new = torch.empty(numel, dtype=torch.bfloat16, device=device)
    for a in range(0, numel, chunk):
        n = min(chunk, numel - a)
        o = gen_old(n, g, device)
        mask = torch.rand(n, generator=g, device=device) < p
        k = torch.randint(1, 4, (n,), generator=g, device=device, dtype=torch.int32)
        sgn = torch.randint(0, 2, (n,), generator=g, device=device, dtype=torch.int32) * 2 - 1
        old[a:a + n] = o
        new[a:a + n] = ulp_shift(o, mask, k * sgn)
    return old, new


def pair_any_patterns(numel, p, seed, device="cpu"):
    """Value stress for the arithmetic payload: old = N(0, 0.02) bf16 with one element in eight
    replaced by an arbitrary 16-bit pattern (infinities, NaNs, subnormals, both zeros) and one in
    eight by a tiny value (exponent field 0..3); a Bernoulli(p) set of elements changes, a third of
    them by +-1..3 ulp, a third to an arbitrary pattern, a third to a tiny value of either sign.
    Returns flat (old, new) bf16 tensors."""
    g = _gen(device, seed)
    o = gen_old(numel, g, device).view(torch.int16).to(torch.int32) & 0xFFFF
    anyp = torch.randint(0, 1 << 16, (numel,), generator=g, device=device, dtype=torch.int32)
    tiny = torch.randint(0, 0x0200, (numel,), generator=g, device=device, dtype=torch.int32) | \
        (torch.randint(0, 2, (numel,), generator=g, device=device, dtype=torch.int32) << 15)
    kind_o = torch.randint(0, 8, (numel,), generator=g, device=device)
    o = torch.where(kind_o == 0, anyp, torch.where(kind_o == 1, tiny, o))
    old = (((o + 0x8000) & 0xFFFF) - 0x8000).to(torch.int16).view(torch.bfloat16)
    mask = torch.rand(numel, generator=g, device=device) < p
    kind_n = torch.randint(0, 3, (numel,), generator=g, device=device)
    k = torch.randint(1, 4, (numel,), generator=g, device=device, dtype=torch.int32)
    sgn = torch.randint(0, 2, (numel,), generator=g, device=device, dtype=torch.int32) * 2 - 1
    near = ulp_shift(old, mask, k * sgn).view(torch.int16).to(torch.int32) & 0xFFFF
    anyn = torch.randint(0, 1 << 16, (numel,), generator=g, device=device, dtype=torch.int32)
    tinyn = torch.randint(0, 0x0200, (numel,), generator=g, device=device, dtype=torch.int32) | \
        (torch.randint(0, 2, (numel,), generator=g, device=device, dtype=torch.int32) << 15)
    n = torch.where(kind_n == 0, near, torch.where(kind_n == 1, anyn, tinyn))
    n = torch.where(mask, n, o)
    new = (((n + 0x8000) & 0xFFFF) - 0x8000).to(torch.int16).view(torch.bfloat16)
    return old, new


def pair_clustered_f32(rows, cols, seed, device="cpu", active_rows=None, sigma=1e-4):
    """fp32-master variant: new32 = float(old_bf16) + N(0, sigma^2) on selected elements,
    exact upcast elsewhere.  Row r gets its own change rate q_r ~ Beta(0.5, 20); with
    ``active_rows`` given only that many rows, sampled uniformly without replacement,
    get a non-zero rate.  Returns (old bf16 [rows*cols], new fp32 [rows*cols])."""
    g = _gen(device, seed)
    n = rows * cols
    old = gen_old(n, g, device)
    # Beta(a,b) = X/(X+Y) with X ~ Gamma(a), Y ~ Gamma(b); drawn on the CPU (small: one per row)
    gc = _gen("cpu", seed ^ 0x5A5A5A5)
    x = torch._standard_gamma(torch.full((rows,), 0.5, dtype=torch.float64), generator=gc)
    y = torch._standard_gamma(torch.full((rows,), 20.0, dtype=torch.float64), generator=gc)
    q = (x / (x + y)).to(torch.float32)
    if active_rows is not None and active_rows < rows:
        keep = torch.zeros(rows, dtype=torch.bool)
        keep[torch.randperm(rows, generator=gc)[:active_rows]] = True
        q = torch.where(keep, q, torch.zeros_like(q))
    q = q.to(device)
    new = old.to(torch.float32)
    rows_per = max(1, (1 << 28) // max(cols, 1))
    for r0 in range(0, rows, rows_per):
        r1 = min(rows, r0 + rows_per)
        m = (r1 - r0) * cols
        sel = torch.rand(m, generator=g, device=device).view(r1 - r0, cols) < q[r0:r1, None]
        eps = torch.randn(m, generator=g, device=device, dtype=torch.float32).view(r1 - r0, cols) * sigma
        blk = new[r0 * cols:r1 * cols].view(r1 - r0, cols)
        blk += torch.where(sel, eps, torch.zeros_like(eps))
    return old, new


def model_pairs(tensors, recipe, seed, device="cpu", only=None, **kw):
    """Yield (ordinal, descriptor, old, new) for every tensor of a parameter set.

    recipe "bernoulli": kw p=...;  recipe "clustered_f32": kw vocab_active=... rows of the
    vocabulary-split tensors (named embed / lm_head) that may change.  `only`: one flag per
    tensor; a tensor whose flag is false is not generated (old = new = None), the others get the
    values they would have had anyway."""
    for i, t in enumerate(tensors):
        if only is not None and not only[i]:
            yield i, t, None, None
            continue
        s = tensor_seed(seed, i)
        if recipe == "bernoulli":
            old, new = pair_bernoulli(t["rows"] * t["cols"], kw["p"], s, device)
        elif recipe == "any_patterns":
            old, new = pair_any_patterns(t["rows"] * t["cols"], kw["p"], s, device)
        elif recipe == "clustered_f32":
            act = kw.get("vocab_active") if t["name"] in ("embed", "lm_head") else None
            old, new = pair_clustered_f32(t["rows"], t["cols"], s, device, active_rows=act)
        else:
            raise ValueError(recipe)
        yield i, t, old, new
