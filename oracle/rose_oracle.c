/*
 * CPU oracle for sparse weight-delta synchronisation (ROSE, Sec. 4.2,
 * "Shard-aware Weight Transfer" and "Sparsity-aware Weight Transfer").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the method computes, used only to check the GPU library
 * and to be timed beside it as a baseline.  It shares no code, header, table
 * or helper with the GPU library and must never be called from it.
 *
 * What the paper fixes (Sec. 4.2): the delta dW_t = W_t - W_{t-1} is sent in
 * COO form, losslessly, only non-zero elements; the COO data is split by the
 * receiver's parallel layout so that every receiving device applies only its
 * own part onto its resident W_{t-1}; each parameter carries a rule naming
 * the dimension that is split and the slice of it that each rank holds.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - weights are 16-bit patterns (bf16); "non-zero delta" means the two bit
 *     patterns differ (so +0 -> -0 is a change, an identical NaN is not);
 *   - the payload of an entry is the NEW 16-bit pattern, applying = overwrite
 *     (an arithmetic bf16 difference is not exact in general, so alone it
 *     could not be lossless); the arithmetic variant further down carries the
 *     rounded difference where that is exact and escapes to the pattern
 *     where it is not;
 *   - an entry's coordinate is one linear index, local to the destination
 *     shard's copy of that tensor (int32);
 *   - entries of one (tensor, shard) segment are in ascending local index;
 *   - a replicated tensor's entries go to every shard.
 *
 * Parity pins live in tests/ (numpy flatnonzero for TP=1, numpy slicing for
 * the shard map, round-trip and counting invariants, torch's CPU cast for
 * round-to-nearest-even, hand-written stage tables for the pipeline split).
 * No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stddef.h>

/* shard rules (values are part of the tested interface) */
enum {
    ORC_REPLICATED = 0, /* every shard holds the whole tensor                */
    ORC_SPLIT_ROWS = 1, /* dim 0 cut into D equal row blocks                 */
    ORC_SPLIT_COLS = 2, /* dim 1 cut into D equal column blocks              */
    ORC_FUSED_ROWS = 3  /* dim 0 is a stack of sections, each cut into D     */
};

enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_BAD_SHAPE = 2, ORC_RANGE = 3, ORC_ORDER = 4 };

/*
 * fp32 bit pattern -> bf16 bit pattern, round to nearest, ties to even
 * (IEEE 754 roundTiesToEven applied to the 16 discarded mantissa bits).
 * NaN stays NaN: keep the top 16 bits and set the quiet bit.
 */
uint16_t orc_rne_bf16(uint32_t u)
{
    uint32_t mag = u & 0x7FFFFFFFu;
    if (mag > 0x7F800000u) {
        return (uint16_t)((u >> 16) | 0x0040u);
    }
    uint32_t keep = u >> 16;        /* truncated result                    */
    uint32_t rest = u & 0xFFFFu;    /* discarded bits, half = 0x8000       */
    if (rest > 0x8000u) {
        keep += 1;                  /* above half: up                      */
    } else if (rest == 0x8000u) {
        if (keep & 1u) keep += 1;   /* exactly half: to even               */
    }
    return (uint16_t)keep;          /* a carry into the exponent is right:
                                       the largest finite rounds to inf    */
}

void orc_rne_bf16_array(const uint32_t *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_rne_bf16(in[i]);
}

/* shape checks shared by the functions below */
static int check_shape(int rule, int64_t R, int64_t C, int n_sec,
                       const int64_t *sec, int D)
{
    if (R < 0 || C < 0 || D < 1) return ORC_BAD_ARG;
    switch (rule) {
    case ORC_REPLICATED: return ORC_OK;
    case ORC_SPLIT_ROWS: return (R % D) ? ORC_BAD_SHAPE : ORC_OK;
    case ORC_SPLIT_COLS: return (C % D) ? ORC_BAD_SHAPE : ORC_OK;
    case ORC_FUSED_ROWS: {
        if (n_sec < 1 || !sec) return ORC_BAD_ARG;
        int64_t sum = 0;
        for (int j = 0; j < n_sec; ++j) {
            if (sec[j] < 0 || sec[j] % D) return ORC_BAD_SHAPE;
            sum += sec[j];
        }
        return (sum == R) ? ORC_OK : ORC_BAD_SHAPE;
    }
    default: return ORC_BAD_ARG;
    }
}

/* number of elements of shard d's local copy of an (R,C) tensor */
int64_t orc_local_numel(int rule, int64_t R, int64_t C, int D)
{
    if (rule == ORC_REPLICATED) return R * C;
    return (R * C) / D;
}

/*
 * Shard map (Sec. 4.2 "Shard-aware": sharded dimension -> per-rank slice
 * ranges; textbook tensor-parallel slicing).  Element (r,c) of the full
 * (R,C) tensor lives on shards d_first .. d_first+n_dest-1 at flat local
 * index *local (the same on each of them).
 */
int orc_shard_map(int rule, int64_t R, int64_t C, int n_sec, const int64_t *sec,
                  int D, int64_t r, int64_t c,
                  int *d_first, int *n_dest, int64_t *local)
{
    int rc = check_shape(rule, R, C, n_sec, sec, D);
    if (rc) return rc;
    if (r < 0 || r >= R || c < 0 || c >= C) return ORC_RANGE;

    if (rule == ORC_REPLICATED) {
        *d_first = 0; *n_dest = D; *local = r * C + c;
    } else if (rule == ORC_SPLIT_ROWS) {
        int64_t rows_per = R / D;
        int64_t d = r / rows_per;
        *d_first = (int)d; *n_dest = 1;
        *local = (r - d * rows_per) * C + c;
    } else if (rule == ORC_SPLIT_COLS) {
        int64_t cols_per = C / D;
        int64_t d = c / cols_per;
        *d_first = (int)d; *n_dest = 1;
        *local = r * cols_per + (c - d * cols_per);
    } else { /* ORC_FUSED_ROWS */
        int64_t sec_first_row = 0;   /* first full-tensor row of section j  */
        int64_t loc_first_row = 0;   /* first local row of section j's part */
        int j = 0;
        while (r >= sec_first_row + sec[j]) {
            sec_first_row += sec[j];
            loc_first_row += sec[j] / D;
            ++j;
        }
        int64_t in_sec = r - sec_first_row;
        int64_t per = sec[j] / D;
        int64_t d = in_sec / per;
        *d_first = (int)d; *n_dest = 1;
        *local = (loc_first_row + (in_sec - d * per)) * C + c;
    }
    return ORC_OK;
}

/*
 * Dense-to-sparse for ONE tensor (Sec. 4.2 "Sparsity-aware"; App. F "D2S").
 *
 * old_bits : R*C bf16 patterns (W_{t-1})
 * new_data : R*C bf16 patterns, or R*C fp32 patterns when new_is_f32 != 0
 *            (then the new weight is first rounded to bf16, ties to even)
 * counts   : [D] out, number of entries for each shard
 * idx, val : [D] arrays of caller buffers, or NULL to only count.  When given,
 *            buffer d must hold counts[d] entries (call once to count first).
 *
 * Three plain loops: row, column, destination.  Entries come out in ascending
 * (r,c); the function checks that this is also ascending local index.
 */
int orc_encode_tensor(const uint16_t *old_bits, const void *new_data, int new_is_f32,
                      int rule, int64_t R, int64_t C, int n_sec, const int64_t *sec,
                      int D, int64_t *counts, int32_t *const *idx, uint16_t *const *val)
{
    int rc = check_shape(rule, R, C, n_sec, sec, D);
    if (rc) return rc;
    if (orc_local_numel(rule, R, C, D) > (int64_t)INT32_MAX) return ORC_RANGE;
    for (int d = 0; d < D; ++d) counts[d] = 0;

    const uint16_t *new16 = (const uint16_t *)new_data;
    const uint32_t *new32 = (const uint32_t *)new_data;

    for (int64_t r = 0; r < R; ++r) {
        for (int64_t c = 0; c < C; ++c) {
            int64_t g = r * C + c;
            uint16_t nb = new_is_f32 ? orc_rne_bf16(new32[g]) : new16[g];
            if (nb == old_bits[g]) continue;            /* zero delta: not sent */
            int d_first, n_dest; int64_t local;
            rc = orc_shard_map(rule, R, C, n_sec, sec, D, r, c, &d_first, &n_dest, &local);
            if (rc) return rc;
            for (int d = d_first; d < d_first + n_dest; ++d) {
                int64_t k = counts[d];
                if (idx) {
                    if (k > 0 && (int64_t)idx[d][k - 1] >= local) return ORC_ORDER;
                    idx[d][k] = (int32_t)local;
                    val[d][k] = nb;
                }
                counts[d] = k + 1;
            }
        }
    }
    return ORC_OK;
}

/*
 * The same for a sender that holds only ITS OWN slice of the tensor (Sec. 4.2: the sharded
 * dimension gives per-rank slice ranges on BOTH sides; train and serve degrees may differ).
 * The sender is rank s of S under the same rule: old_slice / new_slice are shard s of the full
 * tensors (orc_dense_shard with degree S).  A replicated tensor is held by every sender; it is
 * sent by one of them only, which the caller names with sends_replicated != 0.
 *
 * Written over the FULL tensor's coordinates: element (r,c) is emitted by the sender whose slice
 * holds it (shard map with degree S gives the sender and the index inside its slice) to the
 * destination the shard map with degree D gives.  Entries come out in ascending (r,c).
 */
/*
 * Where the sender side keeps row r of a fused tensor when its layout is interleaved by head
 * group (the usual training-side layout of a fused QKV matrix: for each of G groups its query
 * rows, then its key rows, then its value rows), and the senders split that layout in S equal
 * row blocks, i.e. whole groups.  r is the row in the plain [Q;K;V] stacking.  Out: the sender
 * and the row inside its slice.
 */
static int src_row_groups(int64_t R, int n_sec, const int64_t *sec, int S, int G, int64_t r,
                          int *sender, int64_t *slice_row)
{
    if (G < 1 || G % S) return ORC_BAD_SHAPE;
    int64_t group_rows = 0;
    for (int j = 0; j < n_sec; ++j) {
        if (sec[j] % G) return ORC_BAD_SHAPE;
        group_rows += sec[j] / G;
    }
    int64_t first = 0, before = 0;      /* first row of r's section; rows of earlier sections per group */
    int j = 0;
    while (r >= first + sec[j]) {
        first += sec[j];
        before += sec[j] / G;
        ++j;
    }
    int64_t per = sec[j] / G;           /* rows of this section that belong to one group */
    int64_t g = (r - first) / per, w = (r - first) % per;
    int64_t src_row = g * group_rows + before + w;
    int64_t rows_per_sender = R / S;
    *sender = (int)(src_row / rows_per_sender);
    *slice_row = src_row % rows_per_sender;
    return ORC_OK;
}

/* src_groups = 0: the sender side stacks sections plainly, like the destination side;
 * src_groups = G > 0 (fused rows only): the sender side's layout is interleaved by G head groups. */
int orc_encode_tensor_src(const uint16_t *old_slice, const void *new_slice, int new_is_f32,
                          int rule, int64_t R, int64_t C, int n_sec, const int64_t *sec,
                          int D, int S, int s, int sends_replicated, int src_groups,
                          int64_t *counts, int32_t *const *idx, uint16_t *const *val)
{
    if (src_groups != 0 && rule != ORC_FUSED_ROWS) return ORC_BAD_SHAPE;
    int rc = check_shape(rule, R, C, n_sec, sec, D);
    if (rc) return rc;
    rc = check_shape(rule, R, C, n_sec, sec, S);
    if (rc) return rc;
    if (s < 0 || s >= S) return ORC_RANGE;
    if (orc_local_numel(rule, R, C, D) > (int64_t)INT32_MAX) return ORC_RANGE;
    for (int d = 0; d < D; ++d) counts[d] = 0;
    if (rule == ORC_REPLICATED && !sends_replicated) return ORC_OK;

    const uint16_t *new16 = (const uint16_t *)new_slice;
    const uint32_t *new32 = (const uint32_t *)new_slice;

    for (int64_t r = 0; r < R; ++r) {
        for (int64_t c = 0; c < C; ++c) {
            int s_first, n_src; int64_t sl;
            if (src_groups) {
                int64_t row;
                rc = src_row_groups(R, n_sec, sec, S, src_groups, r, &s_first, &row);
                n_src = 1;
                sl = row * C + c;
            } else {
                rc = orc_shard_map(rule, R, C, n_sec, sec, S, r, c, &s_first, &n_src, &sl);
            }
            if (rc) return rc;
            if (s < s_first || s >= s_first + n_src) continue;      /* another sender's element */
            uint16_t nb = new_is_f32 ? orc_rne_bf16(new32[sl]) : new16[sl];
            if (nb == old_slice[sl]) continue;
            int d_first, n_dest; int64_t local;
            rc = orc_shard_map(rule, R, C, n_sec, sec, D, r, c, &d_first, &n_dest, &local);
            if (rc) return rc;
            for (int d = d_first; d < d_first + n_dest; ++d) {
                int64_t k = counts[d];
                if (idx) {
                    if (k > 0 && (int64_t)idx[d][k - 1] >= local) return ORC_ORDER;
                    idx[d][k] = (int32_t)local;
                    val[d][k] = nb;
                }
                counts[d] = k + 1;
            }
        }
    }
    return ORC_OK;
}

/*
 * Pipeline stages (Sec. 4.2, "Shard-aware Weight Transfer": tensor AND pipeline
 * parallelism on both sides, e.g. TP8 x PP2 feeding TP4).  The paper names no
 * split; the reading taken is the uniform one: the n_layers decoder layers go
 * to the pp stages in consecutive groups of n_layers / pp, the tensors in
 * front of the layers (layer = ORC_LAYER_FIRST: the embedding) stay with the
 * first stage and those behind them (ORC_LAYER_LAST: final norm, head) with
 * the last.  Returns the stage, or -1 for arguments outside that reading.
 */
enum { ORC_LAYER_FIRST = -1, ORC_LAYER_LAST = -2 };
int orc_stage_of(int layer, int n_layers, int pp)
{
    if (pp < 1) return -1;
    if (layer == ORC_LAYER_FIRST) return 0;
    if (layer == ORC_LAYER_LAST) return pp - 1;
    if (n_layers < 1 || n_layers % pp != 0 || layer < 0 || layer >= n_layers) return -1;
    int group = n_layers / pp;
    for (int stage = 0; stage < pp; ++stage)         /* the group whose layer range holds `layer` */
        if (stage * group <= layer && layer < (stage + 1) * group) return stage;
    return -1;
}

/*
 * Sparse-to-dense (App. F "S2D"): put each entry's value at its local index
 * of the receiver's resident copy.  Nothing else is touched.
 */
int orc_apply(const int32_t *idx, const uint16_t *val, int64_t count,
              uint16_t *dst, int64_t dst_numel)
{
    for (int64_t k = 0; k < count; ++k) {
        if (idx[k] < 0 || (int64_t)idx[k] >= dst_numel) return ORC_RANGE;
        dst[idx[k]] = val[k];
    }
    return ORC_OK;
}

/*
 * Arithmetic payload (Sec. 4.2 states the update as W_t = W_{t-1} + dW_t; this is the variant
 * that takes it literally).  bf16 arithmetic rounds, so an entry carries the rounded difference
 * only where adding it back reproduces the new pattern; every other entry falls back to carrying
 * the new pattern itself and says so in the sign bit of its index.  With that escape the variant
 * stays lossless for every pair of bit patterns.  (A reading: the paper gives no element format.)
 *
 * The value of a bf16 pattern as a double (exact: a double holds every bf16 value).
 */
#include <math.h>
#include <string.h>

static double bf16_value(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * The bf16 pattern nearest to x, ties to the even significand, by the definition of the format:
 * 8 significant bits, exponents 2^-126 .. 2^127, below that fixed steps of 2^-133, beyond the
 * largest finite value (after rounding) infinity.  NaN gives the default NaN 0x7FC0.
 */
uint16_t orc_bf16_nearest(double x)
{
    if (isnan(x)) return 0x7FC0u;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                  /* a = m * 2^e, 0.5 <= m < 1  ->  leading bit 2^(e-1) */
    int lead = e - 1;
    if (lead < -126) lead = -126;        /* subnormal range: the step stays 2^-133            */
    double step = ldexp(1.0, lead - 7);  /* spacing of bf16 values in this binade             */
    double n = rint(a / step);           /* a power-of-two scaling is exact; rint: ties to even
                                            (the default rounding mode is never changed here)  */
    double r = n * step;                 /* exact: at most 9 significant bits                  */
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)r;                  /* exact                                              */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

/* correctly rounded bf16 sum and difference of two bf16 patterns.  The double result is exact
 * unless the operands' exponents are more than 40 binades apart, and then it differs from the
 * larger operand by far less than a quarter of a bf16 step, so rounding it again cannot land on
 * the other side of a tie. */
uint16_t orc_bf16_add(uint16_t a, uint16_t b) { return orc_bf16_nearest(bf16_value(a) + bf16_value(b)); }
uint16_t orc_bf16_sub(uint16_t a, uint16_t b) { return orc_bf16_nearest(bf16_value(a) - bf16_value(b)); }

/*
 * One entry: *val = the rounded difference and 0 is returned if the difference is a number and
 * old + difference rounds back to exactly the new pattern; otherwise *val = the new pattern and
 * 1 is returned (escape).
 */
int orc_arith_payload(uint16_t old_bits, uint16_t new_bits, uint16_t *val)
{
    uint16_t d = orc_bf16_sub(new_bits, old_bits);
    int d_is_nan = (d & 0x7FFFu) > 0x7F80u;
    if (!d_is_nan && orc_bf16_add(old_bits, d) == new_bits) {
        *val = d;
        return 0;
    }
    *val = new_bits;
    return 1;
}

/*
 * Turn the entries of one (tensor, shard) segment from "new pattern" payloads into arithmetic
 * ones, in place.  old_local is the receiver's resident copy W_{t-1} of that shard (the value the
 * receiver will add to).  An escaped entry gets bit 31 of its index set.
 */
int orc_arith_from_overwrite(int32_t *idx, uint16_t *val, int64_t count,
                             const uint16_t *old_local, int64_t numel)
{
    for (int64_t k = 0; k < count; ++k) {
        if (idx[k] < 0 || (int64_t)idx[k] >= numel) return ORC_RANGE;
        uint16_t v;
        int esc = orc_arith_payload(old_local[idx[k]], val[k], &v);
        val[k] = v;
        if (esc) idx[k] = (int32_t)((uint32_t)idx[k] | 0x80000000u);
    }
    return ORC_OK;
}

/* Sparse-to-dense for arithmetic entries: add (rounded), or overwrite where the entry says so. */
int orc_apply_arith(const int32_t *idx, const uint16_t *val, int64_t count,
                    uint16_t *dst, int64_t dst_numel)
{
    for (int64_t k = 0; k < count; ++k) {
        int64_t i = (int64_t)((uint32_t)idx[k] & 0x7FFFFFFFu);
        if (i >= dst_numel) return ORC_RANGE;
        if (idx[k] < 0) dst[i] = val[k];
        else dst[i] = orc_bf16_add(dst[i], val[k]);
    }
    return ORC_OK;
}

/*
 * Dense path (Sec. 4.2 "Shard-aware" without sparsity): shard d's local copy
 * of the full tensor, written out element by element through the shard map.
 */
int orc_dense_shard(const uint16_t *full, int rule, int64_t R, int64_t C, int n_sec,
                    const int64_t *sec, int D, int d, uint16_t *dst)
{
    int rc = check_shape(rule, R, C, n_sec, sec, D);
    if (rc) return rc;
    if (d < 0 || d >= D) return ORC_RANGE;
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t c = 0; c < C; ++c) {
            int d_first, n_dest; int64_t local;
            rc = orc_shard_map(rule, R, C, n_sec, sec, D, r, c, &d_first, &n_dest, &local);
            if (rc) return rc;
            if (d >= d_first && d < d_first + n_dest) dst[local] = full[r * C + c];
        }
    }
    return ORC_OK;
}
