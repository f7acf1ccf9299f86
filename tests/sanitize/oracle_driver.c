/*
 * Runs the CPU oracle's routines on small seeded inputs under AddressSanitizer and
 * UndefinedBehaviorSanitizer (built and started by tests/test_host_sanitizers.py).  Exit status 0
 * and the last line "ok" mean that no routine read or wrote out of bounds, overflowed a signed
 * integer or shifted out of range on these inputs, and that the round trip still holds.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t orc_local_numel(int rule, int64_t R, int64_t C, int D);
int orc_encode_tensor(const uint16_t *old_bits, const void *new_data, int new_is_f32, int rule, int64_t R, int64_t C,
                      int n_sec, const int64_t *sec, int D, int64_t *counts, int32_t *const *idx, uint16_t *const *val);
int orc_encode_tensor_src(const uint16_t *old_slice, const void *new_slice, int new_is_f32, int rule, int64_t R,
                          int64_t C, int n_sec, const int64_t *sec, int D, int S, int s, int sends_replicated,
                          int src_groups, int64_t *counts, int32_t *const *idx, uint16_t *const *val);
int orc_apply(const int32_t *idx, const uint16_t *val, int64_t count, uint16_t *dst, int64_t dst_numel);
int orc_dense_shard(const uint16_t *full, int rule, int64_t R, int64_t C, int n_sec, const int64_t *sec, int D, int d,
                    uint16_t *dst);
uint16_t orc_rne_bf16(uint32_t u);
int orc_arith_from_overwrite(int32_t *idx, uint16_t *val, int64_t count, const uint16_t *old_local, int64_t numel);
int orc_apply_arith(const int32_t *idx, const uint16_t *val, int64_t count, uint16_t *dst, int64_t dst_numel);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (uint32_t)(state >> 16);
}

static void fail(const char *what, int rc)
{
    printf("FAILED: %s (%d)\n", what, rc);
    exit(1);
}

/* encode (plain and arithmetic), apply on the sliced old weights, compare with the sliced new ones */
static void one_case(int rule, int64_t R, int64_t C, int n_sec, const int64_t *sec, int D, int f32)
{
    int64_t n = R * C;
    uint16_t *old = malloc((size_t)(n ? n : 1) * 2), *new16 = malloc((size_t)(n ? n : 1) * 2);
    uint32_t *new32 = malloc((size_t)(n ? n : 1) * 4);
    for (int64_t i = 0; i < n; ++i) {
        old[i] = (uint16_t)rnd();
        uint16_t w = (rnd() % 3) ? old[i] : (uint16_t)rnd();
        new32[i] = ((uint32_t)w << 16) | ((rnd() % 4) ? 0u : (rnd() & 0xFFFFu));
        new16[i] = f32 ? orc_rne_bf16(new32[i]) : w;
    }
    const void *newp = f32 ? (const void *)new32 : (const void *)new16;
    int64_t counts[16];
    int rc = orc_encode_tensor(old, newp, f32, rule, R, C, n_sec, sec, D, counts, NULL, NULL);
    if (rc) fail("count", rc);
    int32_t *idx[16];
    uint16_t *val[16];
    for (int d = 0; d < D; ++d) {
        idx[d] = malloc((size_t)(counts[d] ? counts[d] : 1) * 4);
        val[d] = malloc((size_t)(counts[d] ? counts[d] : 1) * 2);
    }
    int64_t counts2[16];
    rc = orc_encode_tensor(old, newp, f32, rule, R, C, n_sec, sec, D, counts2, idx, val);
    if (rc) fail("fill", rc);
    int64_t ln = orc_local_numel(rule, R, C, D);
    for (int d = 0; d < D; ++d) {
        uint16_t *lo = malloc((size_t)(ln ? ln : 1) * 2), *lw = malloc((size_t)(ln ? ln : 1) * 2);
        uint16_t *keep = malloc((size_t)(ln ? ln : 1) * 2);
        if ((rc = orc_dense_shard(old, rule, R, C, n_sec, sec, D, d, lo))) fail("shard old", rc);
        if ((rc = orc_dense_shard(new16, rule, R, C, n_sec, sec, D, d, lw))) fail("shard new", rc);
        memcpy(keep, lo, (size_t)ln * 2);
        if ((rc = orc_apply(idx[d], val[d], counts[d], lo, ln))) fail("apply", rc);
        if (memcmp(lo, lw, (size_t)ln * 2)) fail("round trip", 0);
        /* the same entries with arithmetic payloads */
        if ((rc = orc_arith_from_overwrite(idx[d], val[d], counts[d], keep, ln))) fail("arith", rc);
        if ((rc = orc_apply_arith(idx[d], val[d], counts[d], keep, ln))) fail("apply arith", rc);
        if (memcmp(keep, lw, (size_t)ln * 2)) fail("arith round trip", 0);
        free(lo); free(lw); free(keep);
    }
    /* every sender of degree S emits its part; the counts add up */
    for (int S = 1; S <= 4; S *= 2) {
        if (rule == 1 && R % S) continue;
        if (rule == 2 && C % S) continue;
        int ok = 1;
        if (rule == 3) for (int j = 0; j < n_sec; ++j) if (sec[j] % S) ok = 0;
        if (!ok) continue;
        int64_t total[16] = {0};
        int64_t sn = orc_local_numel(rule, R, C, S);
        for (int s = 0; s < S; ++s) {
            uint16_t *so = malloc((size_t)(sn ? sn : 1) * 2), *sw = malloc((size_t)(sn ? sn : 1) * 2);
            if ((rc = orc_dense_shard(old, rule, R, C, n_sec, sec, S, s, so))) fail("sender old", rc);
            if ((rc = orc_dense_shard(new16, rule, R, C, n_sec, sec, S, s, sw))) fail("sender new", rc);
            int64_t c[16];
            rc = orc_encode_tensor_src(so, sw, 0, rule, R, C, n_sec, sec, D, S, s, s == 0, 0, c, NULL, NULL);
            if (rc) fail("sender count", rc);
            for (int d = 0; d < D; ++d) total[d] += c[d];
            free(so); free(sw);
        }
        for (int d = 0; d < D; ++d) if (total[d] != counts[d]) fail("sender totals", d);
    }
    for (int d = 0; d < D; ++d) { free(idx[d]); free(val[d]); }
    free(old); free(new16); free(new32);
}

int main(void)
{
    const int64_t sec3[3] = {16, 8, 8}, sec2[2] = {12, 20}, sec1[1] = {8};
    for (int D = 1; D <= 8; D *= 2) {
        for (int f32 = 0; f32 < 2; ++f32) {
            one_case(0, 3, 41, 0, NULL, D, f32);
            one_case(0, 0, 7, 0, NULL, D, f32);
            one_case(1, 8 * D, 5, 0, NULL, D, f32);
            one_case(1, 0, 16, 0, NULL, D, f32);
            one_case(2, 7, 8 * D, 0, NULL, D, f32);
            one_case(2, 1, 3 * D, 0, NULL, D, f32);
            if (D <= 4) one_case(3, 32, 9, 3, sec3, D, f32);
            if (D <= 4) one_case(3, 32, 3, 2, sec2, D, f32);
            one_case(3, 8, 11, 1, sec1, D, f32);
        }
    }
    printf("ok\n");
    return 0;
}
