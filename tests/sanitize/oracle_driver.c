/* Runs every entry point of the CPU oracle on seeded chains; built by
 * tests/test_sanitizers.py together with oracle/ckpt_oracle.c under
 * AddressSanitizer and UndefinedBehaviorSanitizer (signed overflow included),
 * so that an out-of-bounds access or a wrapping 64-bit sum in the reference
 * itself fails the CPU test suite.  Prints a checksum; exits non-zero on any
 * inconsistency between the oracle's own algorithms. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef int64_t i64;
i64 orc_peak_static(const i64 *, const uint8_t *, int);
i64 orc_peak_dynamic(const i64 *, const uint8_t *, int);
i64 orc_sim_static(const i64 *, const uint8_t *, int);
i64 orc_sim_dynamic(const i64 *, const uint8_t *, int);
void orc_timeline(const i64 *, const uint8_t *, int, int, i64 *);
void orc_select_baseline(int, int, uint8_t *);
i64 orc_brute(const i64 *, int, int, i64 *, i64 *);
i64 orc_num_budgets(int);
void orc_budgets(const i64 *, int, i64 *);
i64 orc_solve_static_literal(const i64 *, int, uint8_t *, i64 *);
i64 orc_solve_static_range(const i64 *, int, uint8_t *, i64 *, i64, i64);
i64 orc_solve_static(const i64 *, int, uint8_t *, i64 *);
i64 orc_static_cs(const i64 *, int, i64);
i64 orc_solve_dynamic(const i64 *, int, uint8_t *, i64 *);
i64 orc_solve_dynamic_literal(const i64 *, int, i64 *);
void orc_batch_peak(const i64 *, const uint8_t *, i64, int, int, i64 *);
void orc_batch_timeline(const i64 *, const uint8_t *, i64, int, int, i64 *);
void orc_batch_solve_dynamic(const i64 *, i64, int, uint8_t *, i64 *);
void orc_batch_solve_static(const i64 *, i64, int, uint8_t *, i64 *, i64 *);
void orc_ragged_peak(const i64 *, const uint8_t *, const i64 *, i64, int, i64 *);
void orc_ragged_timeline(const i64 *, const uint8_t *, const i64 *, i64, int, i64 *);
void orc_ragged_solve_dynamic(const i64 *, const i64 *, i64, uint8_t *, i64 *);
void orc_ragged_solve_static(const i64 *, const i64 *, i64, uint8_t *, i64 *, i64 *);
void orc_static_cs_list(const i64 *, int, const i64 *, i64, i64 *);

static uint64_t state = 0x2545F4914F6CDD1DULL;
static uint64_t next_u64(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return state;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "oracle_driver: %s failed at line %d\n", #c, __LINE__); exit(1); } } while (0)

static void one_chain(int n, int kind, uint64_t *sum)
{
    i64 *d = malloc(sizeof(i64) * (n + 1));
    uint8_t *mask = malloc(n + 1), *m2 = malloc(n + 1);
    i64 *M = malloc(sizeof(i64) * (n + 1)), *tl = malloc(sizeof(i64) * (2 * n + 2));
    for (int k = 0; k <= n; k++) {
        uint64_t r = next_u64();
        /* kind 0: tiny sizes with ties; 1: 4 KiB multiples; 2: sizes near 2^55, so that
         * sum(d) + max(d) stays just inside 63 bits for the longest chains here */
        d[k] = kind == 0 ? (i64)(r % 3 + 1) : kind == 1 ? (i64)(r % 32513 + 256) * 4096 : (i64)(r >> 9) + 1;
        mask[k] = (k == 0 || k == n) ? 1 : (uint8_t)((next_u64() & 3) == 0);
    }
    for (int obj = 0; obj < 2; obj++) {
        i64 p = obj ? orc_peak_dynamic(d, mask, n) : orc_peak_static(d, mask, n);
        i64 q = obj ? orc_sim_dynamic(d, mask, n) : orc_sim_static(d, mask, n);
        CHECK(p == q);
        orc_timeline(d, mask, n, obj, tl);
        i64 top = 0;
        for (int t = n + 1; t <= 2 * n; t++) top = tl[t] > top ? tl[t] : top;
        CHECK(top == p);
        *sum += (uint64_t)p;
    }
    i64 s1 = 0, s2 = 0, s3 = 0;
    i64 v1 = orc_solve_static(d, n, m2, &s1);
    CHECK(orc_peak_static(d, m2, n) == v1);
    if (n <= 40) {
        i64 v2 = orc_solve_static_literal(d, n, mask, &s2);
        CHECK(v1 == v2 && s1 == s2 && memcmp(mask, m2, n + 1) == 0);
    }
    i64 K = orc_num_budgets(n);
    i64 va = orc_solve_static_range(d, n, NULL, &s2, 0, K / 2);
    i64 vb = orc_solve_static_range(d, n, NULL, &s3, K / 2, K);
    CHECK((va < vb ? va : vb) == v1);
    CHECK(s1 + orc_static_cs(d, n, s1) == v1);
    i64 w1 = orc_solve_dynamic(d, n, m2, M);
    CHECK(orc_peak_dynamic(d, m2, n) == w1 && M[0] == w1 && M[n] == d[n]);
    if (n <= 60) CHECK(orc_solve_dynamic_literal(d, n, M) == w1);
    if (n <= 14) {
        i64 cnt, seg;
        CHECK(orc_brute(d, n, 0, &cnt, &seg) == v1 && seg == s1);
        CHECK(orc_brute(d, n, 1, &cnt, &seg) == w1);
    }
    for (int kind2 = 0; kind2 < 3; kind2++) {
        orc_select_baseline(n, kind2, mask);
        CHECK(mask[0] == 1 && mask[n] == 1);
        *sum += (uint64_t)orc_peak_dynamic(d, mask, n);
    }
    *sum += (uint64_t)v1 + (uint64_t)w1;
    free(d); free(mask); free(m2); free(M); free(tl);
}

int main(void)
{
    uint64_t sum = 0;   /* a checksum: wraps on purpose */
    const int lengths[] = {1, 2, 3, 7, 12, 14, 33, 64, 100, 150};
    for (int kind = 0; kind < 3; kind++)
        for (unsigned t = 0; t < sizeof lengths / sizeof *lengths; t++) one_chain(lengths[t], kind, &sum);
    /* batches and ragged batches */
    enum { B = 37, N = 19 };
    i64 *d = malloc(sizeof(i64) * B * (N + 1)), *peak = malloc(sizeof(i64) * B), *s = malloc(sizeof(i64) * B);
    i64 *off = malloc(sizeof(i64) * (B + 1)), *tl = malloc(sizeof(i64) * 2 * B * (N + 1));
    uint8_t *mask = malloc(B * (N + 1));
    for (int k = 0; k < B * (N + 1); k++) d[k] = (i64)(next_u64() % 1000 + 1);
    orc_batch_solve_dynamic(d, B, N, mask, peak);
    orc_batch_peak(d, mask, B, N, 1, s);
    CHECK(memcmp(peak, s, sizeof(i64) * B) == 0);
    orc_batch_timeline(d, mask, B, N, 1, tl);
    orc_batch_solve_static(d, B, N, mask, peak, s);
    orc_batch_peak(d, mask, B, N, 0, s);
    CHECK(memcmp(peak, s, sizeof(i64) * B) == 0);
    /* the same storage cut into chains of lengths 1, 2, 3, .. */
    int c = 0;
    off[0] = 0;
    while (off[c] + c + 2 <= (i64)B * (N + 1) && c < B) { off[c + 1] = off[c] + c + 2; c++; }
    orc_ragged_solve_dynamic(d, off, c, mask, peak);
    orc_ragged_peak(d, mask, off, c, 1, s);
    CHECK(memcmp(peak, s, sizeof(i64) * c) == 0);
    orc_ragged_timeline(d, mask, off, c, 1, tl);
    orc_ragged_solve_static(d, off, c, mask, peak, s);
    i64 *cs = malloc(sizeof(i64) * c);
    orc_ragged_peak(d, mask, off, c, 0, cs);
    CHECK(memcmp(peak, cs, sizeof(i64) * c) == 0);
    for (int k = 0; k < c; k++) sum += (uint64_t)peak[k];
    free(d); free(peak); free(s); free(off); free(tl); free(mask); free(cs);
    printf("oracle_driver ok %llu\n", (unsigned long long)sum);
    return 0;
}
