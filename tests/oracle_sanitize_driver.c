/*
 * Hand cases for every function of oracle/flexshard_oracle.c, meant to be compiled together with
 * it under -fsanitize=address,undefined (tests/test_oracle_sanitized.py does that): the expected
 * values below are computed by hand, and any out-of-bounds access, use after free, signed overflow
 * or misaligned access inside the oracle aborts the run.  Exact-size heap buffers everywhere, so
 * that an access one element past an array is seen.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int64_t num_samples, B;
    int32_t U, W, dp_multiplier, granule;
    int64_t a2a_global, a2a_intra, ar_global, ar_cross;
} tier_params_t;

int oracle_route_bucketize(const int64_t*, const int64_t*, int32_t, int32_t, const int64_t*, const uint32_t*, int64_t,
                           int32_t, int32_t, int32_t, int64_t*, int64_t*, int32_t*, int64_t*, int32_t*);
int oracle_seq_gather_fwd(const void*, int64_t, int32_t, int, const int64_t*, const int32_t*, int64_t, int64_t, void*,
                          int64_t, int32_t*);
int oracle_seq_gather_send(const void*, int64_t, int32_t, int, const int64_t*, int64_t, int64_t, void*, int32_t*);
int oracle_seq_unbucketize(const void*, int32_t, int, const int32_t*, int64_t, int64_t, void*, int64_t, int32_t*);
int oracle_replica_build(const void*, int64_t, int32_t, int, const int64_t*, int64_t, void*, int32_t*, int32_t*);
int oracle_seq_gather_fwd_replica(const void*, int64_t, int32_t, int, const void*, int64_t, const int32_t*,
                                  const int64_t*, const int32_t*, int64_t, int64_t, void*, int64_t, int32_t*);
int oracle_replica_tag_slots(uint32_t*, int64_t, const int32_t*, int32_t*);
int oracle_lookup_slots(const uint32_t*, int64_t, const int64_t*, int64_t, int64_t, int32_t*, int32_t*);
int oracle_seq_gather_fwd_slots(const void*, int64_t, int32_t, int, const void*, int64_t, const int64_t*, const int32_t*,
                                const int32_t*, int64_t, int64_t, void*, int64_t, int32_t*);
int oracle_seq_grad_bwd(const void*, int64_t, int32_t, int, const int64_t*, const int32_t*, int64_t, int64_t, int64_t,
                        int32_t, int64_t*, float*, double*, int64_t, int64_t*, int32_t*);
int oracle_plan_replication(const int64_t*, const int64_t*, int32_t, int32_t, const int64_t*, int64_t, int64_t,
                            uint32_t*, int32_t, int64_t, int64_t, int64_t*, int64_t*, uint32_t*, int32_t*);
int oracle_plan_tiers(const uint32_t*, int64_t, const tier_params_t*, int32_t, int64_t*, int64_t, int64_t*, uint32_t*,
                      int32_t*);
int oracle_sparse_update(void*, int64_t, int32_t, int, const int64_t*, const float*, int64_t, int32_t, float, float,
                         float*, void*, const int32_t*, int64_t, int32_t*);

static int failures = 0;
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

static void* dup_bytes(const void* src, size_t bytes)
{
    void* p = malloc(bytes ? bytes : 1);
    if (bytes) memcpy(p, src, bytes);
    return p;
}
#define HEAP(type, name, ...)                              \
    const type name##_init[] = {__VA_ARGS__};              \
    type* name = (type*)dup_bytes(name##_init, sizeof(name##_init))

#define TIER(t, owner) (((uint32_t)(t) << 30) | (uint32_t)(owner))

static void route_and_gather(void)
{
    /* 2 tables x 2 samples, E = 3 rows each; U = 4 buckets in groups of W = 2, self = 3 (group base 2) */
    HEAP(int64_t, ids, 0, 2, 1, 1, 0, 2);
    HEAP(int64_t, offsets, 0, 2, 3, 3, 6);               /* segment 2 is empty */
    HEAP(int64_t, row_base, 0, 3, 6);
    HEAP(uint32_t, placement, TIER(0, 9), TIER(1, 1), TIER(2, 0), TIER(2, 1), TIER(1, 0), TIER(2, 3));
    int64_t* bo = malloc(5 * sizeof(int64_t));
    int64_t* rows = malloc(6 * sizeof(int64_t));
    int32_t* pos = malloc(6 * sizeof(int32_t));
    int64_t* tiers = malloc(3 * sizeof(int64_t));
    int32_t st = 0;
    /* global rows 0, 2, 1 | 4, 3, 5 -> destinations 3, 0, 3 | 2, 1, 3 */
    CHECK(oracle_route_bucketize(ids, offsets, 2, 2, row_base, placement, 6, 4, 2, 3, bo, rows, pos, tiers, &st) == 0);
    CHECK(st == 0);
    const int64_t bo_want[] = {0, 1, 2, 3, 6}, rows_want[] = {2, 3, 4, 0, 1, 5}, tiers_want[] = {1, 2, 3};
    const int32_t pos_want[] = {1, 4, 3, 0, 2, 5};
    CHECK(memcmp(bo, bo_want, sizeof bo_want) == 0 && memcmp(rows, rows_want, sizeof rows_want) == 0);
    CHECK(memcmp(pos, pos_want, sizeof pos_want) == 0 && memcmp(tiers, tiers_want, sizeof tiers_want) == 0);
    /* faults stay in bounds: an id past its table, a bad owner, tier 3, bad offsets */
    ids[1] = 7; placement[3] = TIER(2, 4); placement[4] = TIER(3, 0);
    st = 0;
    CHECK(oracle_route_bucketize(ids, offsets, 2, 2, row_base, placement, 6, 4, 2, 3, bo, rows, pos, tiers, &st) == 0);
    CHECK(st == (1 | 4) && bo[4] == 6);
    offsets[1] = 5;
    st = 0;
    CHECK(oracle_route_bucketize(ids, offsets, 2, 2, row_base, placement, 6, 4, 2, 3, bo, rows, pos, tiers, &st) == 0);
    CHECK(st & 2);

    /* gather: 6 table rows of 4 floats, row r holds 10 r + column */
    float* w = malloc(6 * 4 * sizeof(float));
    for (int r = 0; r < 6; ++r) for (int d = 0; d < 4; ++d) w[r * 4 + d] = (float)(10 * r + d);
    float* out = malloc(6 * 4 * sizeof(float));
    for (int i = 0; i < 24; ++i) out[i] = -1.0f;
    st = 0;
    CHECK(oracle_seq_gather_fwd(w, 6, 4, 0, rows_want, pos_want, 1, 5, out, 6, &st) == 0 && st == 0);
    CHECK(out[4 * 4 + 1] == 31.0f && out[3 * 4] == 40.0f && out[0] == 0.0f && out[2 * 4 + 3] == 13.0f);
    CHECK(out[1 * 4] == -1.0f && out[5 * 4] == -1.0f);                 /* j = 0 and j = 5 are outside [1, 5) */
    /* the two halves either side of the exchange compose to the same rows */
    float* send = malloc(4 * 4 * sizeof(float));
    float* out2 = malloc(6 * 4 * sizeof(float));
    for (int i = 0; i < 24; ++i) out2[i] = -1.0f;
    CHECK(oracle_seq_gather_send(w, 6, 4, 0, rows_want, 1, 5, send, &st) == 0);
    CHECK(oracle_seq_unbucketize(send, 4, 0, pos_want, 1, 5, out2, 6, &st) == 0 && st == 0);
    CHECK(memcmp(out, out2, 24 * sizeof(float)) == 0);
    /* replica store of rows {4, 1, 4}: slot of row 4 is the first one that names it */
    HEAP(int64_t, sel, 4, 1, 4);
    float* store = malloc(3 * 4 * sizeof(float));
    int32_t* slots = malloc(6 * sizeof(int32_t));
    CHECK(oracle_replica_build(w, 6, 4, 0, sel, 3, store, slots, &st) == 0 && st == 0);
    CHECK(slots[4] == 0 && slots[1] == 1 && slots[0] == -1 && store[0] == 40.0f && store[4] == 10.0f);
    store[1] = 77.0f;                                                   /* shows which source a lookup read */
    float* out3 = malloc(6 * 4 * sizeof(float));
    CHECK(oracle_seq_gather_fwd_replica(w, 6, 4, 0, store, 3, slots, rows_want, pos_want, 0, 6, out3, 6, &st) == 0);
    CHECK(st == 0 && out3[3 * 4 + 1] == 77.0f && out3[4 * 4 + 1] == 31.0f);
    /* the slots handed over in the placement: all six rows replicated, rows 4 and 1 have a slot */
    HEAP(uint32_t, tagged, 9u, 9u, 9u, 9u, 9u, 0x80000001u);
    CHECK(oracle_replica_tag_slots(tagged, 6, slots, &st) == 0 && st == 0);
    CHECK(tagged[4] == 0u && tagged[1] == 1u && tagged[0] == 0x3FFFFFFFu && tagged[5] == 0x80000001u);
    int32_t* lslots = malloc(6 * sizeof(int32_t));
    CHECK(oracle_lookup_slots(tagged, 6, rows_want, 0, 6, lslots, &st) == 0 && st == 0);
    float* out4 = malloc(6 * 4 * sizeof(float));
    CHECK(oracle_seq_gather_fwd_slots(w, 6, 4, 0, store, 3, rows_want, lslots, pos_want, 0, 6, out4, 6, &st) == 0 && st == 0);
    CHECK(memcmp(out3, out4, 24 * sizeof(float)) == 0);               /* what the gather with the slot map wrote (row 5 is not tier 0, and has no slot) */
    free(tagged); free(lslots); free(out4);
    /* a row and a position out of range are skipped and flagged */
    HEAP(int64_t, bad_rows, 9, 1);
    HEAP(int32_t, bad_pos, 0, 6);
    st = 0;
    CHECK(oracle_seq_gather_fwd(w, 6, 4, 0, bad_rows, bad_pos, 0, 2, out, 6, &st) == 0 && st == 1);
    free(ids); free(offsets); free(row_base); free(placement); free(bo); free(rows); free(pos); free(tiers);
    free(w); free(out); free(send); free(out2); free(sel); free(store); free(slots); free(out3); free(bad_rows); free(bad_pos);
}

static void backward(void)
{
    /* one run of six at k = 0, tile 4: partials (2^24 + 1 + 1 + 1) = 2^24 and (1 + 1) = 2 */
    const float big = 16777216.0f;
    float* g = malloc(6 * 4 * sizeof(float));
    for (int i = 0; i < 6; ++i) for (int d = 0; d < 4; ++d) g[i * 4 + d] = (i == 0 ? big : 1.0f) * (d == 1 ? -1.0f : 1.0f);
    HEAP(int64_t, rows, 5, 5, 5, 5, 5, 5);
    HEAP(int32_t, pos, 0, 1, 2, 3, 4, 5);
    int64_t* uniq = malloc(1 * sizeof(int64_t));
    float* rg = malloc(4 * sizeof(float));
    double* rg64 = malloc(4 * sizeof(double));
    int64_t nu = -1;
    int32_t st = 0;
    CHECK(oracle_seq_grad_bwd(g, 6, 4, 0, rows, pos, 0, 6, 10, 4, uniq, rg, rg64, 1, &nu, &st) == 0);
    CHECK(st == 0 && nu == 1 && uniq[0] == 5 && rg[0] == big + 2.0f && rg[1] == -(big + 2.0f) && rg64[0] == 16777221.0);
    CHECK(oracle_seq_grad_bwd(g, 6, 4, 0, rows, pos, 0, 6, 10, 8, uniq, rg, rg64, 1, &nu, &st) == 0 && rg[0] == big);
    /* more distinct rows than capacity: the count is still exact, nothing is written past the capacity */
    rows[3] = 7; rows[5] = 9;
    CHECK(oracle_seq_grad_bwd(g, 6, 4, 0, rows, pos, 0, 6, 10, 256, uniq, rg, rg64, 1, &nu, &st) == 0);
    CHECK(nu == 3 && st == 16 && uniq[0] == 5);
    /* 16-bit inputs: 1.5 as fp16 (0x3E00) and bf16 (0x3FC0), two lookups of one row */
    uint16_t* h = malloc(2 * 8 * sizeof(uint16_t));
    for (int i = 0; i < 16; ++i) h[i] = 0x3E00;
    HEAP(int64_t, rows2, 3, 3);
    float* rg8 = malloc(8 * sizeof(float));
    st = 0;
    CHECK(oracle_seq_grad_bwd(h, 2, 8, 1, rows2, pos, 0, 2, 4, 256, uniq, rg8, NULL, 1, &nu, &st) == 0 && rg8[7] == 3.0f);
    for (int i = 0; i < 16; ++i) h[i] = 0x3FC0;
    CHECK(oracle_seq_grad_bwd(h, 2, 8, 2, rows2, pos, 0, 2, 4, 256, uniq, rg8, NULL, 1, &nu, &st) == 0 && rg8[0] == 3.0f);
    CHECK(st == 0 && nu == 1);
    free(g); free(rows); free(pos); free(uniq); free(rg); free(rg64); free(h); free(rows2); free(rg8);
}

static void plan(void)
{
    /* one table of 5 rows, one sample: appearances 2: 3x, 0: 2x, 4: 2x, 1: 1x, 3: 0x */
    HEAP(int64_t, ids, 2, 0, 4, 2, 1, 0, 2, 4);
    HEAP(int64_t, offsets, 0, 8);
    HEAP(int64_t, row_base, 0, 5);
    uint32_t* counts = calloc(5, sizeof(uint32_t));
    HEAP(uint32_t, placement, TIER(2, 0), TIER(2, 1), TIER(2, 0), TIER(2, 1), TIER(2, 0));
    int64_t* sel = malloc(3 * sizeof(int64_t));
    int64_t k = -1;
    int32_t st = 0;
    CHECK(oracle_plan_replication(ids, offsets, 1, 1, row_base, 8, 5, counts, 1 | 2 | 4, 3 * 64, 64, sel, &k, placement,
                                  &st) == 0);
    CHECK(st == 0 && k == 3 && sel[0] == 2 && sel[1] == 0 && sel[2] == 4);
    CHECK(counts[2] == 3 && counts[3] == 0 && placement[2] == TIER(0, 0) && placement[1] == TIER(2, 1));
    /* a budget larger than the rows that appeared: zero-count rows only with ALLOW_ZERO; saturation */
    int64_t* sel5 = malloc(5 * sizeof(int64_t));
    CHECK(oracle_plan_replication(NULL, NULL, 1, 1, NULL, 0, 5, counts, 2, 99 * 64, 64, sel5, &k, NULL, &st) == 0 && k == 4);
    CHECK(oracle_plan_replication(NULL, NULL, 1, 1, NULL, 0, 5, counts, 2 | 8, 99 * 64, 64, sel5, &k, NULL, &st) == 0);
    CHECK(k == 5 && sel5[4] == 3);
    counts[2] = 0xFFFFFFFEu;
    CHECK(oracle_plan_replication(ids, offsets, 1, 1, row_base, 8, 5, counts, 1, 0, 1, NULL, NULL, NULL, &st) == 0);
    CHECK(counts[2] == 0xFFFFFFFFu && st == 8);

    /* tier planner: B = 4, U = 2, W = 1, dp = 1, S = 8 samples.  DP memory term of a row with count c, times U S:
     * (dp U - 1) S - U B c = 8 - 8 c: <= 0 from c = 1 on, so A = every candidate; the summed terms stay <= 0: B too */
    HEAP(uint32_t, c2, 5, 0, 3, 1, 1, 0);
    tier_params_t p = {8, 4, 2, 1, 1, 1, 1, 6, 3, 2};
    int64_t* cuts = malloc(10 * sizeof(int64_t));
    int64_t* sorted = malloc(6 * sizeof(int64_t));
    uint32_t* pl = calloc(6, sizeof(uint32_t));
    for (int i = 0; i < 6; ++i) pl[i] = TIER(2, (uint32_t)i % 2);
    CHECK(oracle_plan_tiers(c2, 6, &p, 2, sorted, 6, cuts, pl, &st) == 0);
    CHECK(cuts[0] == 4 && cuts[1] == 4 && cuts[2] == 4 && cuts[5] == 4 && cuts[6] == 0 && cuts[7] == 10 && cuts[8] == 10);
    CHECK(sorted[0] == 0 && sorted[1] == 2 && sorted[2] == 3 && sorted[3] == 4 && pl[0] == TIER(0, 0) && pl[1] == TIER(2, 1));
    CHECK(oracle_plan_tiers(c2, 6, &p, 3, sorted, 2, cuts, NULL, &st) == 0 && cuts[5] == 4);
    free(ids); free(offsets); free(row_base); free(counts); free(placement); free(sel); free(sel5);
    free(c2); free(cuts); free(sorted); free(pl);
}

static void update(void)
{
    /* SGD with lr = 0.5 on rows 1 and 3 of a 4 x 4 float table, mirrored into a one-row store for row 3 */
    float* w = malloc(16 * sizeof(float));
    for (int i = 0; i < 16; ++i) w[i] = 1.0f;
    HEAP(int64_t, rows, 1, 3);
    HEAP(float, grads, 2, 2, 2, 2, -4, -4, -4, -4);
    HEAP(int32_t, slots, -1, -1, -1, 0);
    float* store = calloc(4, sizeof(float));
    int32_t st = 0;
    CHECK(oracle_sparse_update(w, 4, 4, 0, rows, grads, 2, 0, 0.5f, 0.0f, NULL, store, slots, 1, &st) == 0 && st == 0);
    CHECK(w[4] == 0.0f && w[12] == 3.0f && w[0] == 1.0f && store[3] == 3.0f);
    /* row-wise Adagrad: state += mean(g^2) = 4; w -= lr g / (sqrt(4) + 0) = 1 - 0.5 * 2 / 2 */
    float* state = calloc(4, sizeof(float));
    for (int i = 0; i < 16; ++i) w[i] = 1.0f;
    CHECK(oracle_sparse_update(w, 4, 4, 0, rows, grads, 1, 1, 0.5f, 0.0f, state, NULL, NULL, 0, &st) == 0);
    CHECK(state[1] == 4.0f && w[4] == 0.5f && w[12] == 1.0f);
    /* element-wise Adagrad on a 16-bit table (bf16 1.0 = 0x3F80): state[r, d] += 4, w = 1 - 0.5 * 2 / 2 = 0.5 = 0x3F00 */
    uint16_t* wb = malloc(4 * 8 * sizeof(uint16_t));
    for (int i = 0; i < 32; ++i) wb[i] = 0x3F80;
    float* g8 = malloc(8 * sizeof(float));
    for (int i = 0; i < 8; ++i) g8[i] = 2.0f;
    float* state2 = calloc(32, sizeof(float));
    CHECK(oracle_sparse_update(wb, 4, 8, 2, rows, g8, 1, 2, 0.5f, 0.0f, state2, NULL, NULL, 0, &st) == 0);
    CHECK(wb[8] == 0x3F00 && wb[15] == 0x3F00 && wb[0] == 0x3F80 && state2[8] == 4.0f && st == 0);
    /* a row out of range is skipped and flagged */
    rows[0] = 4;
    CHECK(oracle_sparse_update(w, 4, 4, 0, rows, grads, 1, 0, 0.5f, 0.0f, NULL, NULL, NULL, 0, &st) == 0 && st == 1);
    free(w); free(rows); free(grads); free(slots); free(store); free(state); free(wb); free(g8); free(state2);
}

int main(void)
{
    route_and_gather();
    backward();
    plan();
    update();
    if (failures == 0) printf("oracle hand cases ok\n");
    return failures == 0 ? 0 : 1;
}
