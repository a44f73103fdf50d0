/*
 * flexshard_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU statement of what the tiered
 * sequence-embedding lookup computes (FlexShard, arXiv 2301.02959), used only
 * by the tests, the smoke check and the benchmark's cpu_baseline leg.  It
 * shares no code, header or table with the HIP library: constants are
 * repeated here on purpose.  Build: gcc -O2 -ffp-contract=off (no fast-math),
 * so every float add below is one IEEE round-to-nearest-even operation.
 *
 * Every function takes host pointers and returns 0 or a host-fault code;
 * data faults are OR-ed into *status (may be NULL).
 *
 * Pins (tests/test_oracle_*.py): stable argsort / bincount / take / put / lexsort /
 * fp64 add.at reductions, brute force over all placements on tiny inputs,
 * hand-computed rounding cases for the summation order, invariants; for the tier
 * planner a whole-cost-curve brute force in exact fractions, closed forms and the
 * tier sizes and coverage columns the paper prints for its four models.
 * No function here is "parity unpinned".
 */
#include <stdint.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

enum { OK = 0, ERR_NULL = 1, ERR_SIZE = 2, ERR_DTYPE = 3, ERR_ALIGN = 4,
       ERR_WORKSPACE = 5, ERR_CONFIG = 6 };
enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };
enum { DEV_BAD_ID = 1, DEV_BAD_OFFSETS = 2, DEV_BAD_PLACEMENT = 4,
       DEV_COUNT_OVERFLOW = 8, DEV_UNIQUE_OVERFLOW = 16, DEV_POS_ORDER = 32 };
enum { PLAN_ACCUMULATE = 1, PLAN_SELECT = 2, PLAN_TAG = 4, PLAN_ALLOW_ZERO = 8 };

static void flag(int32_t* status, int32_t bit) { if (status) *status |= bit; }

/* Segments (Section 2: one variable-length id list per sample and feature):
 * offsets[0] = 0, non-decreasing, offsets[S] = n. */
static int offsets_ok(const int64_t* offsets, int64_t S, int64_t n)
{
    if (offsets[0] != 0 || offsets[S] != n) return 0;
    for (int64_t s = 0; s < S; ++s)
        if (offsets[s] > offsets[s + 1]) return 0;
    return 1;
}

/*
 * Destination of one lookup (Section 3.1: a replicated row is looked up on
 * the GPU that holds the sample, a row-wise sharded row on its owner;
 * Section 4.4: a Flex row is sharded inside a node and that shard is
 * replicated on every node, so the requester's own group serves it).
 * Returns the bucket and writes the tier the lookup is counted under.
 */
static int32_t destination(uint32_t entry, int32_t U, int32_t W, int32_t self,
                           int* tier_out, int32_t* status)
{
    uint32_t tier = entry >> 30;
    uint32_t owner = entry & 0x3FFFFFFFu;
    if (tier == 0) { *tier_out = 0; return self; }
    if (tier == 1) {
        *tier_out = 1;
        if (owner >= (uint32_t)W) { flag(status, DEV_BAD_PLACEMENT); return self; }
        return (self / W) * W + (int32_t)owner;
    }
    if (tier == 2) {
        *tier_out = 2;
        if (owner >= (uint32_t)U) { flag(status, DEV_BAD_PLACEMENT); return self; }
        return (int32_t)owner;
    }
    *tier_out = 0;
    flag(status, DEV_BAD_PLACEMENT);
    return self;
}

/*
 * Route + bucketize (Section 3.2, "input data distribution").  A stable
 * counting sort of the lookups by destination bucket: count, exclusive scan,
 * then place the lookups one by one in their original order.
 */
int oracle_route_bucketize(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts, int32_t* status)
{
    if (!offsets || !row_base || !placement || !bucket_offsets) return ERR_NULL;
    if (n > 0 && (!ids || !out_rows || !out_pos)) return ERR_NULL;
    if (n < 0 || n >= ((int64_t)1 << 31) || T < 1 || B < 1) return ERR_SIZE;
    if ((int64_t)T * B >= ((int64_t)1 << 31)) return ERR_SIZE;
    if (U < 1 || U > 4096 || W < 1 || U % W != 0 || self < 0 || self >= U) return ERR_CONFIG;

    int64_t S = (int64_t)T * B;
    for (int32_t b = 0; b <= U; ++b) bucket_offsets[b] = 0;
    if (tier_counts) tier_counts[0] = tier_counts[1] = tier_counts[2] = 0;
    if (!offsets_ok(offsets, S, n)) {
        flag(status, DEV_BAD_OFFSETS);   /* outputs unspecified: nothing else is written */
        return OK;
    }

    int64_t* g = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    int32_t* dest = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int64_t* cursor = (int64_t*)calloc((size_t)U + 1, sizeof(int64_t));
    int64_t tiers[3] = {0, 0, 0};

    /* remap every lookup */
    for (int64_t s = 0; s < S; ++s) {
        int64_t t = s / B;
        int64_t rows_t = row_base[t + 1] - row_base[t];
        for (int64_t i = offsets[s]; i < offsets[s + 1]; ++i) {
            int64_t id = ids[i];
            if (id < 0 || id >= rows_t) { flag(status, DEV_BAD_ID); id = 0; }
            g[i] = row_base[t] + id;
            int tier;
            dest[i] = destination(placement[g[i]], U, W, self, &tier, status);
            tiers[tier] += 1;
        }
    }
    /* count */
    for (int64_t i = 0; i < n; ++i) cursor[dest[i] + 1] += 1;
    /* exclusive scan */
    for (int32_t b = 0; b < U; ++b) cursor[b + 1] += cursor[b];
    for (int32_t b = 0; b <= U; ++b) bucket_offsets[b] = cursor[b];
    /* stable placement */
    for (int64_t i = 0; i < n; ++i) {
        int64_t j = cursor[dest[i]]++;
        out_rows[j] = g[i];
        out_pos[j] = (int32_t)i;
    }
    if (tier_counts) { tier_counts[0] = tiers[0]; tier_counts[1] = tiers[1]; tier_counts[2] = tiers[2]; }
    free(g); free(dest); free(cursor);
    return OK;
}

static int elem_size(int dtype)
{
    return dtype == DT_F32 ? 4 : (dtype == DT_F16 || dtype == DT_BF16) ? 2 : 0;
}

/*
 * Sequence gather (Section 2, "Embedding Pooling": sequence embeddings are
 * not reduced, every looked-up row is materialised in the output).
 * out[pos[j], :] = weights[rows[j], :], a byte copy.
 */
int oracle_seq_gather_fwd(
    const void* weights, int64_t R, int32_t D, int dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || n < 0 || D < 1 || j0 < 0 || j0 > j1) return ERR_SIZE;
    if (j1 > j0 && (!weights || !rows || !pos || !out)) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t r = rows[j];
        int64_t p = pos[j];
        if (r < 0 || r >= R || p < 0 || p >= n) { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)out + (size_t)p * row_bytes,
               (const char*)weights + (size_t)r * row_bytes, row_bytes);
    }
    return OK;
}

/*
 * The two steps either side of the row exchange (Section 3.2, "dynamic
 * communication": the rows a GPU looked up for another GPU are sent back in
 * the order that GPU's ids arrived; Table 3, column "Dynamic Comms").
 * Owner: send[j - j0, :] = weights[rows[j], :].
 */
int oracle_seq_gather_send(
    const void* weights, int64_t R, int32_t D, int dtype,
    const int64_t* rows, int64_t j0, int64_t j1, void* send, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || D < 1 || j0 < 0 || j0 > j1) return ERR_SIZE;
    if (j1 > j0 && (!weights || !rows || !send)) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t r = rows[j];
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)send + (size_t)(j - j0) * row_bytes,
               (const char*)weights + (size_t)r * row_bytes, row_bytes);
    }
    return OK;
}

/* Requester: out[pos[j], :] = recv[j - j0, :]. */
int oracle_seq_unbucketize(
    const void* recv, int32_t D, int dtype, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (n < 0 || D < 1 || j0 < 0 || j0 > j1) return ERR_SIZE;
    if (j1 > j0 && (!recv || !pos || !out)) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t p = pos[j];
        if (p < 0 || p >= n) { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)out + (size_t)p * row_bytes,
               (const char*)recv + (size_t)(j - j0) * row_bytes, row_bytes);
    }
    return OK;
}

/*
 * Replica store (Section 3.1: a data-parallel row lives on every GPU and is
 * looked up locally; Section 4.3: the rows chosen for replication are the
 * most popular ones).  The chosen rows are copied into a dense array in
 * selection order; slot_of_row maps a row to its first slot, -1 otherwise.
 */
int oracle_replica_build(
    const void* weights, int64_t R, int32_t D, int dtype,
    const int64_t* sel_rows, int64_t k, void* store, int32_t* slot_of_row, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || D < 1 || k < 0) return ERR_SIZE;
    if (!weights || !slot_of_row || (k > 0 && (!sel_rows || !store))) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t r = 0; r < R; ++r) slot_of_row[r] = -1;
    for (int64_t s = 0; s < k; ++s) {
        int64_t r = sel_rows[s];
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)store + (size_t)s * row_bytes,
               (const char*)weights + (size_t)r * row_bytes, row_bytes);
        if (slot_of_row[r] < 0) slot_of_row[r] = (int32_t)s;
    }
    return OK;
}

/* The gather with replicated rows served from the store. */
int oracle_seq_gather_fwd_replica(
    const void* weights, int64_t R, int32_t D, int dtype,
    const void* store, int64_t k, const int32_t* slot_of_row,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || n < 0 || D < 1 || j0 < 0 || j0 > j1 || k < 0) return ERR_SIZE;
    if (j1 > j0 && (!weights || !rows || !pos || !out || !slot_of_row || (k > 0 && !store))) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t r = rows[j];
        int64_t p = pos[j];
        if (r < 0 || r >= R || p < 0 || p >= n) { flag(status, DEV_BAD_ID); continue; }
        int32_t s = slot_of_row[r];
        const char* from;
        if (s < 0) from = (const char*)weights + (size_t)r * row_bytes;
        else if (s < k) from = (const char*)store + (size_t)s * row_bytes;
        else { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)out + (size_t)p * row_bytes, from, row_bytes);
    }
    return OK;
}

/*
 * Replica slots handed over by the router (Section 3.1: a replicated row has
 * no owner to name, every GPU holds it; Section 4.3: the replicated rows are
 * the few most popular ones).  The owner bits of a tier-0 placement entry are
 * free, so they carry the row's slot in the replica store, NO_SLOT if it has
 * none; the router, which reads the entry of every lookup anyway, can then
 * hand each lookup's slot to the gather.
 */
#define NO_SLOT 0x3FFFFFFFu

/* placement[r] of every tier-0 row r: owner bits = slot_of_row[r], or NO_SLOT. */
int oracle_replica_tag_slots(uint32_t* placement, int64_t R, const int32_t* slot_of_row, int32_t* status)
{
    if (!placement || !slot_of_row) return ERR_NULL;
    if (R < 1) return ERR_SIZE;
    for (int64_t r = 0; r < R; ++r) {
        if ((placement[r] >> 30) != 0) continue;
        int32_t s = slot_of_row[r];
        if (s >= 0 && (uint32_t)s >= NO_SLOT) { flag(status, DEV_BAD_ID); s = -1; }   /* no such slot number */
        placement[r] = s >= 0 ? (uint32_t)s : NO_SLOT;
    }
    return OK;
}

/* out_slots[j] = the slot the placement entry of rows[j] carries, -1 if none (or not tier 0). */
int oracle_lookup_slots(
    const uint32_t* placement, int64_t R, const int64_t* rows, int64_t j0, int64_t j1,
    int32_t* out_slots, int32_t* status)
{
    if (R < 1 || j0 < 0 || j0 > j1) return ERR_SIZE;
    if (j1 > j0 && (!placement || !rows || !out_slots)) return ERR_NULL;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t r = rows[j];
        out_slots[j] = -1;
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); continue; }
        uint32_t e = placement[r];
        if ((e >> 30) == 0 && (e & 0x3FFFFFFFu) != NO_SLOT) out_slots[j] = (int32_t)(e & 0x3FFFFFFFu);
    }
    return OK;
}

/* The gather with each lookup's slot given: slots[j] >= 0 reads store[slots[j]], else weights[rows[j]]. */
int oracle_seq_gather_fwd_slots(
    const void* weights, int64_t R, int32_t D, int dtype,
    const void* store, int64_t k, const int64_t* rows, const int32_t* slots,
    const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || n < 0 || D < 1 || j0 < 0 || j0 > j1 || k < 0) return ERR_SIZE;
    if (j1 > j0 && (!weights || !rows || !pos || !out || !slots || (k > 0 && !store))) return ERR_NULL;
    size_t row_bytes = (size_t)D * (size_t)es;
    if (row_bytes % 16 != 0) return ERR_ALIGN;
    for (int64_t j = j0; j < j1; ++j) {
        int64_t r = rows[j];
        int64_t p = pos[j];
        if (r < 0 || r >= R || p < 0 || p >= n) { flag(status, DEV_BAD_ID); continue; }
        int32_t slot = slots[j];
        const char* from;
        if (slot < 0) from = (const char*)weights + (size_t)r * row_bytes;
        else if (slot < k) from = (const char*)store + (size_t)slot * row_bytes;
        else { flag(status, DEV_BAD_ID); continue; }
        memcpy((char*)out + (size_t)p * row_bytes, from, row_bytes);
    }
    return OK;
}

/* IEEE binary16 -> binary32, written out from the format definition. */
static float half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0) {
        if (man == 0) {
            bits = sign;
        } else {               /* subnormal: value = man * 2^-24 */
            int shift = 0;
            while (!(man & 0x400u)) { man <<= 1; ++shift; }
            man &= 0x3FFu;
            bits = sign | ((uint32_t)(127 - 15 - shift + 1) << 23) | (man << 13);
        }
    } else if (exp == 31) {
        bits = sign | 0x7F800000u | (man << 13);
    } else {
        bits = sign | ((exp + (127 - 15)) << 23) | (man << 13);
    }
    float f; memcpy(&f, &bits, 4); return f;
}

/* bfloat16 is the upper half of a binary32. */
static float bf16_to_float(uint16_t b)
{
    uint32_t bits = (uint32_t)b << 16;
    float f; memcpy(&f, &bits, 4); return f;
}

static float load_elem(const void* base, size_t index, int dtype)
{
    if (dtype == DT_F32) return ((const float*)base)[index];
    if (dtype == DT_F16) return half_to_float(((const uint16_t*)base)[index]);
    return bf16_to_float(((const uint16_t*)base)[index]);
}

typedef struct { int64_t row; int64_t pos; int64_t j; } lookup_t;

static int by_row_then_pos(const void* a, const void* b)
{
    const lookup_t* x = (const lookup_t*)a;
    const lookup_t* y = (const lookup_t*)b;
    if (x->row != y->row) return x->row < y->row ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return x->j < y->j ? -1 : (x->j > y->j ? 1 : 0);
}

/*
 * Backward of the sequence lookup (Section 3.2: the dynamic traffic of the
 * forward pass flows back in the backward pass; the owner of a row sums the
 * gradients of all of its appearances).
 *
 * The paper fixes no summation order.  The order used here: sort by
 * (row, pos); a partial sum starts at the first sorted index k of a row and
 * at every k that is a multiple of `tile`; partials are built left to right;
 * the row's gradient is the left-to-right sum of its partials.  All in fp32.
 * row_grads64 (may be NULL) receives the same sums accumulated in fp64.
 */
int oracle_seq_grad_bwd(
    const void* grad_out, int64_t n, int32_t D, int dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R,
    int32_t tile,
    int64_t* uniq_rows, float* row_grads, double* row_grads64,
    int64_t cap_unique, int64_t* num_unique, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || R >= 4294967295LL || n < 0 || D < 1 || j0 < 0 || j0 > j1 ||
        cap_unique < 0 || tile < 1) return ERR_SIZE;
    if (!num_unique) return ERR_NULL;
    if (j1 > j0 && (!grad_out || !rows || !pos)) return ERR_NULL;
    if (((size_t)D * (size_t)es) % 16 != 0) return ERR_ALIGN;

    int64_t m = j1 - j0;
    *num_unique = 0;
    if (m == 0) return OK;
    if (cap_unique > 0 && (!uniq_rows || !row_grads)) return ERR_NULL;

    lookup_t* lk = (lookup_t*)malloc(sizeof(lookup_t) * (size_t)m);
    for (int64_t q = 0; q < m; ++q) {
        int64_t r = rows[j0 + q];
        int64_t p = pos[j0 + q];
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); r = 0; }
        if (p < 0 || p >= n) { flag(status, DEV_BAD_ID); p = 0; }
        lk[q].row = r; lk[q].pos = p; lk[q].j = q;
    }
    /* The order is by (row, pos) whatever the order in j.  Where equal rows do  */
    /* not come with ascending pos in j, DEV_POS_ORDER says so: a caller that    */
    /* relies on that precondition (a stable sort by row alone) would sum the    */
    /* same terms in another order, so only sums-within-tolerance, the distinct  */
    /* rows and their number can be compared on such an input.                   */
    qsort(lk, (size_t)m, sizeof(lookup_t), by_row_then_pos);
    for (int64_t k = 1; k < m; ++k)
        if (lk[k].row == lk[k - 1].row && lk[k].j < lk[k - 1].j) { flag(status, DEV_POS_ORDER); break; }

    float* partial = (float*)malloc(sizeof(float) * (size_t)D);
    float* total = (float*)malloc(sizeof(float) * (size_t)D);
    double* total64 = (double*)malloc(sizeof(double) * (size_t)D);
    int64_t u = -1;           /* index of the current distinct row */
    int have_total = 0;       /* the current row already has a folded partial */
    int64_t k = 0;
    while (k < m) {
        int new_row = (k == 0) || (lk[k].row != lk[k - 1].row);
        if (new_row) { ++u; have_total = 0; for (int d = 0; d < D; ++d) total64[d] = 0.0; }
        /* one partial: from k up to the end of the row's run or of the tile */
        int64_t end = k + 1;
        while (end < m && lk[end].row == lk[k].row && (end % tile) != 0) ++end;
        for (int64_t q = k; q < end; ++q) {
            size_t base = (size_t)lk[q].pos * (size_t)D;
            for (int d = 0; d < D; ++d) {
                float x = load_elem(grad_out, base + (size_t)d, dtype);
                partial[d] = (q == k) ? x : partial[d] + x;
                total64[d] += (double)x;
            }
        }
        for (int d = 0; d < D; ++d) total[d] = have_total ? total[d] + partial[d] : partial[d];
        have_total = 1;
        k = end;
        int row_done = (k == m) || (lk[k].row != lk[k - 1].row);
        if (row_done) {
            if (u < cap_unique) {
                uniq_rows[u] = lk[k - 1].row;
                memcpy(row_grads + (size_t)u * (size_t)D, total, sizeof(float) * (size_t)D);
                if (row_grads64)
                    memcpy(row_grads64 + (size_t)u * (size_t)D, total64, sizeof(double) * (size_t)D);
            } else {
                flag(status, DEV_UNIQUE_OVERFLOW);
            }
        }
    }
    *num_unique = u + 1;
    free(partial); free(total); free(total64); free(lk);
    return OK;
}

/*
 * The lookups of [j0, j1) in the backward's order, (row asc, pos asc), as
 * 32-bit pairs (the order the sums above are taken in, written out).
 */
int oracle_sort_lookups(
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R, int64_t n,
    uint32_t* sorted_rows, uint32_t* sorted_pos, int32_t* status)
{
    if (R < 1 || R >= 4294967295LL || n < 0 || j0 < 0 || j0 > j1) return ERR_SIZE;
    int64_t m = j1 - j0;
    if (m == 0) return OK;
    if (!rows || !pos || !sorted_rows || !sorted_pos) return ERR_NULL;
    lookup_t* lk = (lookup_t*)malloc(sizeof(lookup_t) * (size_t)m);
    for (int64_t q = 0; q < m; ++q) {
        int64_t r = rows[j0 + q];
        int64_t p = pos[j0 + q];
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); r = 0; }
        if (p < 0 || p >= n) { flag(status, DEV_BAD_ID); p = 0; }
        lk[q].row = r; lk[q].pos = p; lk[q].j = q;
    }
    qsort(lk, (size_t)m, sizeof(lookup_t), by_row_then_pos);
    for (int64_t k = 0; k < m; ++k) {
        sorted_rows[k] = (uint32_t)lk[k].row;
        sorted_pos[k] = (uint32_t)lk[k].pos;
    }
    free(lk);
    return OK;
}

typedef struct { uint32_t count; int64_t g; } cand_t;

static int by_count_desc_then_row(const void* a, const void* b)
{
    const cand_t* x = (const cand_t*)a;
    const cand_t* y = (const cand_t*)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1;
    return x->g < y->g ? -1 : (x->g > y->g ? 1 : 0);
}

/*
 * Replication plan (Section 4.1: a row's frequency is its number of
 * appearances in the profiled samples; Section 4.3: rows are taken in
 * descending frequency order, and for a stated amount of extra memory the
 * best hybrid is the longest prefix that fits; Section 4.6: the tables are
 * merged into one distribution before sorting).
 */
int oracle_plan_replication(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, int64_t n, int64_t R,
    uint32_t* counts, int32_t flags,
    int64_t budget_bytes, int64_t bytes_per_row,
    int64_t* sel_rows, int64_t* num_selected,
    uint32_t* placement, int32_t* status)
{
    if (flags & ~15) return ERR_CONFIG;
    if ((flags & PLAN_TAG) && !(flags & PLAN_SELECT)) return ERR_CONFIG;
    if (R < 1 || R >= 4294967295LL) return ERR_SIZE;
    if (!counts) return ERR_NULL;

    if (flags & PLAN_ACCUMULATE) {
        if (n < 0 || n >= ((int64_t)1 << 31) || T < 1 || B < 1) return ERR_SIZE;
        if ((int64_t)T * B >= ((int64_t)1 << 31)) return ERR_SIZE;
        if (!offsets || !row_base || (n > 0 && !ids)) return ERR_NULL;
        int64_t S = (int64_t)T * B;
        if (!offsets_ok(offsets, S, n)) {
            flag(status, DEV_BAD_OFFSETS);
        } else {
            for (int64_t s = 0; s < S; ++s) {
                int64_t t = s / B;
                int64_t rows_t = row_base[t + 1] - row_base[t];
                for (int64_t i = offsets[s]; i < offsets[s + 1]; ++i) {
                    int64_t id = ids[i];
                    if (id < 0 || id >= rows_t) { flag(status, DEV_BAD_ID); id = 0; }
                    int64_t g = row_base[t] + id;
                    if (counts[g] == 0xFFFFFFFFu) flag(status, DEV_COUNT_OVERFLOW);
                    else counts[g] += 1;
                }
            }
        }
    }

    if (flags & PLAN_SELECT) {
        if (budget_bytes < 0 || bytes_per_row < 1) return ERR_SIZE;
        if (!num_selected) return ERR_NULL;
        if ((flags & PLAN_TAG) && !placement) return ERR_NULL;
        int64_t cap = budget_bytes / bytes_per_row;
        cand_t* cand = (cand_t*)malloc(sizeof(cand_t) * (size_t)R);
        int64_t nc = 0;
        for (int64_t g = 0; g < R; ++g)
            if (counts[g] > 0 || (flags & PLAN_ALLOW_ZERO)) { cand[nc].count = counts[g]; cand[nc].g = g; ++nc; }
        qsort(cand, (size_t)nc, sizeof(cand_t), by_count_desc_then_row);
        int64_t k = cap < nc ? cap : nc;
        if (k > 0 && !sel_rows) { free(cand); return ERR_NULL; }
        for (int64_t i = 0; i < k; ++i) sel_rows[i] = cand[i].g;
        if (flags & PLAN_TAG)
            for (int64_t i = 0; i < k; ++i) placement[cand[i].g] &= 0x3FFFFFFFu;
        *num_selected = k;
        free(cand);
    }
    return OK;
}

/*
 * Tier planner (Sections 4.2, 4.3, 4.5; cost terms from Tables 2 and 3 with
 * E = 1 and L = p for one row, p = count / num_samples).
 *
 * Per row, in units of D * dtype bytes (memory) or D * dtype bytes per unit of
 * bandwidth (communication):
 *   replicated (DP) instead of row-wise (RW):
 *     memory   (dp + B p) - (1/U + 2 B p)       = dp - 1/U - B p
 *     traffic  1/ar_global - 2 B p / a2a_global   (all-reduce in the backward pass only,
 *                                                  all-to-all in both passes)
 *   Flex instead of RW:
 *     memory   (dp/W + 2 B p) - (1/U + 2 B p)   = dp/W - 1/U
 *     traffic  2 B p / a2a_intra + (1/W)/ar_cross - 2 B p / a2a_global
 * Everything is kept exact: memory terms are multiplied by U * num_samples,
 * traffic comparisons are cross-multiplied; 128-bit integers hold the products.
 *
 * Rows are walked in descending frequency order (ties: ascending row), rows
 * that never appeared are not candidates.
 *   A  rows before the first one whose DP memory term is positive
 *   B  the longest prefix whose summed DP memory terms are <= 0
 *   C  rows whose DP traffic term is <= 0
 *   FLEX  rows whose Flex traffic term is <= 0
 * two tiers:   DP = first B rows (rounded down to the granule).
 * three tiers: DP = first A rows (rounded down); then Flex rows one by one
 *   while the memory saved by the DP rows pays for them and the row is
 *   inside FLEX; the Flex count is rounded down to the granule.
 */
typedef struct {
    int64_t num_samples;
    int64_t B;
    int32_t U, W, dp_multiplier, granule;
    int64_t a2a_global, a2a_intra, ar_global, ar_cross;
} tier_params_t;

enum { CUT_CANDIDATES = 0, CUT_A = 1, CUT_B = 2, CUT_C = 3, CUT_FLEX = 4, CUT_N_DP = 5, CUT_N_FLEX = 6,
       CUT_SUM_ALL = 7, CUT_SUM_DP = 8, CUT_SUM_FLEX = 9, N_CUTS = 10 };

typedef __int128 wide_t;

int oracle_plan_tiers(
    const uint32_t* counts, int64_t R, const tier_params_t* p, int32_t tiers,
    int64_t* sorted_rows, int64_t cap, int64_t* cuts, uint32_t* placement, int32_t* status)
{
    (void)status;
    if (!p || !cuts) return ERR_NULL;
    if (R < 1 || R >= 4294967295LL || cap < 0) return ERR_SIZE;
    if (tiers != 2 && tiers != 3) return ERR_CONFIG;
    if (p->num_samples < 1 || p->num_samples >= ((int64_t)1 << 40)) return ERR_CONFIG;
    if (p->B < 1 || p->B >= ((int64_t)1 << 31)) return ERR_CONFIG;
    if (p->U < 1 || p->U > 4096 || p->W < 1 || p->U % p->W != 0) return ERR_CONFIG;
    if (p->dp_multiplier < 1 || p->dp_multiplier > 1024) return ERR_CONFIG;
    if (p->granule < 1 || p->granule > (1 << 20)) return ERR_CONFIG;
    const int64_t bw_max = (int64_t)1 << 20;
    if (p->a2a_global < 1 || p->a2a_global >= bw_max || p->a2a_intra < 1 || p->a2a_intra >= bw_max ||
        p->ar_global < 1 || p->ar_global >= bw_max || p->ar_cross < 1 || p->ar_cross >= bw_max)
        return ERR_CONFIG;
    if (!counts) return ERR_NULL;
    if (cap > 0 && !sorted_rows) return ERR_NULL;

    cand_t* cand = (cand_t*)malloc(sizeof(cand_t) * (size_t)R);
    int64_t nc = 0;
    for (int64_t g = 0; g < R; ++g)
        if (counts[g] > 0) { cand[nc].count = counts[g]; cand[nc].g = g; ++nc; }
    qsort(cand, (size_t)nc, sizeof(cand_t), by_count_desc_then_row);

    const wide_t S = p->num_samples, B = p->B, U = p->U, W = p->W, dp = p->dp_multiplier;
    const wide_t static_term = (dp * U - 1) * S;          /* (dp - 1/U) * U * S */
    int64_t kA = nc, kB = 0, kC = 0, kF = 0;
    int seenA = 0;
    wide_t cum = 0;
    for (int64_t i = 0; i < nc; ++i) {
        const wide_t c = cand[i].count;
        const wide_t mem = static_term - U * B * c;       /* (dp - 1/U - B p) * U * S */
        if (!seenA && mem > 0) { kA = i; seenA = 1; }
        cum += mem;
        if (cum <= 0) kB = i + 1;
        /* 1/ar_global <= 2 B p / a2a_global */
        if ((wide_t)p->a2a_global * S <= 2 * B * c * (wide_t)p->ar_global) kC = i + 1;
        /* 2 B p / a2a_intra + 1/(W ar_cross) <= 2 B p / a2a_global */
        if (p->a2a_intra > p->a2a_global &&
            S * (wide_t)p->a2a_global * (wide_t)p->a2a_intra <=
                2 * B * c * (wide_t)(p->a2a_intra - p->a2a_global) * W * (wide_t)p->ar_cross)
            kF = i + 1;
    }

    const int64_t gran = p->granule;
    int64_t n_dp, n_flex = 0;
    if (tiers == 2) {
        n_dp = kB / gran * gran;
    } else {
        n_dp = kA / gran * gran;
        wide_t saved = 0;
        for (int64_t i = 0; i < n_dp; ++i) saved -= static_term - U * B * (wide_t)cand[i].count;
        const wide_t flex_cost = (dp * (U / W) - 1) * S;  /* (dp/W - 1/U) * U * S */
        wide_t spent = 0;
        int64_t i = n_dp;
        while (i < nc && i < kF && spent + flex_cost <= saved) { spent += flex_cost; ++i; }
        n_flex = (i - n_dp) / gran * gran;
    }

    int64_t sum_all = 0, sum_dp = 0, sum_flex = 0;
    for (int64_t i = 0; i < nc; ++i) {
        sum_all += cand[i].count;
        if (i < n_dp) sum_dp += cand[i].count;
        else if (i < n_dp + n_flex) sum_flex += cand[i].count;
    }
    cuts[CUT_CANDIDATES] = nc; cuts[CUT_A] = kA; cuts[CUT_B] = kB; cuts[CUT_C] = kC; cuts[CUT_FLEX] = kF;
    cuts[CUT_N_DP] = n_dp; cuts[CUT_N_FLEX] = n_flex;
    cuts[CUT_SUM_ALL] = sum_all; cuts[CUT_SUM_DP] = sum_dp; cuts[CUT_SUM_FLEX] = sum_flex;

    for (int64_t i = 0; i < n_dp + n_flex && i < cap; ++i) sorted_rows[i] = cand[i].g;
    if (placement) {
        for (int64_t i = 0; i < n_dp; ++i) placement[cand[i].g] &= 0x3FFFFFFFu;
        for (int64_t i = n_dp; i < n_dp + n_flex; ++i)
            placement[cand[i].g] = 0x40000000u | (uint32_t)((i - n_dp) % p->W);
    }
    free(cand);
    return OK;
}

/*
 * Sparse optimizer step on the deduplicated gradients (the step that follows
 * the backward of Section 3.2; the replicated strategy's static-memory factor
 * of the memory-cost table is this optimizer and gradient state).  Textbook
 * rules, in double precision, the new weight rounded once to the table's type
 * (round to nearest even):
 *   SGD              w -= lr g
 *   Adagrad          s += g^2 (per element);          w -= lr g / (sqrt(s) + eps)
 *   row-wise Adagrad s_r += mean over the row of g^2; w -= lr g / (sqrt(s_r) + eps)
 * state is float32 (read, updated in double, rounded back).  A row that has a
 * slot in the replica store gets the same new values there.
 */
enum { OPT_SGD = 0, OPT_ADAGRAD_ROWWISE = 1, OPT_ADAGRAD = 2 };

/* x rounded to a binary format with `mant` explicit mantissa bits and minimum normal exponent
 * emin (value 2^emin), ties to even; returns the sign, biased exponent and mantissa fields packed
 * for a 16-bit format with `ebits` exponent bits. */
static uint16_t round_to_16(double x, int mant, int ebits)
{
    const int bias = (1 << (ebits - 1)) - 1;
    const int emin = 1 - bias;
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    if (isnan(x)) return (uint16_t)(sign | (((1u << ebits) - 1u) << mant) | (1u << (mant - 1)));
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | (((1u << ebits) - 1u) << mant));
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);               /* a = f * 2^e, f in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
    int exp = e - 1;                  /* a = 1.xxx * 2^exp */
    if (exp < emin) exp = emin;       /* subnormal range: fixed quantum 2^(emin - mant) */
    double quantum = ldexp(1.0, exp - mant);
    double q = nearbyint(a / quantum);          /* ties to even in the default rounding mode */
    /* q is in [0, 2^(mant+1)]; fields follow from the integer */
    uint32_t qi = (uint32_t)q;
    uint32_t field;
    if (qi < (1u << mant)) field = qi;                                   /* subnormal (or zero) */
    else field = ((uint32_t)(exp - emin + 1) << mant) + (qi - (1u << mant));  /* a carry runs into the exponent */
    if (field >= (((1u << ebits) - 1u) << mant)) field = ((1u << ebits) - 1u) << mant;   /* overflow -> infinity */
    return (uint16_t)(sign | field);
}

static void store_elem(void* base, size_t index, int dtype, double x)
{
    if (dtype == DT_F32) ((float*)base)[index] = (float)x;
    else if (dtype == DT_F16) ((uint16_t*)base)[index] = round_to_16(x, 10, 5);
    else ((uint16_t*)base)[index] = round_to_16(x, 7, 8);
}

int oracle_sparse_update(
    void* weights, int64_t R, int32_t D, int dtype,
    const int64_t* uniq_rows, const float* row_grads, int64_t n_u,
    int32_t optimizer, float lr, float eps, float* state,
    void* store, const int32_t* slot_of_row, int64_t k, int32_t* status)
{
    int es = elem_size(dtype);
    if (!es) return ERR_DTYPE;
    if (R < 1 || D < 1 || n_u < 0 || k < 0) return ERR_SIZE;
    if (optimizer != OPT_SGD && optimizer != OPT_ADAGRAD_ROWWISE && optimizer != OPT_ADAGRAD) return ERR_CONFIG;
    if (!weights || (n_u > 0 && (!uniq_rows || !row_grads))) return ERR_NULL;
    if (optimizer != OPT_SGD && !state) return ERR_NULL;
    if ((store != NULL) != (slot_of_row != NULL)) return ERR_NULL;
    if (((size_t)D * (size_t)es) % 16 != 0) return ERR_ALIGN;
    for (int64_t u = 0; u < n_u; ++u) {
        int64_t r = uniq_rows[u];
        if (r < 0 || r >= R) { flag(status, DEV_BAD_ID); continue; }
        const float* g = row_grads + (size_t)u * (size_t)D;
        double row_state = 0.0;
        if (optimizer == OPT_ADAGRAD_ROWWISE) {
            double sq = 0.0;
            for (int32_t d = 0; d < D; ++d) sq += (double)g[d] * (double)g[d];
            row_state = (double)state[r] + sq / (double)D;
            state[r] = (float)row_state;
        }
        int32_t slot = slot_of_row ? slot_of_row[r] : -1;
        if (slot >= k) { flag(status, DEV_BAD_ID); slot = -1; }
        for (int32_t d = 0; d < D; ++d) {
            size_t at = (size_t)r * (size_t)D + (size_t)d;
            double w = (double)load_elem(weights, at, dtype);
            double gd = (double)g[d];
            double step;
            if (optimizer == OPT_SGD) {
                step = (double)lr * gd;
            } else if (optimizer == OPT_ADAGRAD) {
                double s = (double)state[at] + gd * gd;
                state[at] = (float)s;
                step = (double)lr * gd / (sqrt(s) + (double)eps);
            } else {
                step = (double)lr * gd / (sqrt(row_state) + (double)eps);
            }
            store_elem(weights, at, dtype, w - step);
            if (slot >= 0) store_elem(store, (size_t)slot * (size_t)D + (size_t)d, dtype, w - step);
        }
    }
    return OK;
}
