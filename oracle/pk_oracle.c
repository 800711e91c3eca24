/* CPU oracle for the packed multi-field embedding layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, single-threaded
 * definition against which the HIP path is checked.  It shares no code with
 * the HIP path; only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  Floating point is accumulated in double and rounded once.
 *
 * What it follows:
 *   - Sec. II-D lists the embedding layer's operators: Unique (drop repeated
 *     IDs), Gather (fetch rows), SegmentReduction (pool rows per segment), and
 *     states that the backward pass mirrors the forward pass.
 *   - Sec. III-B (D-Packing, Fig. 7) merges the ID tensors of all fields whose
 *     tables share an embedding dimension into one packed ID tensor, processed
 *     by one packed operation per step; the number of packed operations is
 *     proportional to the number of distinct dimensions.  Eq. 1 estimates the
 *     parameter volume of a pack, and packs above the norm are split evenly.
 *   - The optimiser is not part of the paper; the workload configurations fix
 *     Adagrad (lr, eps outside the square root, accumulator starting at 0).
 *
 * Readings where the paper is silent (also listed in the design notes):
 *   hash = (uint64)id mod rows; a pack's tables are stacked in table order and
 *   a key is base_row + hashed row; unique keys are in ascending order; mean
 *   pooling divides by the bag length counting repeats; an empty bag pools to
 *   zero and receives no gradient; repeated IDs have their gradients summed
 *   before the single Adagrad step of the row.
 *
 * Every function below is pinned by tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bfloat16 <-> float ------------------------------------------------- */
static float bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest, ties to even; inputs here are finite */
static uint16_t bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lower = u & 0xFFFFu, upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1;
    return (uint16_t)upper;
}

uint16_t orc_bf16_round(float f) { return bf16_round(f); }
float orc_bf16_widen(uint16_t b) { return bf16_widen(b); }

/* ---- H0: plan (Sec. III-B, D-Packing: one pack per distinct dimension) ----
 * Packs are the distinct (dim, dtype) pairs in ascending (dim, dtype) order.
 * Inside a pack the tables keep their index order and are stacked: base_row is
 * the running sum of rows.  A field's slot is its rank among the pack's fields
 * in field order.  The pooled outputs of one sample are concatenated in field
 * order: col(f) is the running sum of the dims of the fields before f.
 * Returns the number of packs; pack_* arrays need room for n_tables entries. */
int32_t orc_plan(int32_t n_tables, const int64_t *rows, const int32_t *dim, const int32_t *dtype,
                 int32_t n_fields, const int32_t *field_table,
                 int32_t *table_pack, int64_t *table_base,
                 int32_t *pack_dim, int32_t *pack_dtype, int64_t *pack_rows,
                 int32_t *field_pack, int32_t *field_slot, int64_t *field_col)
{
    int32_t n_packs = 0;
    for (int32_t t = 0; t < n_tables; ++t) {            /* collect distinct pairs */
        int found = 0;
        for (int32_t p = 0; p < n_packs; ++p)
            if (pack_dim[p] == dim[t] && pack_dtype[p] == dtype[t]) found = 1;
        if (!found) { pack_dim[n_packs] = dim[t]; pack_dtype[n_packs] = dtype[t]; ++n_packs; }
    }
    for (int32_t i = 1; i < n_packs; ++i)               /* insertion sort by (dim, dtype) */
        for (int32_t j = i; j > 0; --j) {
            int less = pack_dim[j] < pack_dim[j - 1] ||
                       (pack_dim[j] == pack_dim[j - 1] && pack_dtype[j] < pack_dtype[j - 1]);
            if (!less) break;
            int32_t d = pack_dim[j]; pack_dim[j] = pack_dim[j - 1]; pack_dim[j - 1] = d;
            int32_t y = pack_dtype[j]; pack_dtype[j] = pack_dtype[j - 1]; pack_dtype[j - 1] = y;
        }
    for (int32_t p = 0; p < n_packs; ++p) pack_rows[p] = 0;
    for (int32_t t = 0; t < n_tables; ++t)
        for (int32_t p = 0; p < n_packs; ++p)
            if (pack_dim[p] == dim[t] && pack_dtype[p] == dtype[t]) {
                table_pack[t] = p;
                table_base[t] = pack_rows[p];
                pack_rows[p] += rows[t];
            }
    int64_t col = 0;
    for (int32_t f = 0; f < n_fields; ++f) {
        int32_t p = table_pack[field_table[f]];
        int32_t slot = 0;
        for (int32_t g = 0; g < f; ++g)
            if (table_pack[field_table[g]] == p) ++slot;
        field_pack[f] = p;
        field_slot[f] = slot;
        field_col[f] = col;
        col += dim[field_table[f]];
    }
    return n_packs;
}

/* ---- Eq. 1: parameter volume of a packed table -----------------------------
 * CalcVParam(T) = N * sum_{t in T} dim_t * sum_{ID in t} freq(ID).  With freq
 * the relative frequency of an ID among all N occurrences, N * sum freq is the
 * number of occurrences that fall into table t, so the volume is the number
 * of floats the pack gathers.  occurrences[t] carries that count. */
double orc_calc_vparam(int32_t n_tables, const int32_t *table_pack, const int32_t *dim,
                       const double *occurrences, int32_t pack)
{
    double v = 0.0;
    for (int32_t t = 0; t < n_tables; ++t)
        if (table_pack[t] == pack) v += (double)dim[t] * occurrences[t];
    return v;
}

/* ---- Eq. 1 shard split (Sec. III-B) ----------------------------------------
 * A packed operation whose volume is high is split evenly into shards.  The
 * paper's text and example fix the rule used here: a pack is split only when its
 * volume is ABOVE THE AVERAGE over the packs (zero-volume packs aside), and
 * with one operation for the dim-8 tables and uniform data the dim-32 tables
 * get four shards, i.e. a pack that is split gets its volume relative to the
 * lightest pack's,
 *   shards(p) = round(V_p / min_q V_q) if V_p > mean_q V_q, else 1; at most
 *   max_shards and at most the pack's table count;
 * the pack's tables (in table order) are dealt to its shards in turn, so each
 * shard holds an equal share of them.  Shards become packs of their own,
 * ordered by (dim, dtype, shard); tables are stacked per shard in table order.
 * Packs with zero volume do not set the minimum and are not split.
 * In: the unsplit plan (n_base packs, base_pack per table).  Out: n_shards per
 * unsplit pack, and the split plan's table_pack / table_base / pack_* arrays
 * (room for n_tables packs).  Returns the number of packs after the split. */
int32_t orc_shard_split(int32_t n_tables, const int64_t *rows, const int32_t *dim, const int32_t *dtype,
                        int32_t n_base, const int32_t *base_pack, const double *occurrences,
                        int32_t max_shards, int32_t *n_shards,
                        int32_t *table_pack, int64_t *table_base,
                        int32_t *pack_dim, int32_t *pack_dtype, int64_t *pack_rows)
{
    double vmin = 0.0, vsum = 0.0;
    int32_t n_vol = 0;
    for (int32_t p = 0; p < n_base; ++p) {
        double v = orc_calc_vparam(n_tables, base_pack, dim, occurrences, p);
        if (v > 0.0 && (vmin == 0.0 || v < vmin)) vmin = v;
        if (v > 0.0) { vsum += v; ++n_vol; }
    }
    const double vmean = n_vol > 0 ? vsum / n_vol : 0.0;
    int32_t n_packs = 0;
    for (int32_t p = 0; p < n_base; ++p) {
        double v = orc_calc_vparam(n_tables, base_pack, dim, occurrences, p);
        int32_t n_tab = 0;
        for (int32_t t = 0; t < n_tables; ++t) if (base_pack[t] == p) ++n_tab;
        int32_t s = 1;
        if (vmin > 0.0 && v > vmean) s = (int32_t)floor(v / vmin + 0.5);      /* only packs above the average are split */
        if (s > max_shards) s = max_shards;
        if (s > n_tab) s = n_tab;
        if (s < 1) s = 1;
        n_shards[p] = s;
        int32_t seen = 0;
        for (int32_t t = 0; t < n_tables; ++t) {
            if (base_pack[t] != p) continue;
            int32_t q = n_packs + seen % s;               /* dealt in turn */
            if (seen < s) { pack_rows[q] = 0; pack_dim[q] = dim[t]; pack_dtype[q] = dtype[t]; }
            table_pack[t] = q;
            table_base[t] = pack_rows[q];
            pack_rows[q] += rows[t];
            ++seen;
        }
        n_packs += s;
    }
    return n_packs;
}

/* Sec. III-C, Eq. 2 (D-Interleaving): the micro-batch size is the smallest, over
 * the layer's operators, of the bound of the operator's dominant resource
 * divided by what one data instance costs of it,
 *   BS_micro = min_op RBound_op / RInstance_op ,
 * taken as whole samples and never more than the batch; the batch is then cut
 * into micro-batches of equal size (the paper's default), so with
 * M = ceil(B / BS_micro) micro-batches the size is ceil(B / M).  0 if not even
 * one sample fits. */
int32_t orc_micro_batch_size(int32_t B, int32_t n_ops, const double *rbound, const double *rinstance)
{
    double bs = (double)B;
    for (int32_t o = 0; o < n_ops; ++o) {
        double r = floor(rbound[o] / rinstance[o]);
        if (r < bs) bs = r;
    }
    if (bs < 1.0) return 0;
    int32_t b = (int32_t)bs;
    int32_t M = (B + b - 1) / b;
    return (B + M - 1) / M;
}

/* Fields follow their tables: slot = rank among the pack's fields in field
 * order; col(f) = running sum of the dims of the fields before f. */
void orc_field_slots(int32_t n_fields, const int32_t *field_table, const int32_t *table_pack, const int32_t *dim,
                     int32_t *field_pack, int32_t *field_slot, int64_t *field_col)
{
    int64_t col = 0;
    for (int32_t f = 0; f < n_fields; ++f) {
        int32_t p = table_pack[field_table[f]];
        int32_t slot = 0;
        for (int32_t g = 0; g < f; ++g)
            if (table_pack[field_table[g]] == p) ++slot;
        field_pack[f] = p;
        field_slot[f] = slot;
        field_col[f] = col;
        col += dim[field_table[f]];
    }
}

/* ---- H1: packed ID tensor + hash (Sec. III-B D-Packing; Fig. 2 "hashing") ----
 * Bags are field-major in the input: bag g = f*B + b owns ids[offsets[g] ..
 * offsets[g+1]).  The pack's tensor lists, slot by slot and sample by sample,
 * every ID of every field of the pack; key = base_row(table) + (uint64)id mod
 * rows(table).  pack_fields lists the pack's fields in slot order.
 * Returns nnz of the pack; packed_offsets has k*B+1 entries. */
int64_t orc_pack_keys(int32_t k, const int32_t *pack_fields, const int32_t *field_table,
                      const int64_t *rows, const int64_t *table_base, int32_t B,
                      const int64_t *ids, const int32_t *offsets,
                      uint64_t *key, int32_t *packed_offsets)
{
    int64_t q = 0;
    for (int32_t j = 0; j < k; ++j) {
        int32_t f = pack_fields[j];
        int32_t t = field_table[f];
        for (int32_t b = 0; b < B; ++b) {
            int64_t g = (int64_t)f * B + b;
            packed_offsets[(int64_t)j * B + b] = (int32_t)q;
            for (int32_t i = offsets[g]; i < offsets[g + 1]; ++i) {
                uint64_t id = (uint64_t)ids[i];
                key[q++] = (uint64_t)table_base[t] + id % (uint64_t)rows[t];
            }
        }
    }
    packed_offsets[(int64_t)k * B] = (int32_t)q;
    return q;
}

/* ---- H2: Unique (Sec. II-D) ------------------------------------------------
 * unique = the distinct keys in ascending order; inverse[q] = position of
 * key[q] in unique.  Returns the number of distinct keys. */
static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

int32_t orc_unique(int64_t n, const uint64_t *key, uint64_t *unique, int32_t *inverse)
{
    if (n == 0) return 0;
    uint64_t *s = (uint64_t *)malloc((size_t)n * sizeof(uint64_t));
    memcpy(s, key, (size_t)n * sizeof(uint64_t));
    qsort(s, (size_t)n, sizeof(uint64_t), cmp_u64);
    int32_t U = 0;
    for (int64_t i = 0; i < n; ++i)
        if (i == 0 || s[i] != s[i - 1]) unique[U++] = s[i];
    free(s);
    for (int64_t q = 0; q < n; ++q) {
        int32_t lo = 0, hi = U - 1;
        while (lo < hi) {
            int32_t mid = lo + (hi - lo) / 2;
            if (unique[mid] < key[q]) lo = mid + 1; else hi = mid;
        }
        inverse[q] = lo;
    }
    return U;
}

/* occurrences of each distinct key: seg_offsets[u] = number of positions whose
 * key is smaller than unique[u]; seg_perm = positions ordered by (key, q). */
void orc_segments(int64_t n, const int32_t *inverse, int32_t U, int32_t *seg_offsets, int32_t *seg_perm)
{
    for (int32_t u = 0; u <= U; ++u) seg_offsets[u] = 0;
    for (int64_t q = 0; q < n; ++q) seg_offsets[inverse[q] + 1] += 1;
    for (int32_t u = 0; u < U; ++u) seg_offsets[u + 1] += seg_offsets[u];
    int32_t *cur = (int32_t *)malloc(((size_t)U + 1) * sizeof(int32_t));
    memcpy(cur, seg_offsets, ((size_t)U + 1) * sizeof(int32_t));
    for (int64_t q = 0; q < n; ++q) seg_perm[cur[inverse[q]]++] = (int32_t)q;
    free(cur);
}

/* ---- H3: Gather (Sec. II-D) -------------------------------------------------
 * E[u,:] = W[unique[u],:] widened exactly to double.  W is the pack's stacked
 * table [R, D], fp32 (dtype 0) or bf16 bit patterns (dtype 1). */
void orc_gather(const void *W, int32_t dtype, int32_t D, int32_t U, const uint64_t *unique, double *E)
{
    for (int32_t u = 0; u < U; ++u)
        for (int32_t d = 0; d < D; ++d) {
            size_t e = (size_t)unique[u] * D + d;
            E[(size_t)u * D + d] = dtype == 0 ? (double)((const float *)W)[e]
                                              : (double)bf16_widen(((const uint16_t *)W)[e]);
        }
}

/* ---- H4+H5: SegmentReduction per bag, concatenated per sample (Sec. II-D) ----
 * For slot j (field f) and sample b: out[b, col(f) + d] = sum over the bag of
 * E[inverse[q], d]; mean pooling (pool[f] == 1) divides by the bag length; an
 * empty bag gives zeros.  out has row stride out_stride floats. */
void orc_pool(int32_t k, const int32_t *pack_fields, const int32_t *pool, const int64_t *field_col,
              int32_t B, int32_t D, const double *E, const int32_t *inverse,
              const int32_t *packed_offsets, float *out, int64_t out_stride)
{
    for (int32_t j = 0; j < k; ++j) {
        int32_t f = pack_fields[j];
        for (int32_t b = 0; b < B; ++b) {
            int32_t q0 = packed_offsets[(int64_t)j * B + b], q1 = packed_offsets[(int64_t)j * B + b + 1];
            for (int32_t d = 0; d < D; ++d) {
                double acc = 0.0;
                for (int32_t q = q0; q < q1; ++q) acc += E[(size_t)inverse[q] * D + d];
                if (pool[f] == 1 && q1 > q0) acc /= (double)(q1 - q0);
                out[(size_t)b * out_stride + field_col[f] + d] = (float)acc;
            }
        }
    }
}

/* ---- H6: gradient of H4 w.r.t. E, reduced per distinct key (Sec. II-D: the
 * backward pass mirrors the forward pass) ------------------------------------
 * G[u,d] = sum over positions q with inverse[q] == u of
 *          grad_out[b(q), col(f(q)) + d] * (1/L for mean pooling, else 1). */
void orc_scatter_add(int32_t k, const int32_t *pack_fields, const int32_t *pool, const int64_t *field_col,
                     int32_t B, int32_t D, const float *grad_out, int64_t grad_stride,
                     const int32_t *inverse, const int32_t *packed_offsets, int32_t U, double *G)
{
    for (size_t i = 0; i < (size_t)U * D; ++i) G[i] = 0.0;
    for (int32_t j = 0; j < k; ++j) {
        int32_t f = pack_fields[j];
        for (int32_t b = 0; b < B; ++b) {
            int32_t q0 = packed_offsets[(int64_t)j * B + b], q1 = packed_offsets[(int64_t)j * B + b + 1];
            for (int32_t q = q0; q < q1; ++q)
                for (int32_t d = 0; d < D; ++d) {
                    double g = (double)grad_out[(size_t)b * grad_stride + field_col[f] + d];
                    if (pool[f] == 1) g /= (double)(q1 - q0);
                    G[(size_t)inverse[q] * D + d] += g;
                }
        }
    }
}

/* ---- H7: sparse Adagrad on the rows of the distinct keys ---------------------
 * a' = a + g^2 ; w' = w - lr * g / (sqrt(a') + eps), element-wise, in double;
 * a' is stored as fp32, w' as fp32 or as bf16 (round to nearest even).
 * Wrow: the rows' current values widened to double (what orc_gather returns);
 * Arow: the rows' accumulators.  Rows of keys that do not occur are untouched
 * by construction: they never enter this function. */
void orc_adagrad_rows(int32_t U, int32_t D, int32_t dtype, const double *Wrow, const float *Arow,
                      const double *G, double lr, double eps, void *Wnew, float *Anew)
{
    for (size_t i = 0; i < (size_t)U * D; ++i) {
        double g = G[i];
        double a = (double)Arow[i] + g * g;
        double w = Wrow[i] - lr * g / (sqrt(a) + eps);
        Anew[i] = (float)a;
        if (dtype == 0) ((float *)Wnew)[i] = (float)w;
        else ((uint16_t *)Wnew)[i] = bf16_round((float)w);
    }
}

/* ---- second, independent route: per field, no packing, no Unique -------------
 * The plain definition of the layer's forward result: for field f with table
 * Wt [rows, D] and sample b, pool Wt[(uint64)id mod rows] over the bag. */
void orc_direct_field_forward(const void *Wt, int32_t dtype, int64_t rows, int32_t D, int32_t pool,
                              int32_t B, const int64_t *ids, const int32_t *bag_offsets /* B+1 */,
                              float *out, int64_t out_stride, int64_t col)
{
    for (int32_t b = 0; b < B; ++b)
        for (int32_t d = 0; d < D; ++d) {
            double acc = 0.0;
            int32_t L = bag_offsets[b + 1] - bag_offsets[b];
            for (int32_t i = bag_offsets[b]; i < bag_offsets[b + 1]; ++i) {
                size_t r = (size_t)((uint64_t)ids[i] % (uint64_t)rows);
                acc += dtype == 0 ? (double)((const float *)Wt)[r * D + d]
                                  : (double)bf16_widen(((const uint16_t *)Wt)[r * D + d]);
            }
            if (pool == 1 && L > 0) acc /= (double)L;
            out[(size_t)b * out_stride + col + d] = (float)acc;
        }
}

/* Dense gradient of one field's table: dW[r,:] += grad_out[b, col:col+D] * scale
 * for every occurrence of row r (fields sharing a table accumulate into the
 * same dW), followed by dense Adagrad restricted to rows with an occurrence. */
void orc_direct_field_grad(int64_t rows, int32_t D, int32_t pool, int32_t B, const int64_t *ids,
                           const int32_t *bag_offsets, const float *grad_out, int64_t grad_stride,
                           int64_t col, double *dW, uint8_t *touched)
{
    for (int32_t b = 0; b < B; ++b) {
        int32_t L = bag_offsets[b + 1] - bag_offsets[b];
        for (int32_t i = bag_offsets[b]; i < bag_offsets[b + 1]; ++i) {
            size_t r = (size_t)((uint64_t)ids[i] % (uint64_t)rows);
            touched[r] = 1;
            for (int32_t d = 0; d < D; ++d) {
                double g = (double)grad_out[(size_t)b * grad_stride + col + d];
                if (pool == 1) g /= (double)L;
                dW[r * D + d] += g;
            }
        }
    }
}

void orc_direct_table_adagrad(void *Wt, float *At, int32_t dtype, int64_t rows, int32_t D,
                              const double *dW, const uint8_t *touched, double lr, double eps)
{
    for (int64_t r = 0; r < rows; ++r) {
        if (!touched[r]) continue;
        for (int32_t d = 0; d < D; ++d) {
            size_t e = (size_t)r * D + d;
            double g = dW[e];
            double a = (double)At[e] + g * g;
            double w0 = dtype == 0 ? (double)((float *)Wt)[e] : (double)bf16_widen(((uint16_t *)Wt)[e]);
            double w = w0 - lr * g / (sqrt(a) + eps);
            At[e] = (float)a;
            if (dtype == 0) ((float *)Wt)[e] = (float)w;
            else ((uint16_t *)Wt)[e] = bf16_round((float)w);
        }
    }
}

/* Sec. II-D (operator list) and Sec. III-B (the fused Unique&Partition kernel): Partition splits the
 * distinct IDs by the worker that stores their rows.  Reading (the paper does not say how rows are dealt
 * to workers): row r of a packed table lives on worker r mod n_owners.  The distinct keys of a pack
 * (ascending) are regrouped by owner, owner 0 first, ascending inside an owner; offsets[o] = number of
 * keys of the owners before o (n_owners + 1 entries), index[i] = where part_keys[i] stands in `unique`
 * (what Stitch needs to put the rows that come back in their places). */
void orc_partition(int32_t U, const uint64_t *unique, int32_t n_owners, uint64_t *part_keys, int32_t *index,
                   int32_t *offsets)
{
    int32_t at = 0;
    for (int32_t o = 0; o < n_owners; ++o) {
        offsets[o] = at;
        for (int32_t u = 0; u < U; ++u)
            if ((int32_t)(unique[u] % (uint64_t)n_owners) == o) { part_keys[at] = unique[u]; index[at] = u; ++at; }
    }
    offsets[n_owners] = at;
}
