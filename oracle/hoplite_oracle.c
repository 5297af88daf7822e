/*
 * hoplite_oracle.c -- plain CPU reference for the tree-ordered N-way reduce of
 * Hoplite (arXiv 2002.05814).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to say what the GPU library must
 * compute; it is slow on purpose (one recursive tree walk per element, scalar
 * loops, no threads, no blocking) and shares no source with the HIP path.
 * Only the tests, the smoke check and the CPU-baseline leg of the benchmark
 * may call it.
 *
 * What it follows, by passage of the paper:
 *   - Reduce(target, num_objects, sources, op), op in {sum,min,max}: Table 1.
 *   - d-ary reduce tree, arriving objects placed by generalised in-order
 *     traversal (first child, node, second..d-th child): section 3.4.2.
 *   - Only the first num_objects arrivals enter the tree: section 3.4.2.
 *   - A failed participant is removed and replaced, in the same tree
 *     position, by the next ready source object; the result is the reduce
 *     over the survivors: section 3.5.2.
 *   - Every object is folded in once and only once: section 3.4.2.
 *   - Broadcast delivers identical copies of one object: section 3.4.1.
 *
 * Readings where the paper is silent (each is listed in the design notes):
 *   - tree shape: complete d-ary tree in level order, children of node j are
 *     d*j+1 .. d*j+d (those below k);
 *   - a node combines, left to right, [first child's result, its own object,
 *     second child's result, ..., d-th child's result];
 *   - a slot whose occupant failed and has no replacement is a hole and
 *     contributes no term; the tree keeps its k-node shape;
 *   - fail_mask[i] = c >= 0 means object i delivers exactly c chunks and then
 *     fails (c = 0: it never becomes ready and never holds a slot; c >= C:
 *     it completed, i.e. healthy); failures are handled in the order they
 *     happen (by chunk count c, ties in arrival order), all participants
 *     streaming their chunks side by side;
 *   - 16-bit floats are widened exactly to binary32, combined in binary32 and
 *     rounded to nearest-even once, at the end;
 *   - int32 sum wraps modulo 2^32; min/max use the comparison forms
 *     max(a,b) = (b > a) ? b : a, min(a,b) = (b < a) ? b : a.
 *
 * parity pins: see tests/test_oracle_*.py (worked example of Fig. 5, closed
 * forms, brute force, library conversions).  No function here is unpinned.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

enum { ORA_SUM = 0, ORA_MIN = 1, ORA_MAX = 2 };
enum { ORA_F32 = 0, ORA_BF16 = 1, ORA_I32 = 2 };
enum { ORA_OK = 0, ORA_PARTIAL = 1, ORA_ERR_INVALID = -1, ORA_ERR_NO_SURVIVOR = -3 };

/* ------------------------------------------------------------------ */
/* Tree shape and slot numbering (section 3.4.2)                       */
/* ------------------------------------------------------------------ */

/* Child c (1-based) of node j in the level-ordered complete d-ary tree on k
 * nodes, or -1 when it does not exist. 64-bit so that a huge d cannot wrap. */
static int64_t child_of(int64_t j, int64_t c, int64_t d, int64_t k)
{
    int64_t x = d * j + c;
    return (c >= 1 && c <= d && x < k) ? x : -1;
}

typedef struct {
    int64_t k, d;
    int32_t *node_of_slot;   /* [k] t-th node of the traversal            */
    int32_t *slot_of_node;   /* [k] inverse                               */
    int64_t next;
} shape_t;

/* Generalised in-order traversal: first child, the node, then the other
 * children left to right. The t-th node visited is the tree position that
 * the t-th arriving object takes. */
static void visit_inorder(shape_t *s, int64_t j)
{
    int64_t c1 = child_of(j, 1, s->d, s->k);
    if (c1 >= 0) visit_inorder(s, c1);
    s->node_of_slot[s->next] = (int32_t)j;
    s->slot_of_node[j] = (int32_t)s->next;
    s->next++;
    for (int64_t c = 2; c <= s->d; ++c) {
        int64_t x = child_of(j, c, s->d, s->k);
        if (x < 0) break;
        visit_inorder(s, x);
    }
}

/* node_of_slot[t] = tree node given to the t-th arrival; parent_of_node[j] =
 * parent of node j (-1 for the root). */
int oracle_tree_slots(int k, int d, int32_t *node_of_slot, int32_t *parent_of_node)
{
    if (k < 1 || d < 1 || !node_of_slot) return ORA_ERR_INVALID;
    shape_t s;
    s.k = k; s.d = d; s.next = 0;
    s.node_of_slot = node_of_slot;
    s.slot_of_node = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    if (!s.slot_of_node) return ORA_ERR_INVALID;
    visit_inorder(&s, 0);
    free(s.slot_of_node);
    if (parent_of_node) {
        parent_of_node[0] = -1;
        for (int64_t j = 1; j < k; ++j) parent_of_node[j] = (int32_t)((j - 1) / d);
    }
    return ORA_OK;
}

/* ------------------------------------------------------------------ */
/* Who ends up in which slot (sections 3.4.2 and 3.5.2)                */
/* ------------------------------------------------------------------ */

static int64_t chunks_delivered(const int64_t *fail_mask, int i, int64_t C)
{
    if (!fail_mask) return C;
    int64_t c = fail_mask[i];
    return (c < 0 || c >= C) ? C : c;
}

/* occupant[t] = object finally sitting in slot t, or -1 for a hole.
 * n_chunks = C, the number of chunks an object is made of. */
int oracle_occupants(int n, int k, int64_t n_chunks, const int32_t *ready_order,
                     const int64_t *fail_mask, int32_t *occupant,
                     int32_t *k_eff, int32_t *n_replaced)
{
    if (n < 1 || k < 1 || k > n || n_chunks < 1 || !occupant) return ORA_ERR_INVALID;
    int32_t *arrival = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    char *seen = (char *)calloc((size_t)n, 1);
    char *dead = (char *)calloc((size_t)n, 1);
    int32_t *slot_of_obj = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    if (!arrival || !seen || !dead || !slot_of_obj) return ORA_ERR_INVALID;

    /* arrivals: ready order without the objects that never become ready */
    int n_arr = 0;
    for (int t = 0; t < n; ++t) {
        int i = ready_order ? ready_order[t] : t;
        if (i < 0 || i >= n || seen[i]) { free(arrival); free(seen); free(dead); free(slot_of_obj); return ORA_ERR_INVALID; }
        seen[i] = 1;
        if (chunks_delivered(fail_mask, i, n_chunks) == 0) continue;
        arrival[n_arr++] = i;
    }
    for (int i = 0; i < n; ++i) slot_of_obj[i] = -1;
    for (int t = 0; t < k; ++t) {
        occupant[t] = (t < n_arr) ? arrival[t] : -1;
        if (t < n_arr) slot_of_obj[arrival[t]] = t;
    }
    int pool_next = k;           /* arrival[pool_next..n_arr) wait as replacements */
    int replaced = 0;

    /* failures in the order they happen: by delivered chunk count, ties in
     * arrival order (selection by repeated scan keeps this obviously right) */
    int64_t last_c = 0; int last_pos = -1;
    for (;;) {
        int best = -1; int64_t best_c = 0;
        for (int p = 0; p < n_arr; ++p) {
            int i = arrival[p];
            int64_t c = chunks_delivered(fail_mask, i, n_chunks);
            if (c >= n_chunks) continue;
            /* strictly after the last handled (c, p) pair */
            if (c < last_c || (c == last_c && p <= last_pos)) continue;
            if (best < 0 || c < best_c) { best = p; best_c = c; }
        }
        if (best < 0) break;
        last_c = best_c; last_pos = best;
        int i = arrival[best];
        dead[i] = 1;
        int t = slot_of_obj[i];
        if (t < 0) continue;                 /* failed while waiting in the pool */
        slot_of_obj[i] = -1;
        while (pool_next < n_arr && dead[arrival[pool_next]]) pool_next++;
        if (pool_next < n_arr) {
            int j = arrival[pool_next++];
            occupant[t] = j; slot_of_obj[j] = t; replaced++;
        } else {
            occupant[t] = -1;
        }
    }
    int live = 0;
    for (int t = 0; t < k; ++t) if (occupant[t] >= 0) live++;
    if (k_eff) *k_eff = live;
    if (n_replaced) *n_replaced = replaced;
    free(arrival); free(seen); free(dead); free(slot_of_obj);
    if (live == 0) return ORA_ERR_NO_SURVIVOR;
    return live < k ? ORA_PARTIAL : ORA_OK;
}

/* ------------------------------------------------------------------ */
/* Element types                                                       */
/* ------------------------------------------------------------------ */

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;      /* exact: bf16 is the top half of binary32 */
    float f; memcpy(&f, &u, 4); return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even; NaN stays NaN (quiet). */
static uint16_t f32_to_bf16(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

void oracle_f32_to_bf16(const float *src, uint16_t *dst, size_t n)
{
    for (size_t i = 0; i < n; ++i) dst[i] = f32_to_bf16(src[i]);
}

void oracle_bf16_to_f32(const uint16_t *src, float *dst, size_t n)
{
    for (size_t i = 0; i < n; ++i) dst[i] = bf16_to_f32(src[i]);
}

static float combine_f32(int op, float a, float b)
{
    switch (op) {
    case ORA_SUM: return a + b;
    case ORA_MIN: return (b < a) ? b : a;
    default:      return (b > a) ? b : a;
    }
}

static int32_t combine_i32(int op, int32_t a, int32_t b)
{
    switch (op) {
    case ORA_SUM: return (int32_t)((uint32_t)a + (uint32_t)b);   /* wraps mod 2^32 */
    case ORA_MIN: return (b < a) ? b : a;
    default:      return (b > a) ? b : a;
    }
}

/* ------------------------------------------------------------------ */
/* The tree-ordered expression, one element at a time                  */
/* ------------------------------------------------------------------ */

typedef struct {
    int64_t k, d;
    int op, dtype;
    const int32_t *slot_of_node;
    const int32_t *occupant;          /* by slot; -1 = hole */
    const void *const *objs;
} expr_t;

/* Value of the subtree rooted at node j for element e. Returns 0 when the
 * subtree holds no object at all (then *out is untouched). Terms are
 * combined strictly left to right: first child, the node's own object, then
 * children 2..d. */
static int expr_f32(const expr_t *x, int64_t j, size_t e, float *out)
{
    int have = 0; float acc = 0.0f, v;
    int64_t c1 = child_of(j, 1, x->d, x->k);
    if (c1 >= 0 && expr_f32(x, c1, e, &v)) { acc = v; have = 1; }
    int obj = x->occupant[x->slot_of_node[j]];
    if (obj >= 0) {
        v = (x->dtype == ORA_BF16) ? bf16_to_f32(((const uint16_t *)x->objs[obj])[e])
                                   : ((const float *)x->objs[obj])[e];
        if (have) acc = combine_f32(x->op, acc, v); else { acc = v; have = 1; }
    }
    for (int64_t c = 2; c <= x->d; ++c) {
        int64_t ch = child_of(j, c, x->d, x->k);
        if (ch < 0) break;
        if (expr_f32(x, ch, e, &v)) {
            if (have) acc = combine_f32(x->op, acc, v); else { acc = v; have = 1; }
        }
    }
    if (have) *out = acc;
    return have;
}

static int expr_i32(const expr_t *x, int64_t j, size_t e, int32_t *out)
{
    int have = 0; int32_t acc = 0, v;
    int64_t c1 = child_of(j, 1, x->d, x->k);
    if (c1 >= 0 && expr_i32(x, c1, e, &v)) { acc = v; have = 1; }
    int obj = x->occupant[x->slot_of_node[j]];
    if (obj >= 0) {
        v = ((const int32_t *)x->objs[obj])[e];
        if (have) acc = combine_i32(x->op, acc, v); else { acc = v; have = 1; }
    }
    for (int64_t c = 2; c <= x->d; ++c) {
        int64_t ch = child_of(j, c, x->d, x->k);
        if (ch < 0) break;
        if (expr_i32(x, ch, e, &v)) {
            if (have) acc = combine_i32(x->op, acc, v); else { acc = v; have = 1; }
        }
    }
    if (have) *out = acc;
    return have;
}

/*
 * dst[e] = tree-ordered op over the objects that finally hold the k slots.
 * objs: n host pointers, each n_elems elements of dtype. chunk_elems only
 * fixes C = ceil(n_elems / chunk_elems), the unit in which fail_mask counts.
 * Returns ORA_OK, ORA_PARTIAL (fewer than k survivors; all of them reduced)
 * or a negative error; dst is written only on OK / PARTIAL.
 */
int oracle_reduce(void *dst, const void *const *objs, int n, size_t n_elems,
                  const int32_t *ready_order, int k, int op, int dtype,
                  size_t chunk_elems, int d, const int64_t *fail_mask,
                  int32_t *k_eff, int32_t *n_replaced)
{
    if (!dst || !objs || n < 1 || k < 1 || k > n || d < 1 || chunk_elems < 1) return ORA_ERR_INVALID;
    if (op < ORA_SUM || op > ORA_MAX || dtype < ORA_F32 || dtype > ORA_I32) return ORA_ERR_INVALID;
    int64_t C = n_elems ? (int64_t)((n_elems + chunk_elems - 1) / chunk_elems) : 1;

    int32_t *node_of_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    int32_t *slot_of_node = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    int32_t *occupant = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    if (!node_of_slot || !slot_of_node || !occupant) return ORA_ERR_INVALID;

    int rc = oracle_tree_slots(k, d, node_of_slot, NULL);
    if (rc == ORA_OK) {
        for (int t = 0; t < k; ++t) slot_of_node[node_of_slot[t]] = t;
        rc = oracle_occupants(n, k, C, ready_order, fail_mask, occupant, k_eff, n_replaced);
    }
    if (rc == ORA_OK || rc == ORA_PARTIAL) {
        expr_t x;
        x.k = k; x.d = d; x.op = op; x.dtype = dtype;
        x.slot_of_node = slot_of_node; x.occupant = occupant; x.objs = objs;
        for (size_t e = 0; e < n_elems; ++e) {
            if (dtype == ORA_I32) {
                int32_t v = 0;
                expr_i32(&x, 0, e, &v);
                ((int32_t *)dst)[e] = v;
            } else {
                float v = 0.0f;
                expr_f32(&x, 0, e, &v);
                if (dtype == ORA_BF16) ((uint16_t *)dst)[e] = f32_to_bf16(v);
                else ((float *)dst)[e] = v;
            }
        }
    }
    free(node_of_slot); free(slot_of_node); free(occupant);
    return rc;
}

/*
 * The same result without any order: for every element, op over the set of
 * surviving occupants, carried in binary64 (floats) so that it can serve as
 * the "true" value in tolerance checks. occupant comes from
 * oracle_occupants(). For int32 the sum is exact in int64 and returned
 * unwrapped in dst_i64.
 */
int oracle_reduce_set(double *dst_f64, int64_t *dst_i64, const void *const *objs,
                      size_t n_elems, const int32_t *occupant, int k, int op, int dtype)
{
    if (!objs || !occupant || k < 1) return ORA_ERR_INVALID;
    for (size_t e = 0; e < n_elems; ++e) {
        int have = 0; double a = 0.0; int64_t ai = 0;
        for (int t = 0; t < k; ++t) {
            int obj = occupant[t];
            if (obj < 0) continue;
            if (dtype == ORA_I32) {
                int64_t v = ((const int32_t *)objs[obj])[e];
                if (!have) ai = v;
                else if (op == ORA_SUM) ai += v;
                else if (op == ORA_MIN) ai = (v < ai) ? v : ai;
                else ai = (v > ai) ? v : ai;
            } else {
                double v = (dtype == ORA_BF16) ? (double)bf16_to_f32(((const uint16_t *)objs[obj])[e])
                                               : (double)((const float *)objs[obj])[e];
                if (!have) a = v;
                else if (op == ORA_SUM) a += v;
                else if (op == ORA_MIN) a = (v < a) ? v : a;
                else a = (v > a) ? v : a;
            }
            have = 1;
        }
        if (dtype == ORA_I32) { if (dst_i64) dst_i64[e] = ai; }
        else if (dst_f64) dst_f64[e] = a;
    }
    return ORA_OK;
}

/* Broadcast: every destination receives a byte-identical copy (section 3.4.1). */
int oracle_broadcast(void *const *dsts, int n_dst, const void *src, size_t n_bytes)
{
    if (n_dst < 0 || (n_dst > 0 && !dsts) || (n_bytes && !src)) return ORA_ERR_INVALID;
    for (int j = 0; j < n_dst; ++j) {
        const unsigned char *s = (const unsigned char *)src;
        unsigned char *t = (unsigned char *)dsts[j];
        for (size_t b = 0; b < n_bytes; ++b) t[b] = s[b];
    }
    return ORA_OK;
}
