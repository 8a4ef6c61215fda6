/*
 * CPU oracle for the paper's parallel NMS ("Work-Efficient Parallel Non-Maximum
 * Suppression Kernels").  TEST INFRASTRUCTURE ONLY: it exists to check the HIP
 * library and to be timed as the CPU baseline.  Nothing in the product path may
 * call, link or import it, and it shares no code with the HIP sources.
 *
 * Plain single-threaded loops, float32 arithmetic with every operation rounded
 * on its own (build with -O2 -ffp-contract=off -fno-fast-math; SSE scalar math).
 * No blocking, no early exit, no sorting shortcuts: each function is the
 * definition it cites, written out.
 *
 * Readings of the paper taken here (each is exercised by a pin in tests/):
 *   - A box is kept iff NO box that outranks it overlaps it beyond the
 *     threshold, whether or not that other box is itself kept (Algorithm 1 and
 *     Algorithm 2; postconditions of MapKernel and ReduceKernel in the section
 *     "Algorithm Correctness": V_i is the AND over all j of B_ij).
 *   - Overlap = area of the intersection divided by the area of the
 *     higher-scoring box d_j, with the pixel-inclusive "+1" on widths, heights
 *     and area (Algorithm 1; MapKernel postcondition A(d_i n d_j)/A(d_j)).
 *   - B_ij is the test "overlap < theta", so a pair with overlap == theta
 *     eliminates (Algorithm 1, last assignment).
 *   - The paper's boxes are squares {x, y, z, s}; here each axis has its own
 *     extent: x+z becomes x2, y+z becomes y2 and (z+1)^2 becomes
 *     ((x2-x1)+1)*((y2-y1)+1).  nmso_alg12_square() below evaluates the paper's
 *     own statement on {x, y, z, s} tuples (strict score guard, zero-filled
 *     capacity, k row partitions), and the tests check that the two agree on
 *     square inputs.
 *   - Equal scores: the paper's strict "<" lets two equal-score boxes ignore
 *     each other.  This build's stated rule is a total order: of two boxes with
 *     equal scores the one with the lower index outranks the other.
 *   - The "D[j].z != 0" term of Algorithm 1 guards the zero-filled tail of the
 *     fixed-capacity vector D.  Here n is explicit and there is no tail, so the
 *     term does not appear (nmso_alg12_square() keeps it).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- ranking -------------------------------------------------------------- */

/* Does box j outrank box i?  Algorithm 1's guard "D[i].s < D[j].s", completed
 * to a total order by the lower-index-wins tie rule.  -0.0f == +0.0f in C, so
 * the two zeros tie, as floating-point comparison says they should. */
static int outranks(const float *scores, int j, int i)
{
    if (scores[j] > scores[i]) return 1;
    if (scores[j] == scores[i] && j < i) return 1;
    return 0;
}

/* ---- overlap measure ------------------------------------------------------- */

/* Area of a box with the inclusive-pixel convention (Algorithm 1, the line
 * computing a; generalised from (z+1)*(z+1) to one extent per axis). */
static float box_area(const float *b)
{
    float w = (b[2] - b[0]) + 1.0f;
    float h = (b[3] - b[1]) + 1.0f;
    return w * h;
}

/* Overlap of victim box bi with the outranking box bj: intersection width and
 * height as in Algorithm 1 (min of the far edges minus max of the near edges,
 * plus one, floored at zero), their product divided by the area of bj. */
static float overlap(const float *bi, const float *bj)
{
    float far_x = bi[2] < bj[2] ? bi[2] : bj[2];
    float near_x = bi[0] > bj[0] ? bi[0] : bj[0];
    float w = (far_x - near_x) + 1.0f;
    if (!(w > 0.0f)) w = 0.0f;

    float far_y = bi[3] < bj[3] ? bi[3] : bj[3];
    float near_y = bi[1] > bj[1] ? bi[1] : bj[1];
    float h = (far_y - near_y) + 1.0f;
    if (!(h > 0.0f)) h = 0.0f;

    float a = box_area(bj);
    return (w * h) / a;
}

/* Exported so that tests can recompute single pairs (witnesses, invariants). */
float nmso_overlap(const float *bi, const float *bj) { return overlap(bi, bj); }
float nmso_area(const float *b) { return box_area(b); }
int nmso_outranks(const float *scores, int j, int i) { return outranks(scores, j, i); }

/* ---- map: the boolean matrix B ------------------------------------------------ */

/* MapKernel postcondition: B[i*n+j] = 1 unless j outranks i and their overlap
 * is not below theta.  B starts as all ones (the paper's memset) and only the
 * guarded entries are rewritten, exactly as Algorithm 1 does. */
void nmso_map(const float *boxes, const float *scores, int n, float theta, uint8_t *B)
{
    memset(B, 1, (size_t)n * (size_t)n);
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j < n; ++j) {
            if (outranks(scores, j, i)) {
                float q = overlap(boxes + 4 * (size_t)i, boxes + 4 * (size_t)j);
                B[(size_t)i * n + j] = (q < theta) ? 1 : 0;
            }
        }
    }
}

/* ReduceKernel postcondition: V_i = AND over j of B_ij. */
void nmso_reduce(const uint8_t *B, int n, uint8_t *V)
{
    for (int i = 0; i < n; ++i) {
        uint8_t v = 1;
        for (int j = 0; j < n; ++j) v = (uint8_t)(v & B[(size_t)i * n + j]);
        V[i] = v;
    }
}

/* ---- the whole path without materialising B ------------------------------------ */

/* keep[i] = V_i, in the order of the input (Equation 2 masks D by V index for
 * index).  Same double loop as nmso_map + nmso_reduce, the matrix element used
 * as soon as it is known; no early exit. */
void nmso_keep(const float *boxes, const float *scores, int n, float theta, uint8_t *keep)
{
    for (int i = 0; i < n; ++i) {
        uint8_t v = 1;
        for (int j = 0; j < n; ++j) {
            uint8_t b = 1;
            if (outranks(scores, j, i)) {
                float q = overlap(boxes + 4 * (size_t)i, boxes + 4 * (size_t)j);
                b = (q < theta) ? 1 : 0;
            }
            v = (uint8_t)(v & b);
        }
        keep[i] = v;
    }
}

/* ---- rank order and the ranked views that the library's steps expose ----------- */

/* order[r] = index of the box with exactly r boxes outranking it.  The rank is
 * counted from the definition; nothing is sorted. */
void nmso_order(const float *scores, int n, int32_t *order)
{
    for (int i = 0; i < n; ++i) {
        int r = 0;
        for (int j = 0; j < n; ++j) r += outranks(scores, j, i);
        order[r] = i;
    }
}

/* Boxes gathered into rank order with their areas: out[r*5 + 0..3] = box of
 * rank r, out[r*5 + 4] = its area.  (Row-per-box on purpose: the library's own
 * buffer layout is the library's business; tests convert.) */
void nmso_ranked_boxes(const float *boxes, const int32_t *order, int n, float *out)
{
    for (int r = 0; r < n; ++r) {
        const float *b = boxes + 4 * (size_t)order[r];
        out[5 * (size_t)r + 0] = b[0];
        out[5 * (size_t)r + 1] = b[1];
        out[5 * (size_t)r + 2] = b[2];
        out[5 * (size_t)r + 3] = b[3];
        out[5 * (size_t)r + 4] = box_area(b);
    }
}

/* Elimination bits in rank order, one byte per ordered pair: E[r*n + c] = 1 iff
 * the box of rank c outranks (c < r) and eliminates the box of rank r, i.e. the
 * complement of B restricted to the ranked lower triangle; 0 elsewhere. */
void nmso_ranked_eliminations(const float *boxes, const int32_t *order, int n, float theta, uint8_t *E)
{
    memset(E, 0, (size_t)n * (size_t)n);
    for (int r = 0; r < n; ++r) {
        for (int c = 0; c < r; ++c) {
            float q = overlap(boxes + 4 * (size_t)order[r], boxes + 4 * (size_t)order[c]);
            E[(size_t)r * n + c] = (q < theta) ? 0 : 1;
        }
    }
}

/* Same bits packed 64 to a word: word w of rank r holds ranks 64w..64w+63 in
 * bits 0..63.  words[r*W + w], W = ceil(n/64).  For large n where the byte
 * matrix would not fit. */
void nmso_ranked_elimination_words(const float *boxes, const int32_t *order, int n, float theta, uint64_t *words)
{
    int W = (n + 63) / 64;
    memset(words, 0, (size_t)n * (size_t)W * sizeof(uint64_t));
    for (int r = 0; r < n; ++r) {
        for (int c = 0; c < r; ++c) {
            float q = overlap(boxes + 4 * (size_t)order[r], boxes + 4 * (size_t)order[c]);
            if (!(q < theta)) words[(size_t)r * W + (c >> 6)] |= (uint64_t)1 << (c & 63);
        }
    }
}

/* ---- the paper's own statement: square boxes in a vector of fixed capacity ------- */

/* The paper states the method on detections D = {x, y, z, s}: squares of side z with
 * their corner at (x, y), held in a vector of capacity dmax whose unused slots are all
 * zero (section "Proposed Parallel Algorithm").  This function evaluates that statement
 * with the measure defined above: slot t is the box spanning x..x+z and y..y+z, so its
 * extent per axis is z and its pixel-inclusive area (z+1)*(z+1), as in Algorithm 1.
 *   map     B_ij is written only where s_i < s_j STRICTLY (Algorithm 1's guard: equal
 *           scores do not touch each other -- no index tie-break here); there
 *           B_ij = (overlap < theta) AND (z_j != 0), the second term as the listing has
 *           it.  Elsewhere B keeps its preset 1.
 *   reduce  Algorithm 2 folds a row in k partitions of dmax/k columns each;
 *           V_i = AND over the partitions of (AND over the partition's columns).
 * x + z is computed in float32; it is exact for the integer inputs the pins use, and
 * only then does (x + z) - x give back z bit for bit.  dmax must be a multiple of k. */
void nmso_alg12_square(const float *D, int dmax, float theta, int k, uint8_t *B, uint8_t *V)
{
    float *box = (float *)malloc(sizeof(float) * 4 * (size_t)(dmax > 0 ? dmax : 1));
    for (int t = 0; t < dmax; ++t) {
        const float *d = D + 4 * (size_t)t;
        box[4 * t + 0] = d[0];
        box[4 * t + 1] = d[1];
        box[4 * t + 2] = d[0] + d[2];
        box[4 * t + 3] = d[1] + d[2];
    }
    for (int i = 0; i < dmax; ++i) {
        for (int j = 0; j < dmax; ++j) {
            uint8_t b = 1;
            float s_i = D[4 * (size_t)i + 3], s_j = D[4 * (size_t)j + 3], z_j = D[4 * (size_t)j + 2];
            if (s_i < s_j) {
                int below = overlap(box + 4 * (size_t)i, box + 4 * (size_t)j) < theta;
                b = (uint8_t)(below && z_j != 0.0f);
            }
            B[(size_t)i * dmax + j] = b;
        }
    }
    int columns = dmax / k;
    for (int i = 0; i < dmax; ++i) {
        uint8_t v = 1;
        for (int part = 0; part < k; ++part) {
            uint8_t whole = 1;
            for (int t = 0; t < columns; ++t) whole = (uint8_t)(whole & B[(size_t)i * dmax + part * columns + t]);
            v = (uint8_t)(v & whole);
        }
        V[i] = v;
    }
    free(box);
}

/* ---- classic sequential greedy NMS (a different function; not the default) -------- */

/* Visit boxes in rank order; a box is kept iff no KEPT box that outranks it
 * overlaps it with overlap >= theta (same overlap measure and tie rule as
 * above).  This is what the paper's introduction calls the conventional greedy
 * procedure; Algorithms 1 and 2 do not compute it (an eliminated box still
 * eliminates others there).  Used by tests for the containment invariant and
 * as the oracle of the selectable greedy rule. */
void nmso_greedy_keep(const float *boxes, const float *scores, int n, float theta, uint8_t *keep)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    nmso_order(scores, n, order);
    for (int r = 0; r < n; ++r) {
        int i = order[r];
        uint8_t v = 1;
        for (int c = 0; c < r; ++c) {
            int j = order[c];
            if (keep[j]) {
                float q = overlap(boxes + 4 * (size_t)i, boxes + 4 * (size_t)j);
                if (!(q < theta)) v = 0;
            }
        }
        keep[i] = v;
    }
    free(order);
}

/* ---- selectable variants of the rule ------------------------------------------------ */

/* The same map/reduce pattern with the choices that the paper's closing section says it
 * extends to, each one a switch; all switches off (and classes NULL) is nmso_keep /
 * nmso_greedy_keep above.
 *   measure 0: intersection over the area of the outranking box (Algorithm 1)
 *           1: intersection over union, union = (area_i + area_j) - intersection
 *   strict  0: overlap >= theta eliminates (Algorithm 1's "B = overlap < theta")
 *           1: only overlap > theta eliminates
 *   ties    0: equal scores are ordered by index (this build's total order)
 *           1: equal scores never eliminate each other (Algorithm 1's strict "<" as printed)
 *   offset    added to every extent before areas and intersections are formed: 1 is the
 *             paper's pixel-inclusive convention, 0 treats coordinates as continuous
 *   classes   NULL, or one label per box: only boxes with equal labels interact
 *   greedy  0: every outranking box counts (Algorithms 1 + 2)
 *           1: only outranking boxes that are themselves kept count */
static float extent(float lo, float hi, float offset) { return (hi - lo) + offset; }

static int eliminates_ex(const float *boxes, const float *scores, const int32_t *classes, int j, int i,
                         float theta, int measure, int strict, int ties, float offset)
{
    if (ties ? !(scores[j] > scores[i]) : !outranks(scores, j, i)) return 0;
    if (classes && classes[j] != classes[i]) return 0;
    const float *bi = boxes + 4 * (size_t)i;
    const float *bj = boxes + 4 * (size_t)j;

    float right = bi[2] < bj[2] ? bi[2] : bj[2];   /* intersection: the nearer of the far edges ... */
    float left = bi[0] > bj[0] ? bi[0] : bj[0];    /* ... and the farther of the near edges */
    float w = extent(left, right, offset);
    if (!(w > 0.0f)) w = 0.0f;
    float bottom = bi[3] < bj[3] ? bi[3] : bj[3];
    float top = bi[1] > bj[1] ? bi[1] : bj[1];
    float h = extent(top, bottom, offset);
    if (!(h > 0.0f)) h = 0.0f;
    float inter = w * h;

    float area_j = extent(bj[0], bj[2], offset) * extent(bj[1], bj[3], offset);
    float q;
    if (measure == 0) {
        q = inter / area_j;
    } else {
        float area_i = extent(bi[0], bi[2], offset) * extent(bi[1], bi[3], offset);
        q = inter / ((area_i + area_j) - inter);
    }
    return strict ? (q > theta) : !(q < theta);
}

void nmso_keep_ex(const float *boxes, const float *scores, const int32_t *classes, int n, float theta,
                  int greedy, int measure, int strict, int ties, float offset, uint8_t *keep)
{
    if (!greedy) {
        for (int i = 0; i < n; ++i) {
            uint8_t v = 1;
            for (int j = 0; j < n; ++j)
                if (eliminates_ex(boxes, scores, classes, j, i, theta, measure, strict, ties, offset)) v = 0;
            keep[i] = v;
        }
        return;
    }
    /* boxes are visited from the best rank down, so keep[j] is final for every j that can
     * eliminate i (such a j has a strictly better rank in the total order) */
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    nmso_order(scores, n, order);
    for (int r = 0; r < n; ++r) {
        int i = order[r];
        uint8_t v = 1;
        for (int c = 0; c < r; ++c) {
            int j = order[c];
            if (keep[j] && eliminates_ex(boxes, scores, classes, j, i, theta, measure, strict, ties, offset)) v = 0;
        }
        keep[i] = v;
    }
    free(order);
}

/* One pair under the options, for tests that recompute witnesses: does j eliminate i? */
int nmso_eliminates_ex(const float *boxes, const float *scores, const int32_t *classes, int j, int i,
                       float theta, int measure, int strict, int ties, float offset)
{
    return eliminates_ex(boxes, scores, classes, j, i, theta, measure, strict, ties, offset);
}
