/* Runs every exported function of the CPU oracle on a case read from a file and dumps the
 * results, so that the oracle can be exercised under AddressSanitizer and
 * UndefinedBehaviorSanitizer as a program of its own (tests/test_oracle_sanitized.py builds
 * this file with -fsanitize=address,undefined and compares the dump with the ordinary build). */
#include <stdio.h>

#include "../../oracle/nms_oracle.c"

static void dump(const char *tag, const void *p, size_t bytes)
{
    printf("%s %zu ", tag, bytes);
    const unsigned char *b = (const unsigned char *)p;
    for (size_t i = 0; i < bytes; ++i) printf("%02x", b[i]);
    printf("\n");
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 3;
    int32_t n, dmax, k;
    float theta;
    if (fread(&n, 4, 1, f) != 1 || fread(&dmax, 4, 1, f) != 1 || fread(&k, 4, 1, f) != 1 || fread(&theta, 4, 1, f) != 1) return 4;
    size_t nn = (size_t)(n > 0 ? n : 1), dd = (size_t)(dmax > 0 ? dmax : 1);
    float *boxes = (float *)malloc(nn * 4 * sizeof(float));
    float *scores = (float *)malloc(nn * sizeof(float));
    int32_t *classes = (int32_t *)malloc(nn * sizeof(int32_t));
    float *D = (float *)malloc(dd * 4 * sizeof(float));
    if (fread(boxes, sizeof(float), (size_t)n * 4, f) != (size_t)n * 4) return 4;
    if (fread(scores, sizeof(float), (size_t)n, f) != (size_t)n) return 4;
    if (fread(classes, sizeof(int32_t), (size_t)n, f) != (size_t)n) return 4;
    if (fread(D, sizeof(float), (size_t)dmax * 4, f) != (size_t)dmax * 4) return 4;
    fclose(f);

    uint8_t *B = (uint8_t *)malloc(nn * nn), *V = (uint8_t *)malloc(nn), *keep = (uint8_t *)malloc(nn);
    int32_t *order = (int32_t *)malloc(nn * sizeof(int32_t));
    float *ranked = (float *)malloc(nn * 5 * sizeof(float));
    size_t W = (size_t)((n + 63) / 64);
    uint64_t *words = (uint64_t *)malloc((nn * (W ? W : 1)) * sizeof(uint64_t));
    nmso_map(boxes, scores, n, theta, B);
    dump("map", B, (size_t)n * n);
    nmso_reduce(B, n, V);
    dump("reduce", V, (size_t)n);
    nmso_keep(boxes, scores, n, theta, keep);
    dump("keep", keep, (size_t)n);
    nmso_order(scores, n, order);
    dump("order", order, (size_t)n * 4);
    nmso_ranked_boxes(boxes, order, n, ranked);
    dump("ranked", ranked, (size_t)n * 20);
    nmso_ranked_eliminations(boxes, order, n, theta, B);
    dump("elims", B, (size_t)n * n);
    nmso_ranked_elimination_words(boxes, order, n, theta, words);
    dump("words", words, (size_t)n * W * 8);
    memset(keep, 0, nn);
    nmso_greedy_keep(boxes, scores, n, theta, keep);
    dump("greedy", keep, (size_t)n);
    for (int combo = 0; combo < 64; ++combo) {
        memset(keep, 0, nn);
        nmso_keep_ex(boxes, scores, (combo & 32) ? classes : NULL, n, theta, combo & 1, (combo >> 1) & 1, (combo >> 2) & 1,
                     (combo >> 3) & 1, (combo & 16) ? 0.0f : 1.0f, keep);
        char tag[16];
        snprintf(tag, sizeof tag, "ex%d", combo);
        dump(tag, keep, (size_t)n);
    }
    if (n >= 2) {
        float q = nmso_overlap(boxes, boxes + 4), a = nmso_area(boxes);
        int o = nmso_outranks(scores, 1, 0), e = nmso_eliminates_ex(boxes, scores, classes, 1, 0, theta, 1, 1, 1, 0.0f);
        dump("overlap", &q, 4);
        dump("area", &a, 4);
        dump("outranks", &o, 4);
        dump("elim_ex", &e, 4);
    }
    uint8_t *Bs = (uint8_t *)malloc(dd * dd), *Vs = (uint8_t *)malloc(dd);
    nmso_alg12_square(D, dmax, theta, k, Bs, Vs);
    dump("squareB", Bs, (size_t)dmax * dmax);
    dump("squareV", Vs, (size_t)dmax);
    free(boxes); free(scores); free(classes); free(D); free(B); free(V); free(keep); free(order); free(ranked);
    free(words); free(Bs); free(Vs);
    return 0;
}
