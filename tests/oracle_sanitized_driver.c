/*
 * Runs the CPU oracle (oracle/suffix_trie.c, compiled into this program with
 * AddressSanitizer and UndefinedBehaviorSanitizer) over a case file written by
 * tests/test_oracle_sanitized.py and prints every result as text; the test compares the text
 * with what the ordinary build of the oracle returns for the same case.  Test infrastructure.
 *
 * Case file, int32 words unless noted: D, P, den_mode, linear, then alpha and min_score as two
 * doubles (4 words), n_docs, per document (len, tokens...), n_ctx, per context (len,
 * tokens..., split, then floor(alpha*P) + 1 target tokens).
 */
#include <stdio.h>

#include "../oracle/suffix_trie.c"

static int32_t *g_words;
static long g_n, g_at;

static int32_t next_word(void) {
    if (g_at >= g_n) { fprintf(stderr, "case file too short\n"); exit(3); }
    return g_words[g_at++];
}

int main(int argc, char **argv) {
    if (argc != 2) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    fseek(f, 0, SEEK_END);
    g_n = ftell(f) / 4;
    fseek(f, 0, SEEK_SET);
    g_words = (int32_t *)malloc(sizeof(int32_t) * (size_t)(g_n > 0 ? g_n : 1));
    if (fread(g_words, 4, (size_t)g_n, f) != (size_t)g_n) return 2;
    fclose(f);

    const int D = next_word(), P = next_word(), den_mode = next_word(), linear = next_word();
    double alpha, min_score;
    memcpy(&alpha, g_words + g_at, 8); g_at += 2;
    memcpy(&min_score, g_words + g_at, 8); g_at += 2;
    int K = (int)floor(alpha * (double)P);
    if (K < 1) K = 1;

    sdo_trie *tg = sdo_trie_new(D);
    const int n_docs = next_word();
    for (int i = 0; i < n_docs; i++) {
        const int len = next_word();
        sdo_trie_add_doc(tg, g_words + g_at, len, NULL);
        g_at += len;
    }
    double weight = 0.0;
    const double h = sdo_trie_entropy(tg, &weight);
    printf("global nodes %lld entropy %a weight %a\n", (long long)sdo_trie_num_nodes(tg), h, weight);

    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    int32_t *par = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    double *sc = (double *)malloc(sizeof(double) * (size_t)K);
    const int n_ctx = next_word();
    for (int c = 0; c < n_ctx; c++) {
        const int len = next_word();
        const int32_t *x = g_words + g_at;
        g_at += len;
        const int split = next_word();
        const int32_t *target = g_words + g_at;
        g_at += K + 1;
        /* the request's own trie, extended online in two pieces */
        sdo_trie *tr = sdo_trie_new(D);
        sdo_trie_append(tr, x, split);
        sdo_trie_append(tr, x + split, len - split);
        /* every pattern length on both structures: match, counts, children */
        for (int p = 1; p <= P && p <= len; p++) {
            int64_t cnt, ends, kids;
            sdo_trie_lookup(tg, x + len - p, p, &cnt, &ends, &kids);
            printf("ctx %d p %d global %d count %lld ends %lld children %lld", c, p,
                   (int)sdo_match(tg, x, len, p), (long long)cnt, (long long)ends, (long long)kids);
            sdo_trie_lookup(tr, x + len - p, p, &cnt, &ends, &kids);
            printf(" request count %lld ends %lld children %lld\n", (long long)cnt, (long long)ends,
                   (long long)kids);
        }
        double total;
        int32_t ml, src;
        const int n = sdo_generate(tg, tr, x, len, P, alpha, min_score, den_mode, linear, tok, par, sc,
                                   &total, &ml, &src);
        printf("ctx %d tree n %d p %d source %d score %a:", c, n, (int)ml, (int)src, total);
        for (int j = 0; j < n; j++) printf(" (%d %d %a)", (int)tok[j], (int)par[j], sc[j]);
        int32_t bonus;
        const int L = sdo_accept(n, tok, par, target, path, &bonus);
        printf(" accept %d bonus %d path", L, (int)bonus);
        for (int j = 0; j < L; j++) printf(" %d", (int)path[j]);
        printf("\n");
        sdo_trie_free(tr);
    }
    sdo_trie_free(tg);
    free(tok); free(par); free(path); free(sc); free(g_words);
    return 0;
}
