/*
 * CPU ORACLE for SuffixDecoding draft generation.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain pointer suffix trie, one token per node, written for clarity, not
 * speed.  Nothing in the HIP product path includes, links or calls this file;
 * only tests, the smoke check and the cpu_baseline leg of the benchmark do.
 *
 * What it follows (arxiv 2411.04975):
 *   - Section 3, opening paragraphs: the root stands for the start of any
 *     suffix, a child stands for one possible next token, a root-to-node path
 *     is one distinct observed subsequence.
 *   - Section 3 "Suffix Tree Construction": a global structure over previous
 *     outputs and a per-request one over prompt + output, extended online.
 *   - Section 3 "Speculation Tree Expansion" (definitions of C(N), D(N),
 *     COUNT) and Algorithm 1 (ExpandSpeculationTree, MatchPattern,
 *     GenerateCandidateTree).
 *   - Section 3 "Adaptive Speculation Lengths": MAX_SPEC = alpha * p.
 *   - Section 3 "Speculation Tree Scoring": SCORE = sum of D(N).
 *   - Section 2 "Speculative Decoding" item 2 and Section 4.1 "Simulated
 *     Ablations": accept drafted tokens up to the first disagreement with the
 *     target model's greedy token.
 *   - Appendix "Predicting SuffixDecoding Effectiveness": the empirical entropy
 *     of a tree, steps (2) and (3).
 *
 * Readings this oracle takes where the paper is silent (each is listed in the
 * design notes of the repository):
 *   - depth bound D: every suffix is inserted truncated to its first D tokens;
 *   - suffixes never cross a document boundary; counts are per position;
 *   - DEN mode 0 (default): C(N) = COUNT(N) / COUNT(PARENT(N));
 *     DEN mode 1 (the printed equation): COUNT(N) / sum of sibling COUNTs;
 *   - the frontier is every not-yet-added child of any node already in the
 *     speculation tree (candidates taken from the children of the current
 *     leaves alone, as Algorithm 1 prints it, would only ever give a chain,
 *     which the paper presents as a separate "linear" variant);
 *   - arg-max ties: higher score, then lower token id, then lower parent index;
 *   - a candidate whose score is below min_score is never added;
 *   - N_p itself is not a draft node: tree size and SCORE count draft nodes;
 *   - between candidate trees a strictly greater SCORE wins, scanning the
 *     global structure p = 1..P first, then the per-request one;
 *   - "linear" variant (caption of the baseline-comparison figure: a variant
 *     restricted to chains of tokens): the candidates of a step are
 *     the children of the node added last (of N_p at the start), nothing else.
 *   - empirical entropy: a node's output distribution is COUNT(child) over the
 *     sum of its children's COUNTs; entropy in bits; every node with a child
 *     (the root included) is weighted by that sum, i.e. by how many times a
 *     next token was observed below it.
 *
 * Pins: tests/test_oracle_pins.py checks this file against brute-force corpus
 * scans, closed forms and trie invariants written independently in Python.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

typedef struct {
    int32_t token;
    int32_t count;        /* occurrences of the path root..this node           */
    int32_t ends;         /* inserted (truncated) suffixes that stop here      */
    int32_t first_child;  /* -1 if none                                        */
    int32_t next_sibling; /* -1 if none                                        */
    int32_t depth;
} sdo_node;

typedef struct {
    int32_t node;
    int32_t depth;
} sdo_cursor;

typedef struct {
    int D;
    sdo_node *nodes;
    int64_t n_nodes, cap_nodes;
    /* child lookup: open addressing on (parent, token) -> node */
    uint64_t *hkey;
    int32_t *hval;
    int64_t hcap, hused;
    /* online extension of ONE sequence: suffixes still shorter than D */
    sdo_cursor *cur;
    int n_cur;
} sdo_trie;

static uint64_t mix64(uint64_t x) {
    x ^= x >> 33; x *= 0xff51afd7ed558ccdULL;
    x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL;
    x ^= x >> 33; return x;
}

static uint64_t make_key(int32_t parent, int32_t token) {
    return ((uint64_t)(uint32_t)parent << 32) | (uint64_t)(uint32_t)token;
}

#define EMPTY_KEY 0xffffffffffffffffULL

static void hash_alloc(sdo_trie *t, int64_t cap) {
    t->hkey = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)cap);
    t->hval = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    for (int64_t i = 0; i < cap; i++) t->hkey[i] = EMPTY_KEY;
    t->hcap = cap;
    t->hused = 0;
}

static void hash_put(sdo_trie *t, uint64_t key, int32_t val) {
    uint64_t m = (uint64_t)t->hcap - 1;
    uint64_t i = mix64(key) & m;
    while (t->hkey[i] != EMPTY_KEY) i = (i + 1) & m;
    t->hkey[i] = key;
    t->hval[i] = val;
    t->hused++;
}

static void hash_grow(sdo_trie *t) {
    uint64_t *ok = t->hkey; int32_t *ov = t->hval; int64_t oc = t->hcap;
    hash_alloc(t, oc * 2);
    for (int64_t i = 0; i < oc; i++)
        if (ok[i] != EMPTY_KEY) hash_put(t, ok[i], ov[i]);
    free(ok); free(ov);
}

static int32_t find_child(const sdo_trie *t, int32_t parent, int32_t token) {
    uint64_t key = make_key(parent, token);
    uint64_t m = (uint64_t)t->hcap - 1;
    uint64_t i = mix64(key) & m;
    while (t->hkey[i] != EMPTY_KEY) {
        if (t->hkey[i] == key) return t->hval[i];
        i = (i + 1) & m;
    }
    return -1;
}

static int32_t add_child(sdo_trie *t, int32_t parent, int32_t token) {
    if (t->n_nodes == t->cap_nodes) {
        t->cap_nodes *= 2;
        t->nodes = (sdo_node *)realloc(t->nodes, sizeof(sdo_node) * (size_t)t->cap_nodes);
    }
    int32_t id = (int32_t)t->n_nodes++;
    sdo_node *n = &t->nodes[id];
    n->token = token; n->count = 0; n->ends = 0; n->first_child = -1;
    n->next_sibling = t->nodes[parent].first_child;
    n->depth = t->nodes[parent].depth + 1;
    t->nodes[parent].first_child = id;
    if ((t->hused + 1) * 10 > t->hcap * 6) hash_grow(t);
    hash_put(t, make_key(parent, token), id);
    return id;
}

static int32_t find_or_add(sdo_trie *t, int32_t parent, int32_t token) {
    int32_t c = find_child(t, parent, token);
    return c >= 0 ? c : add_child(t, parent, token);
}

sdo_trie *sdo_trie_new(int D) {
    sdo_trie *t = (sdo_trie *)calloc(1, sizeof(sdo_trie));
    t->D = D;
    t->cap_nodes = 1024;
    t->nodes = (sdo_node *)malloc(sizeof(sdo_node) * (size_t)t->cap_nodes);
    t->n_nodes = 1;
    t->nodes[0].token = -1; t->nodes[0].count = 0; t->nodes[0].ends = 0;
    t->nodes[0].first_child = -1; t->nodes[0].next_sibling = -1; t->nodes[0].depth = 0;
    hash_alloc(t, 4096);
    t->cur = (sdo_cursor *)malloc(sizeof(sdo_cursor) * (size_t)(D + 1));
    t->n_cur = 0;
    return t;
}

void sdo_trie_free(sdo_trie *t) {
    if (!t) return;
    free(t->nodes); free(t->hkey); free(t->hval); free(t->cur); free(t);
}

int64_t sdo_trie_num_nodes(const sdo_trie *t) { return t->n_nodes; }

/* Insert every suffix of one document, truncated to D tokens.  COUNT grows on
 * each node along the inserted path, ENDS on its last node.  If `allowed` is
 * not NULL only suffixes whose first token t has allowed[t] != 0 are inserted:
 * the trie is then exact below those first tokens and empty elsewhere. */
void sdo_trie_add_doc(sdo_trie *t, const int32_t *tok, int64_t len, const uint8_t *allowed) {
    for (int64_t i = 0; i < len; i++) {
        if (allowed && !allowed[tok[i]]) continue;
        int64_t stop = i + t->D < len ? i + t->D : len;
        int32_t node = 0;
        for (int64_t k = i; k < stop; k++) {
            node = find_or_add(t, node, tok[k]);
            t->nodes[node].count++;
        }
        t->nodes[node].ends++;
        t->nodes[0].count++;
    }
}

/* Extend the single sequence held by this trie by k tokens, so that the trie
 * equals the one sdo_trie_add_doc would build over the longer sequence.  Each
 * suffix that is still shorter than D tokens keeps a cursor at its last node. */
void sdo_trie_append(sdo_trie *t, const int32_t *tok, int64_t k) {
    for (int64_t a = 0; a < k; a++) {
        t->cur[t->n_cur].node = 0;
        t->cur[t->n_cur].depth = 0;
        t->n_cur++;
        t->nodes[0].count++;
        int w = 0;
        for (int c = 0; c < t->n_cur; c++) {
            int32_t node = t->cur[c].node;
            if (node != 0) t->nodes[node].ends--;
            int32_t ch = find_or_add(t, node, tok[a]);
            t->nodes[ch].count++;
            t->nodes[ch].ends++;
            int depth = t->cur[c].depth + 1;
            if (depth < t->D) { t->cur[w].node = ch; t->cur[w].depth = depth; w++; }
        }
        t->n_cur = w;
    }
}

/* Walk the path w[0..len).  Returns the node id or -1. */
static int32_t walk(const sdo_trie *t, const int32_t *w, int len) {
    int32_t node = 0;
    for (int i = 0; i < len; i++) {
        node = find_child(t, node, w[i]);
        if (node < 0) return -1;
    }
    return node;
}

/* COUNT, ENDS and number of children of the path w; returns 0 if absent. */
int sdo_trie_lookup(const sdo_trie *t, const int32_t *w, int len, int64_t *count, int64_t *ends,
                    int64_t *n_children) {
    int32_t node = walk(t, w, len);
    if (node < 0) { *count = 0; *ends = 0; *n_children = 0; return 0; }
    *count = t->nodes[node].count;
    *ends = t->nodes[node].ends;
    int64_t c = 0;
    for (int32_t ch = t->nodes[node].first_child; ch >= 0; ch = t->nodes[ch].next_sibling) c++;
    *n_children = c;
    return 1;
}

/* Children (token, COUNT) of the path w, unordered; returns how many exist. */
int64_t sdo_trie_children(const sdo_trie *t, const int32_t *w, int len, int32_t *tokens,
                          int64_t *counts, int64_t cap) {
    int32_t node = walk(t, w, len);
    if (node < 0) return 0;
    int64_t c = 0;
    for (int32_t ch = t->nodes[node].first_child; ch >= 0; ch = t->nodes[ch].next_sibling) {
        if (c < cap) { tokens[c] = t->nodes[ch].token; counts[c] = t->nodes[ch].count; }
        c++;
    }
    return c;
}

/* Raw node table, for invariant checks done outside this file. */
void sdo_trie_dump(const sdo_trie *t, int32_t *token, int32_t *count, int32_t *ends,
                   int32_t *parent, int32_t *depth) {
    for (int64_t i = 0; i < t->n_nodes; i++) {
        token[i] = t->nodes[i].token; count[i] = t->nodes[i].count; ends[i] = t->nodes[i].ends;
        depth[i] = t->nodes[i].depth;
    }
    parent[0] = -1;
    for (int64_t i = 0; i < t->n_nodes; i++)
        for (int32_t ch = t->nodes[i].first_child; ch >= 0; ch = t->nodes[ch].next_sibling)
            parent[ch] = (int32_t)i;
}

/* Empirical entropy of the tree (Appendix, "Predicting SuffixDecoding
 * Effectiveness", steps 2 and 3): for every node with children, the entropy (in
 * bits) of the distribution COUNT(child) / sum of the children's COUNTs;
 * returned is the average over those nodes weighted by that sum.  *weight
 * receives the total weight.  0 for a tree without any child. */
double sdo_trie_entropy(const sdo_trie *t, double *weight) {
    double acc = 0.0, wsum = 0.0;
    for (int64_t v = 0; v < t->n_nodes; v++) {
        double s = 0.0;
        for (int32_t ch = t->nodes[v].first_child; ch >= 0; ch = t->nodes[ch].next_sibling)
            s += (double)t->nodes[ch].count;
        if (s <= 0.0) continue;
        double h = 0.0;
        for (int32_t ch = t->nodes[v].first_child; ch >= 0; ch = t->nodes[ch].next_sibling) {
            const double q = (double)t->nodes[ch].count / s;
            h -= q * log2(q);
        }
        acc += s * h;
        wsum += s;
    }
    if (weight) *weight = wsum;
    return wsum > 0.0 ? acc / wsum : 0.0;
}

/* MatchPattern (Algorithm 1): follow the last p tokens of x[0..tlen) from the
 * root.  Returns the node N_p, or -1 if a child is missing or p > tlen. */
int32_t sdo_match(const sdo_trie *t, const int32_t *x, int64_t tlen, int p) {
    if (p < 1 || (int64_t)p > tlen) return -1;
    return walk(t, x + (tlen - p), p);
}

static double den_of(const sdo_trie *t, int32_t v, int den_mode) {
    if (den_mode == 0) return (double)t->nodes[v].count;
    int64_t s = 0;
    for (int32_t ch = t->nodes[v].first_child; ch >= 0; ch = t->nodes[ch].next_sibling)
        s += t->nodes[ch].count;
    return (double)s;
}

typedef struct {
    double score;
    int32_t token, parent, node;
} sdo_cand;

typedef struct {
    sdo_cand *a;
    int64_t n, cap;
} sdo_frontier;

static void frontier_add_children(const sdo_trie *t, sdo_frontier *f, int32_t v, int32_t parent_idx,
                                  double parent_score, int den_mode) {
    double den = den_of(t, v, den_mode);
    for (int32_t ch = t->nodes[v].first_child; ch >= 0; ch = t->nodes[ch].next_sibling) {
        if (f->n == f->cap) {
            f->cap = f->cap ? f->cap * 2 : 64;
            f->a = (sdo_cand *)realloc(f->a, sizeof(sdo_cand) * (size_t)f->cap);
        }
        sdo_cand *c = &f->a[f->n++];
        double ratio = (double)t->nodes[ch].count / den;    /* C(N): one division          */
        c->score = parent_score * ratio;                    /* D(N): one multiplication    */
        c->token = t->nodes[ch].token;
        c->parent = parent_idx;
        c->node = ch;
    }
}

/* the total order of the arg-max: score high, token low, parent index low */
static int cand_better(const sdo_cand *a, const sdo_cand *b) {
    if (a->score != b->score) return a->score > b->score;
    if (a->token != b->token) return a->token < b->token;
    return a->parent < b->parent;
}

/* ExpandSpeculationTree (Algorithm 1) from node np with at most K draft nodes.
 * Outputs tokens/parents/scores of the draft nodes in the order they were
 * added (parent -1 = child of N_p) and SCORE = sum of scores in that order.
 * Returns the number of draft nodes. */
int sdo_expand(const sdo_trie *t, int32_t np, int K, double min_score, int den_mode, int linear,
               int32_t *tokens, int32_t *parents, double *scores, double *tree_score) {
    sdo_frontier f = {0, 0, 0};
    int n = 0;
    double total = 0.0;
    *tree_score = 0.0;
    if (np < 0) return 0;
    frontier_add_children(t, &f, np, -1, 1.0, den_mode);
    while (n < K && f.n > 0) {
        int64_t best = 0;
        for (int64_t i = 1; i < f.n; i++)
            if (cand_better(&f.a[i], &f.a[best])) best = i;
        sdo_cand b = f.a[best];
        if (b.score < min_score) break;
        tokens[n] = b.token; parents[n] = b.parent; scores[n] = b.score;
        total += b.score;
        f.a[best] = f.a[f.n - 1];
        f.n--;
        if (linear) f.n = 0; /* a chain: only the new node's children may follow */
        frontier_add_children(t, &f, b.node, n, b.score, den_mode);
        n++;
    }
    free(f.a);
    *tree_score = total;
    return n;
}

/* One (structure, p) unit: match then expand with K = floor(alpha * p). */
int sdo_speculate_unit(const sdo_trie *t, const int32_t *x, int64_t tlen, int p, double alpha,
                       double min_score, int den_mode, int linear, int32_t *tokens,
                       int32_t *parents, double *scores, double *tree_score) {
    *tree_score = 0.0;
    int32_t np = sdo_match(t, x, tlen, p);
    if (np < 0) return -1;
    int K = (int)floor(alpha * (double)p);
    return sdo_expand(t, np, K, min_score, den_mode, linear, tokens, parents, scores, tree_score);
}

/* GenerateCandidateTree (Algorithm 1): best tree over {global, request} x p=1..P.
 * Either trie may be NULL (treated as empty).  Outputs are written for the
 * winner only; returns its node count (0 if nothing scored above 0) and sets
 * match_len (0 if none) and source (0 global, 1 request, -1 none).
 * tokens/parents/scores need room for floor(alpha*P) entries; tmp_* likewise. */
int sdo_generate(const sdo_trie *tg, const sdo_trie *tr, const int32_t *x, int64_t tlen, int P,
                 double alpha, double min_score, int den_mode, int linear, int32_t *tokens,
                 int32_t *parents, double *scores, double *tree_score, int32_t *match_len,
                 int32_t *source) {
    int maxn = (int)floor(alpha * (double)P);
    if (maxn < 1) maxn = 1;
    int32_t *tt = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxn);
    int32_t *tp = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxn);
    double *ts = (double *)malloc(sizeof(double) * (size_t)maxn);
    double best = 0.0;
    int best_n = 0;
    *match_len = 0; *source = -1; *tree_score = 0.0;
    for (int s = 0; s < 2; s++) {
        const sdo_trie *t = s == 0 ? tg : tr;
        if (!t) continue;
        for (int p = 1; p <= P; p++) {
            double sc;
            int n = sdo_speculate_unit(t, x, tlen, p, alpha, min_score, den_mode, linear, tt, tp, ts,
                                       &sc);
            if (n > 0 && sc > best) {
                best = sc; best_n = n; *match_len = p; *source = s;
                memcpy(tokens, tt, sizeof(int32_t) * (size_t)n);
                memcpy(parents, tp, sizeof(int32_t) * (size_t)n);
                memcpy(scores, ts, sizeof(double) * (size_t)n);
            }
        }
    }
    *tree_score = best;
    free(tt); free(tp); free(ts);
    return best_n;
}

/* Greedy verification walk.  target[0] is the target model's token after the
 * context (at the root of the draft tree), target[1+j] its token after draft
 * node j.  Accept the child whose token equals the target at the current
 * node, move there, repeat.  path receives the accepted node indices, bonus
 * the target token at the last accepted node.  Returns the accepted length. */
int sdo_accept(int n_nodes, const int32_t *tokens, const int32_t *parents, const int32_t *target,
               int32_t *path, int32_t *bonus) {
    int v = -1, L = 0;
    for (;;) {
        int32_t want = target[v + 1];
        int next = -1;
        for (int j = 0; j < n_nodes; j++)
            if (parents[j] == v && tokens[j] == want) { next = j; break; }
        if (next < 0) break;
        path[L++] = next;
        v = next;
    }
    *bonus = target[v + 1];
    return L;
}
