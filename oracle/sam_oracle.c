/*
 * CPU checker for suffix-automaton draft retrieval.  TEST INFRASTRUCTURE ONLY:
 * this file is the slow, plain reference that the GPU library is compared with.
 * It shares no code with the GPU library and nothing in the product path may
 * call it.
 *
 * What it follows (arxiv 2411.10666):
 *   - state fields link / next / length / min_endpos and the root's initial
 *     values: Appendix A.1;
 *   - Expand and Build-SAM: Algorithm 2 (Appendix A.1);
 *   - Transfer: Algorithm 1 (Section 3.2);
 *   - per accepted token, static Transfer; dynamic Transfer on the automaton as
 *     it stands, then Expand: Section 3.3;
 *   - linear draft d = T[p+1 : p+n] with p = min_endpos of the matched state:
 *     Section 3.2; source choice "static only if l1 > l2 + l_bias": Section 3.2.
 *
 * Conventions: tokens are int32, arrays 0-indexed, states are numbered in the
 * order Algorithm 2 creates them (root 0; per token the new state, then the
 * clone if one is made).  min_endpos is the paper's 1-indexed end position,
 * i.e. a prefix length, so the paper's inclusive slice T[p+1 : p+n] is the
 * 0-indexed half-open slice T0[p : p+n).
 *
 * Each state's `next` is a token-sorted array searched by bisection; there is
 * no blocking, hashing or reordering of the algorithms' steps.
 *
 * Readings of points the paper leaves open (each is also listed in the design
 * notes of the repository):
 *   - one sentinel, -1, stands for "no state" (the listing mixes -1 and None);
 *   - after Expand clones the state q that the dynamic cursor sits on, the
 *     cursor's matched string (length len(p)+1 = len(clone)) belongs to the
 *     clone, so the cursor moves one suffix link up when len(link(s)) >= l;
 *   - a draft is cut at the end of the text and padded with -1;
 *   - a cursor at the root (l = 0) yields no draft;
 *   - ties between the two sources go to the dynamic one and there is no
 *     fallback to the other source when the chosen draft is empty;
 *   - tree drafts (Appendix A.1 freq, Algorithm 3, Algorithm 4): the root's freq
 *     starts at 0 (it is made neither by expansion nor by cloning); Algorithm
 *     3's dfs visits every state once (as printed it would re-add a shared
 *     child's count on every visit); TopK ranks successors by freq, ties by
 *     smaller token id; probabilities are the double quotient rounded to
 *     float; Prim multiplies in float, pops the largest probability, ties to
 *     the entry pushed first; the start token is element 0 of the draft (its
 *     parent is -1) and counts towards MAX_SIZE;
 *   - the auxiliary drafter of Section 3.4 has the fixed virtual match length
 *     l_threshold; by analogy with the strict "l1 > l2 + l_bias" rule the
 *     automaton's draft is kept only if its match length is strictly above it,
 *     otherwise the source is reported as "auxiliary" (3); l_threshold < 0
 *     means there is no auxiliary drafter.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t token;
    int32_t dst;
} oedge;

typedef struct {
    int32_t link;
    int32_t length;
    int32_t min_endpos;
    int32_t n_next;
    int32_t cap_next;
    oedge  *next;           /* sorted by token */
} ostate;

typedef struct {
    ostate  *st;
    int64_t  n_states;
    int64_t  cap_states;
    int32_t  last;
    int32_t  max_length;
    int64_t  n_trans;
    /* operation counters (what the algorithm touches) */
    int64_t  c_insert;      /* p.next[t] = c in the first loop of Expand        */
    int64_t  c_redirect;    /* p.next[t] = cl in the clone loop                 */
    int64_t  c_clone;       /* clones made                                      */
    int64_t  c_copy;        /* transitions copied into clones                   */
    int64_t  c_expand_probe;/* "t in p.next" tests made by Expand               */
    /* tree drafts: filled by osam_init_topk */
    uint8_t  *is_clone;     /* per state, set by Expand (freq starts at 0)      */
    int64_t   cap_clone;
    uint64_t *freq;         /* per state                                        */
    int32_t   topk;         /* k, 0 = not computed                              */
    int32_t  *topk_tok;     /* [n_states * k], -1 = unused entry                */
    int32_t  *topk_dst;
    float    *topk_prob;
} osam;

/* counters of a cursor walking an automaton with Transfer */
typedef struct {
    int64_t probes;         /* "t in s.next" tests                              */
    int64_t link_hops;      /* s = s.link moves                                 */
    int64_t next_moves;     /* s = s.next[t] moves                              */
} owalk;

/* ---- next map ---------------------------------------------------------- */

static int32_t next_find(const ostate *s, int32_t t)
{
    int32_t lo = 0, hi = s->n_next;
    while (lo < hi) {
        int32_t mid = lo + (hi - lo) / 2;
        if (s->next[mid].token < t) lo = mid + 1; else hi = mid;
    }
    if (lo < s->n_next && s->next[lo].token == t) return lo;
    return -1;
}

/* set next[t] = dst; returns 1 if a new transition was added, 0 if replaced,
 * -1 on allocation failure */
static int next_set(ostate *s, int32_t t, int32_t dst)
{
    int32_t lo = 0, hi = s->n_next;
    while (lo < hi) {
        int32_t mid = lo + (hi - lo) / 2;
        if (s->next[mid].token < t) lo = mid + 1; else hi = mid;
    }
    if (lo < s->n_next && s->next[lo].token == t) {
        s->next[lo].dst = dst;
        return 0;
    }
    if (s->n_next == s->cap_next) {
        int32_t nc = s->cap_next ? s->cap_next * 2 : 2;
        oedge *ne = (oedge *)realloc(s->next, (size_t)nc * sizeof(oedge));
        if (!ne) return -1;
        s->next = ne;
        s->cap_next = nc;
    }
    memmove(&s->next[lo + 1], &s->next[lo], (size_t)(s->n_next - lo) * sizeof(oedge));
    s->next[lo].token = t;
    s->next[lo].dst = dst;
    s->n_next++;
    return 1;
}

/* ---- Expand-State, INIT_SAM (Algorithm 2, Appendix A.1) ---------------- */

static int32_t expand_state(osam *S, int32_t link, int32_t length, int32_t pos)
{
    if (S->n_states == S->cap_states) {
        int64_t nc = S->cap_states ? S->cap_states * 2 : 16;
        ostate *ns = (ostate *)realloc(S->st, (size_t)nc * sizeof(ostate));
        if (!ns) return -1;
        S->st = ns;
        S->cap_states = nc;
    }
    ostate *s = &S->st[S->n_states];
    s->link = link;
    s->length = length;
    s->min_endpos = pos;
    s->n_next = 0;
    s->cap_next = 0;
    s->next = NULL;
    return (int32_t)S->n_states++;
}

osam *osam_new(void)
{
    osam *S = (osam *)calloc(1, sizeof(osam));
    if (!S) return NULL;
    /* root: link -1, next empty, length 0, min_endpos 0 */
    if (expand_state(S, -1, 0, 0) != 0) { free(S); return NULL; }
    S->last = 0;
    S->max_length = 0;
    return S;
}

void osam_free(osam *S)
{
    if (!S) return;
    for (int64_t i = 0; i < S->n_states; i++) free(S->st[i].next);
    free(S->st);
    free(S->is_clone);
    free(S->freq);
    free(S->topk_tok);
    free(S->topk_dst);
    free(S->topk_prob);
    free(S);
}

/* ---- Expand (Algorithm 2) ---------------------------------------------- */

int osam_expand(osam *S, int32_t t)
{
    S->max_length += 1;
    int32_t l = S->max_length;
    int32_t c = expand_state(S, -1, l, l);
    if (c < 0) return -1;
    int32_t p = S->last;
    while (p != -1) {
        S->c_expand_probe++;
        if (next_find(&S->st[p], t) >= 0) break;
        if (next_set(&S->st[p], t, c) < 0) return -1;
        S->n_trans++;
        S->c_insert++;
        p = S->st[p].link;
    }
    if (p == -1) {
        S->st[c].link = 0;
    } else {
        int32_t q = S->st[p].next[next_find(&S->st[p], t)].dst;
        if (S->st[p].length + 1 == S->st[q].length) {
            S->st[c].link = q;
        } else {
            int32_t cl = expand_state(S, -1, -1, -1);
            if (cl < 0) return -1;
            if (cl >= S->cap_clone) {
                int64_t nc = S->cap_clone ? S->cap_clone * 2 : 64;
                while (nc <= cl) nc *= 2;
                uint8_t *nb = (uint8_t *)realloc(S->is_clone, (size_t)nc);
                if (!nb) return -1;
                memset(nb + S->cap_clone, 0, (size_t)(nc - S->cap_clone));
                S->is_clone = nb;
                S->cap_clone = nc;
            }
            S->is_clone[cl] = 1;
            ostate *Q = &S->st[q];
            ostate *C = &S->st[cl];
            C->link = Q->link;
            if (Q->n_next > 0) {
                C->next = (oedge *)malloc((size_t)Q->n_next * sizeof(oedge));
                if (!C->next) return -1;
                memcpy(C->next, Q->next, (size_t)Q->n_next * sizeof(oedge));
            }
            C->n_next = C->cap_next = Q->n_next;
            S->n_trans += Q->n_next;
            S->c_copy += Q->n_next;
            S->c_clone++;
            C->length = S->st[p].length + 1;
            C->min_endpos = Q->min_endpos;
            while (p != -1) {
                S->c_expand_probe++;
                int32_t k = next_find(&S->st[p], t);
                if (k < 0 || S->st[p].next[k].dst != q) break;
                S->st[p].next[k].dst = cl;
                S->c_redirect++;
                p = S->st[p].link;
            }
            S->st[q].link = cl;
            S->st[c].link = cl;
        }
    }
    S->last = c;
    return 0;
}

/* Build-SAM (Algorithm 2): INIT_SAM then Expand per token */
osam *osam_build(const int32_t *tokens, int64_t n)
{
    osam *S = osam_new();
    if (!S) return NULL;
    for (int64_t i = 0; i < n; i++) {
        if (osam_expand(S, tokens[i]) != 0) { osam_free(S); return NULL; }
    }
    return S;
}

/* Expand by a run of tokens (Build-SAM's loop, resumable) */
int osam_extend(osam *S, const int32_t *tokens, int64_t n)
{
    for (int64_t i = 0; i < n; i++)
        if (osam_expand(S, tokens[i]) != 0) return -1;
    return 0;
}

/* ---- Transfer (Algorithm 1) -------------------------------------------- */

void osam_transfer(const osam *S, int32_t t, int32_t *s_io, int32_t *l_io, owalk *w)
{
    int32_t s = *s_io, l = *l_io;
    int32_t k;
    for (;;) {
        if (w) w->probes++;
        k = next_find(&S->st[s], t);
        if (s == 0 || k >= 0) break;
        s = S->st[s].link;
        l = S->st[s].length;
        if (w) w->link_hops++;
    }
    if (k >= 0) {
        s = S->st[s].next[k].dst;
        l = l + 1;
        if (w) w->next_moves++;
    } else {
        l = 0;
    }
    *s_io = s;
    *l_io = l;
}

/* ---- top-k successors and transition probabilities (Algorithm 3) -------- */

static int is_clone_state(const osam *S, int64_t v)
{
    return v < S->cap_clone && S->is_clone[v];
}

/* dfs of Algorithm 3 with an explicit stack (the automaton of a long text is
 * deeper than any call stack): a state's successors are finished first, then
 * its freq is its own start value plus theirs, then its TopK is taken. */
int osam_init_topk(osam *S, int32_t k)
{
    const int64_t n = S->n_states;
    if (k < 1) return -1;
    free(S->freq); free(S->topk_tok); free(S->topk_dst); free(S->topk_prob);
    S->freq = (uint64_t *)calloc((size_t)n, sizeof(uint64_t));
    S->topk_tok = (int32_t *)malloc((size_t)n * k * sizeof(int32_t));
    S->topk_dst = (int32_t *)malloc((size_t)n * k * sizeof(int32_t));
    S->topk_prob = (float *)malloc((size_t)n * k * sizeof(float));
    uint8_t *done = (uint8_t *)calloc((size_t)n, 1);
    int32_t *stack = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *child = (int32_t *)calloc((size_t)n, sizeof(int32_t));   /* next successor to visit */
    if (!S->freq || !S->topk_tok || !S->topk_dst || !S->topk_prob || !done || !stack || !child) {
        free(done); free(stack); free(child);
        return -1;
    }
    S->topk = k;
    for (int64_t v = 0; v < n; v++)
        S->freq[v] = (v == 0 || is_clone_state(S, v)) ? 0 : 1;
    int64_t sp = 0;
    stack[sp++] = 0;                       /* Init_topk: dfs(root) */
    done[0] = 2;                           /* 2 = on the stack, 1 = finished */
    while (sp > 0) {
        int32_t v = stack[sp - 1];
        ostate *st = &S->st[v];
        if (child[v] < st->n_next) {
            int32_t u = st->next[child[v]++].dst;
            if (!done[u]) { done[u] = 2; stack[sp++] = u; }
            continue;
        }
        /* all successors finished */
        for (int32_t j = 0; j < st->n_next; j++) S->freq[v] += S->freq[st->next[j].dst];
        for (int32_t i = 0; i < k; i++) {
            /* i-th largest successor by (freq desc, token asc) not taken yet */
            int32_t best = -1;
            for (int32_t j = 0; j < st->n_next; j++) {
                int taken = 0;
                for (int32_t h = 0; h < i; h++)
                    if (S->topk_tok[(size_t)v * k + h] == st->next[j].token) taken = 1;
                if (taken) continue;
                if (best < 0 || S->freq[st->next[j].dst] > S->freq[st->next[best].dst]) best = j;
            }
            if (best < 0) {
                S->topk_tok[(size_t)v * k + i] = -1;
                S->topk_dst[(size_t)v * k + i] = -1;
                S->topk_prob[(size_t)v * k + i] = 0.0f;
            } else {
                S->topk_tok[(size_t)v * k + i] = st->next[best].token;
                S->topk_dst[(size_t)v * k + i] = st->next[best].dst;
                S->topk_prob[(size_t)v * k + i] =
                    (float)((double)S->freq[st->next[best].dst] / (double)S->freq[v]);
            }
        }
        done[v] = 1;
        sp--;
    }
    free(done); free(stack); free(child);
    return 0;
}

void osam_dump_topk(const osam *S, uint64_t *freq, int32_t *tok, int32_t *dst, float *prob)
{
    memcpy(freq, S->freq, (size_t)S->n_states * sizeof(uint64_t));
    memcpy(tok, S->topk_tok, (size_t)S->n_states * S->topk * sizeof(int32_t));
    memcpy(dst, S->topk_dst, (size_t)S->n_states * S->topk * sizeof(int32_t));
    memcpy(prob, S->topk_prob, (size_t)S->n_states * S->topk * sizeof(float));
}

/* ---- Prim (Algorithm 4): best-first tree draft --------------------------- */

/* Returns the number of draft entries written (<= max_size).  Entry 0 is the
 * start token with parent -1 and probability 1. */
int32_t osam_prim(const osam *S, int32_t s, int32_t t, int32_t max_size,
                  int32_t *tokens, int32_t *parents, float *probs)
{
    const int32_t k = S->topk;
    if (k < 1 || max_size < 1) return 0;
    const int64_t cap = (int64_t)max_size * k + 1;
    float   *qp = (float *)malloc((size_t)cap * sizeof(float));
    int32_t *qs = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    int32_t *qt = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    int32_t *qpar = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    uint8_t *qlive = (uint8_t *)calloc((size_t)cap, 1);
    if (!qp || !qs || !qt || !qpar || !qlive) { free(qp); free(qs); free(qt); free(qpar); free(qlive); return -1; }
    int64_t qn = 0;
    qp[qn] = 1.0f; qs[qn] = s; qt[qn] = t; qpar[qn] = -1; qlive[qn] = 1; qn++;
    int32_t dn = 0;
    while (dn < max_size) {
        /* q.top(): largest probability, the entry pushed first among equals */
        int64_t best = -1;
        for (int64_t i = 0; i < qn; i++)
            if (qlive[i] && (best < 0 || qp[i] > qp[best])) best = i;
        if (best < 0) break;
        qlive[best] = 0;                                   /* q.pop() */
        tokens[dn] = qt[best]; parents[dn] = qpar[best]; probs[dn] = qp[best];
        const int32_t me = dn++;
        const int32_t st = qs[best];
        for (int32_t i = 0; i < k; i++) {
            if (S->topk_dst[(size_t)st * k + i] < 0) continue;
            float pn = qp[best] * S->topk_prob[(size_t)st * k + i];
            qp[qn] = pn; qs[qn] = S->topk_dst[(size_t)st * k + i];
            qt[qn] = S->topk_tok[(size_t)st * k + i]; qpar[qn] = me; qlive[qn] = 1; qn++;
        }
    }
    free(qp); free(qs); free(qt); free(qpar); free(qlive);
    return dn;
}

/* ---- accessors --------------------------------------------------------- */

int64_t osam_num_states(const osam *S) { return S->n_states; }
int64_t osam_num_trans(const osam *S)  { return S->n_trans; }
int32_t osam_last(const osam *S)       { return S->last; }
int32_t osam_max_length(const osam *S) { return S->max_length; }

void osam_state(const osam *S, int64_t s, int32_t *link, int32_t *length,
                int32_t *min_endpos, int32_t *n_next)
{
    *link = S->st[s].link;
    *length = S->st[s].length;
    *min_endpos = S->st[s].min_endpos;
    *n_next = S->st[s].n_next;
}

/* copy the state table out: link/length/min_endpos/n_next, each [n_states] */
void osam_dump_states(const osam *S, int32_t *link, int32_t *length,
                      int32_t *min_endpos, int32_t *n_next)
{
    for (int64_t i = 0; i < S->n_states; i++) {
        link[i] = S->st[i].link;
        length[i] = S->st[i].length;
        min_endpos[i] = S->st[i].min_endpos;
        n_next[i] = S->st[i].n_next;
    }
}

/* transitions of one state, token-sorted; returns how many were written */
int32_t osam_edges(const osam *S, int64_t s, int32_t *tokens, int32_t *dsts, int32_t cap)
{
    int32_t n = S->st[s].n_next < cap ? S->st[s].n_next : cap;
    for (int32_t i = 0; i < n; i++) {
        tokens[i] = S->st[s].next[i].token;
        dsts[i] = S->st[s].next[i].dst;
    }
    return n;
}

/* all transitions as (src, token, dst) triples in state order; returns count */
int64_t osam_dump_trans(const osam *S, int32_t *src, int32_t *tokens, int32_t *dsts)
{
    int64_t k = 0;
    for (int64_t i = 0; i < S->n_states; i++)
        for (int32_t j = 0; j < S->st[i].n_next; j++) {
            src[k] = (int32_t)i;
            tokens[k] = S->st[i].next[j].token;
            dsts[k] = S->st[i].next[j].dst;
            k++;
        }
    return k;
}

void osam_counters(const osam *S, int64_t *out5)
{
    out5[0] = S->c_insert;
    out5[1] = S->c_redirect;
    out5[2] = S->c_clone;
    out5[3] = S->c_copy;
    out5[4] = S->c_expand_probe;
}

/* ---- one decoding sequence: static cursor + its own dynamic automaton --- */

typedef struct {
    const osam    *stat;        /* corpus automaton, may be NULL             */
    const int32_t *corpus;      /* corpus text (borrowed)                    */
    int64_t        corpus_len;
    int32_t        s1, l1;      /* static cursor                             */
    osam          *dyn;         /* automaton of this sequence's own tokens   */
    int32_t        s2, l2;      /* dynamic cursor                            */
    int32_t       *text;        /* this sequence's tokens                    */
    int64_t        text_len, text_cap;
    owalk          w1, w2;
    int64_t        identity_violations;  /* (s2,l2) != (link(last), len(link(last))) */
    int64_t        canon_hops;
} oseq;

oseq *oseq_new(const osam *stat, const int32_t *corpus, int64_t corpus_len)
{
    oseq *q = (oseq *)calloc(1, sizeof(oseq));
    if (!q) return NULL;
    q->stat = stat;
    q->corpus = corpus;
    q->corpus_len = corpus_len;
    q->dyn = osam_new();
    if (!q->dyn) { free(q); return NULL; }
    return q;
}

void oseq_free(oseq *q)
{
    if (!q) return;
    osam_free(q->dyn);
    free(q->text);
    free(q);
}

/* Feed tokens one by one in the order of Section 3.3. */
int oseq_feed(oseq *q, const int32_t *tokens, int32_t count)
{
    for (int32_t i = 0; i < count; i++) {
        int32_t t = tokens[i];
        if (q->stat) osam_transfer(q->stat, t, &q->s1, &q->l1, &q->w1);
        /* dynamic: match against the automaton of the tokens so far, then add t */
        osam_transfer(q->dyn, t, &q->s2, &q->l2, &q->w2);
        if (osam_expand(q->dyn, t) != 0) return -1;
        /* the matched string may now belong to a clone of s2 */
        if (q->s2 != 0 && q->dyn->st[q->dyn->st[q->s2].link].length >= q->l2) {
            q->s2 = q->dyn->st[q->s2].link;
            q->canon_hops++;
        }
        {
            int32_t lk = q->dyn->st[q->dyn->last].link;
            if (q->s2 != lk || q->l2 != q->dyn->st[lk].length) q->identity_violations++;
        }
        if (q->text_len == q->text_cap) {
            int64_t nc = q->text_cap ? q->text_cap * 2 : 256;
            int32_t *nt = (int32_t *)realloc(q->text, (size_t)nc * sizeof(int32_t));
            if (!nt) return -1;
            q->text = nt;
            q->text_cap = nc;
        }
        q->text[q->text_len++] = t;
    }
    return 0;
}

/* Select the source and read the draft.
 * out5 = { match_len, source (0 none, 1 dynamic, 2 static, 3 auxiliary), draft_len,
 *          min_endpos of the chosen state (or -1), chosen state id (or -1) } */
void oseq_draft(const oseq *q, int32_t L, int32_t l_bias, int32_t l_threshold, int32_t *out5,
                int32_t *draft)
{
    int32_t use_static = q->stat && (q->l1 > q->l2 + l_bias);
    int32_t ml = use_static ? q->l1 : q->l2;
    int32_t dl = 0, p = -1, st = -1, src = 0;
    for (int32_t i = 0; i < L; i++) draft[i] = -1;
    if (ml > 0) {
        const int32_t *T;
        int64_t Tn;
        if (use_static) {
            src = 2; st = q->s1; p = q->stat->st[st].min_endpos;
            T = q->corpus; Tn = q->corpus_len;
        } else {
            src = 1; st = q->s2; p = q->dyn->st[st].min_endpos;
            T = q->text; Tn = q->text_len;
        }
        for (int32_t i = 0; i < L && (int64_t)p + i < Tn; i++) {
            draft[i] = T[p + i];
            dl++;
        }
    }
    if (l_threshold >= 0 && ml <= l_threshold) src = 3;
    out5[0] = ml; out5[1] = src; out5[2] = dl; out5[3] = p; out5[4] = st;
}

/* cursors: { s1, l1, s2, l2 } */
void oseq_cursors(const oseq *q, int32_t *out4)
{
    out4[0] = q->s1; out4[1] = q->l1; out4[2] = q->s2; out4[3] = q->l2;
}

const osam *oseq_dynamic(const oseq *q) { return q->dyn; }
int64_t oseq_text_len(const oseq *q)    { return q->text_len; }

/* counters: static walk {probes, link_hops, next_moves}, dynamic walk {same},
 * identity_violations, canon_hops */
void oseq_counters(const oseq *q, int64_t *out8)
{
    out8[0] = q->w1.probes; out8[1] = q->w1.link_hops; out8[2] = q->w1.next_moves;
    out8[3] = q->w2.probes; out8[4] = q->w2.link_hops; out8[5] = q->w2.next_moves;
    out8[6] = q->identity_violations; out8[7] = q->canon_hops;
}

/* One batch step: for every sequence feed its accepted tokens, then select and
 * read the draft.  accepted is [B, A], counts [B]; outputs match_len/source/
 * draft_len [B] and draft [B, L].  A count of 0 leaves the sequence as it is. */
int obatch_step(oseq **seqs, int32_t B, const int32_t *accepted, const int32_t *counts,
                int32_t A, int32_t L, int32_t l_bias, int32_t l_threshold,
                int32_t *match_len, int32_t *source, int32_t *draft_len, int32_t *draft)
{
    for (int32_t b = 0; b < B; b++) {
        int32_t out5[5];
        if (oseq_feed(seqs[b], accepted + (size_t)b * A, counts[b]) != 0) return -1;
        oseq_draft(seqs[b], L, l_bias, l_threshold, out5, draft + (size_t)b * L);
        match_len[b] = out5[0];
        source[b] = out5[1];
        draft_len[b] = out5[2];
    }
    return 0;
}

/* n_steps batch steps in a row: row i of accepted [n_steps, B, A] and counts
 * [n_steps, B] gives row i of match_len/source/draft_len [n_steps, B] and draft
 * [n_steps, B, L].  Nothing but the loop over obatch_step. */
int obatch_run(oseq **seqs, int32_t B, int32_t n_steps, const int32_t *accepted,
               const int32_t *counts, int32_t A, int32_t L, int32_t l_bias, int32_t l_threshold,
               int32_t *match_len, int32_t *source, int32_t *draft_len, int32_t *draft)
{
    for (int32_t i = 0; i < n_steps; i++) {
        const size_t r = (size_t)i * B;
        if (obatch_step(seqs, B, accepted + r * A, counts + r, A, L, l_bias, l_threshold,
                        match_len + r, source + r, draft_len + r, draft + r * L) != 0)
            return -1;
    }
    return 0;
}
