// Driver for tests/test_sanitizers.py: the CPU checker (oracle/sam_oracle.c) and the
// library's host builder (csrc/sam_host.cpp) compiled with
// -fsanitize=address,undefined and run over random corpora with many clones, a
// save / load round trip, the top-k pass, the tree draft and the worked example
// "ABCBC" (arxiv 2411.10666: Algorithm 1, Algorithm 2, Appendix A.1-A.2).  The two
// implementations are also compared with each other, state by state and
// transition by transition.  Prints "ok" and returns 0 if everything agreed.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <random>
#include <string>
#include <vector>

#include "../paper_2411_10666_amd/csrc/sam_host.h"

extern "C" {
struct osam;
struct oseq;
osam   *osam_build(const int32_t *tokens, int64_t n);
void    osam_free(osam *S);
int     osam_init_topk(osam *S, int32_t k);
void    osam_dump_topk(const osam *S, uint64_t *freq, int32_t *tok, int32_t *dst, float *prob);
int32_t osam_prim(const osam *S, int32_t s, int32_t t, int32_t max_size, int32_t *tokens,
                  int32_t *parents, float *probs);
int64_t osam_num_states(const osam *S);
int64_t osam_num_trans(const osam *S);
void    osam_dump_states(const osam *S, int32_t *link, int32_t *length, int32_t *min_endpos,
                         int32_t *n_next);
int64_t osam_dump_trans(const osam *S, int32_t *src, int32_t *tokens, int32_t *dsts);
oseq   *oseq_new(const osam *stat, const int32_t *corpus, int64_t corpus_len);
void    oseq_free(oseq *q);
int     oseq_feed(oseq *q, const int32_t *tokens, int32_t count);
void    oseq_draft(const oseq *q, int32_t L, int32_t l_bias, int32_t l_threshold, int32_t *out5,
                   int32_t *draft);
void    oseq_cursors(const oseq *q, int32_t *out4);
}

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); return 1; } \
    } while (0)

static int compare(const std::vector<int32_t> &t, int vocab, int k, const char *tmp_path)
{
    const int64_t n = (int64_t)t.size();
    sam::HostSam h;
    std::string err;
    CHECK(h.build(t.data(), n, vocab, err) == 0);
    osam *o = osam_build(t.data(), n);
    CHECK(o != nullptr);
    const int64_t ns = osam_num_states(o), nt = osam_num_trans(o);
    CHECK(ns == (int64_t)h.n_states && nt == (int64_t)h.n_trans);
    std::vector<int32_t> link(ns), len(ns), endpos(ns), deg(ns);
    osam_dump_states(o, link.data(), len.data(), endpos.data(), deg.data());
    for (int64_t s = 0; s < ns; s++) {
        CHECK((uint32_t)len[s] == h.len[s] && (uint32_t)endpos[s] == h.endpos[s]);
        CHECK(link[s] == (h.link[s] == sam::kNil ? -1 : (int32_t)h.link[s]));
    }
    std::vector<int32_t> src(nt), tok(nt), dst(nt);
    CHECK(osam_dump_trans(o, src.data(), tok.data(), dst.data()) == nt);
    for (int64_t i = 0; i < nt; i++) CHECK(h.find((uint32_t)src[i], (uint32_t)tok[i]) == (uint32_t)dst[i]);
    uint64_t found = 0;
    for (uint32_t s = 0; s < h.n_states && s < 400; s++)
        for (int a = 0; a < vocab; a++)
            if (h.find(s, (uint32_t)a) != sam::kNil) found++;
    uint64_t want = 0;
    for (int64_t s = 0; s < ns && s < 400; s++) want += (uint64_t)deg[s];
    CHECK(found == want);

    // top-k and the tree draft
    CHECK(h.build_topk(k, err) == 0);
    CHECK(osam_init_topk(o, k) == 0);
    std::vector<uint64_t> freq(ns);
    std::vector<int32_t> ttok(ns * k), tdst(ns * k);
    std::vector<float> tprob(ns * k);
    osam_dump_topk(o, freq.data(), ttok.data(), tdst.data(), tprob.data());
    for (int64_t s = 0; s < ns; s++) {
        CHECK(freq[s] == h.freq[s]);
        for (int i = 0; i < k; i++) {
            const sam::TopEnt &e = h.topk[(size_t)s * k + i];
            if (tdst[s * k + i] < 0) { CHECK(e.dst == 0); continue; }
            CHECK(e.token == (uint32_t)ttok[s * k + i] && e.dst == (uint32_t)tdst[s * k + i] &&
                  e.prob == tprob[s * k + i]);
        }
    }
    std::vector<int32_t> dt(24), dp(24);
    std::vector<float> dpr(24);
    const int32_t got = osam_prim(o, (int32_t)(ns / 2), 0, 24, dt.data(), dp.data(), dpr.data());
    CHECK(got >= 1 && got <= 24 && dp[0] == -1);

    // the link records handed to the device
    std::vector<sam::LinkPair> lr;
    h.make_linkrec(lr);
    for (int64_t s = 1; s < ns; s++) CHECK(lr[s].link == (uint32_t)link[s] && lr[s].lenlink == (uint32_t)len[link[s]]);

    // file round trip
    if (tmp_path) {
        CHECK(h.save(tmp_path, err) == 0);
        sam::HostSam g;
        CHECK(g.load(tmp_path, err) == 0);
        CHECK(g.n_states == h.n_states && g.n_trans == h.n_trans && g.n_buckets == h.n_buckets);
        for (int64_t i = 0; i < nt; i++) CHECK(g.find((uint32_t)src[i], (uint32_t)tok[i]) == (uint32_t)dst[i]);
        remove(tmp_path);
    }

    // a sequence walking both automata (Section 3.3 order), drafts read after every token
    oseq *q = oseq_new(o, t.data(), n);
    CHECK(q != nullptr);
    std::mt19937 g2((uint32_t)n);
    for (int i = 0; i < 300; i++) {
        int32_t x = (i % 7 < 4 && i < n) ? t[(size_t)((i * 31) % n)] : (int32_t)(g2() % vocab);
        CHECK(oseq_feed(q, &x, 1) == 0);
        int32_t out5[5], draft[8];
        oseq_draft(q, 8, 0, -1, out5, draft);
        CHECK(out5[2] >= 0 && out5[2] <= 8);
    }
    oseq_free(q);
    osam_free(o);
    return 0;
}

int main(int argc, char **argv)
{
    const char *tmp = argc > 1 ? argv[1] : nullptr;
    std::mt19937 g(12345);
    for (int it = 0; it < 60; it++) {
        const int vocab = 2 + (int)(g() % 6);
        const int n = 1 + (int)(g() % 2500);
        std::vector<int32_t> t((size_t)n);
        for (auto &x : t) x = (int32_t)(g() % vocab);
        // repeated stretches make clones and long suffix paths
        for (int r = 0; r < 6 && n > 40; r++) {
            const int len = 5 + (int)(g() % 30), a = (int)(g() % (n - len)), b = (int)(g() % (n - len));
            memmove(&t[(size_t)b], &t[(size_t)a], (size_t)len * sizeof(int32_t));
        }
        if (compare(t, vocab, 1 + (int)(g() % 8), it % 10 == 0 ? tmp : nullptr)) return 1;
    }
    // a^m b: every state on one suffix path
    {
        std::vector<int32_t> t(500, 0);
        t.push_back(1);
        if (compare(t, 2, 2, nullptr)) return 1;
    }
    // the worked example "ABCBC" fed "CBCA" (static) and itself (dynamic)
    {
        const int32_t text[5] = {0, 1, 2, 1, 2};
        osam *o = osam_build(text, 5);
        CHECK(o && osam_num_states(o) == 8 && osam_num_trans(o) == 9);
        oseq *q = oseq_new(o, text, 5);
        const int32_t feed[4] = {2, 1, 2, 0};
        const int32_t want_state[4] = {7, 4, 6, 1}, want_len[4] = {1, 2, 3, 1};
        for (int i = 0; i < 4; i++) {
            CHECK(oseq_feed(q, &feed[i], 1) == 0);
            int32_t cur[4];
            oseq_cursors(q, cur);
            CHECK(cur[0] == want_state[i] && cur[1] == want_len[i]);
        }
        oseq_free(q);
        osam_free(o);
    }
    printf("ok\n");
    return 0;
}
