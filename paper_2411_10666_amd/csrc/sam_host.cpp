// Build-SAM on the host (Algorithm 2, Appendix A.1 of arxiv 2411.10666), written
// straight into the device layout: state fields in flat arrays, the root's
// transitions in a direct-indexed table, all other transitions in the bucketed
// open-addressed hash.  While building, Slot::w chains each state's slots so a
// clone can enumerate the transitions it copies; the last pass overwrites it
// with min_endpos(target), which is what the device wants there.
#include "sam_host.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>

#include <atomic>
#include <new>
#include <thread>

#include "../../include/sam.h"

namespace sam {

HostSam::~HostSam() { free(slots); }

namespace {
constexpr size_t kHuge = 2u << 20;
void *huge_alloc(size_t bytes)
{
    const size_t rounded = (bytes + kHuge - 1) / kHuge * kHuge;
    void *p = aligned_alloc(kHuge, rounded);
    if (p) (void)madvise(p, rounded, MADV_HUGEPAGE);
    return p;
}

// Run fn(lo, hi) over [0, n) cut into one contiguous range per worker thread.  The
// passes that use it (token check, table clear, the end-position pass, the link
// records) touch every element once and independently; Build-SAM itself is
// sequential and stays on the calling thread.
template <class F>
void parallel_ranges(uint64_t n, F fn)
{
    unsigned hw = std::thread::hardware_concurrency();
    unsigned workers = hw < 1 ? 1 : (hw > 16 ? 16 : hw);
    if (n < (1u << 20)) workers = 1;
    if (workers == 1) { fn((uint64_t)0, n); return; }
    std::vector<std::thread> pool;
    const uint64_t per = (n + workers - 1) / workers;
    try {
        for (unsigned w = 1; w < workers; w++) {
            const uint64_t lo = per * w, hi = lo + per < n ? lo + per : n;
            if (lo < hi) pool.emplace_back([=] { fn(lo, hi); });
        }
    } catch (...) {
        // no more threads to be had: the calling thread does what is left
        const uint64_t done = per * (1 + pool.size());
        if (done < n) fn(done, n);
    }
    fn((uint64_t)0, per < n ? per : n);
    for (auto &t : pool) t.join();
}
}  // namespace

template <class T>
bool HugeArray<T>::reserve(size_t cap)
{
    release();
    p_ = (T *)huge_alloc(cap * sizeof(T));
    return p_ != nullptr;
}

template <class T>
void HugeArray<T>::release()
{
    free(p_);
    p_ = nullptr;
    n_ = 0;
}

template class HugeArray<uint32_t>;
template class HugeArray<HostState>;

namespace {

// Probe for (state, token).  Returns the slot index if present; otherwise kNil64
// and *empty_at = first empty slot on the probe path (where an insert goes).
constexpr uint64_t kNil64 = ~0ull;

inline uint64_t probe(const Slot *slots, uint64_t n_buckets, uint32_t state, uint32_t token,
                      uint64_t *empty_at)
{
    uint64_t b = bucket_of(hash_key(state, token), n_buckets);
    for (;;) {
        const Slot *s = slots + b * kBucketSlots;
        for (int i = 0; i < kBucketSlots; i++) {
            if (s[i].state == state && s[i].token == token) return b * kBucketSlots + i;
            if (s[i].state == kNil) {
                if (empty_at) *empty_at = b * kBucketSlots + i;
                return kNil64;
            }
        }
        if (++b == n_buckets) b = 0;
    }
}

}  // namespace

int HostSam::build(const int32_t *tokens, int64_t n, int32_t vocab_, std::string &err,
                   ProgressFn progress, void *user, uint64_t min_buckets)
{
    if (!tokens || n < 1 || n > 0x7FFFFFFELL || vocab_ < 1) {
        err = "sam_build: need tokens != NULL, 1 <= n_tokens <= 2^31-2, vocab >= 1";
        return SAM_EINVAL;
    }
    {
        std::atomic<int64_t> first_bad(n);
        parallel_ranges((uint64_t)n, [&](uint64_t lo, uint64_t hi) {
            for (uint64_t i = lo; i < hi; i++)
                if (tokens[i] < 0 || tokens[i] >= vocab_) {
                    int64_t seen = first_bad.load();
                    while ((int64_t)i < seen && !first_bad.compare_exchange_weak(seen, (int64_t)i)) {}
                    return;
                }
        });
        const int64_t i = first_bad.load();
        if (i < n) {
            err = "sam_build: corpus token " + std::to_string(tokens[i]) + " at position " +
                  std::to_string(i) + " is outside [0, vocab)";
            return SAM_ETOKEN;
        }
    }
    n_tokens = n;
    vocab = vocab_;
    n_buckets = static_buckets_for(n);
    if (n_buckets < min_buckets) n_buckets = min_buckets;
    const uint64_t n_slots = n_buckets * kBucketSlots;
    if (n_slots >= 0xFFFFFFFFull) {
        err = "sam_build: corpus too large for 32-bit slot indices";
        return SAM_EINVAL;
    }
    try {
        text.assign(tokens, tokens + n);
        root.assign((size_t)vocab, RootEnt{0, 0});
    } catch (const std::bad_alloc &) {
        err = "sam_build: out of host memory for the corpus text";
        return SAM_ENOMEM;
    }
    const size_t cap = (size_t)2 * n + 2;     // states <= 2n - 1 (n >= 2), 2 for n = 1
    if (!st.reserve(cap)) {
        err = "sam_build: out of host memory for the state arrays";
        return SAM_ENOMEM;
    }
    // the table is probed at random: 2 MB pages keep the host TLB out of the way
    slots = (Slot *)huge_alloc(n_slots * sizeof(Slot));
    if (!slots) {
        err = "sam_build: out of host memory for the transition table";
        return SAM_ENOMEM;
    }
    parallel_ranges(n_slots, [&](uint64_t lo, uint64_t hi) {
        memset(slots + lo, 0xFF, (hi - lo) * sizeof(Slot));
    });

    auto new_state = [&](uint32_t l, uint32_t lk, uint32_t ep) -> uint32_t {
        st.push_back(HostState{l, lk, ep, kNil});
        return n_states++;
    };
    auto put = [&](uint64_t at, uint32_t state, uint32_t token, uint32_t dst) {
        slots[at] = Slot{state, token, dst, head[state]};
        head[state] = (uint32_t)at;
        n_trans++;
    };

    new_state(0, kNil, 0);     // root
    uint32_t last = 0;

    for (int64_t i = 0; i < n; i++) {
        if (progress && (i & ((1 << 24) - 1)) == 0) progress("build", i, n, user);
        const uint32_t t = (uint32_t)tokens[i];
        const uint32_t c = new_state((uint32_t)(i + 1), 0, (uint32_t)(i + 1));
        // the next token's first insert goes into the bucket of (c, next token): ask for
        // that line now, one token of work ahead of its use
        if (i + 1 < n)
            __builtin_prefetch(slots + bucket_of(hash_key(c, (uint32_t)tokens[i + 1]), n_buckets) *
                                           kBucketSlots, 1, 0);
        uint32_t p = last;
        uint32_t q = kNil;
        uint64_t at = kNil64;          // slot of (p, t) when p is not the root
        // give t-transitions to the states on last's suffix path that lack one
        while (p != kNil) {
            if (p == 0) {
                if (root[t].dst) { q = root[t].dst; break; }
                root[t].dst = c;
                n_trans++;
                p = kNil;
            } else {
                uint64_t empty_at = 0;
                at = probe(slots, n_buckets, p, t, &empty_at);
                if (at != kNil64) { q = slots[at].dst; break; }
                put(empty_at, p, t, c);
                p = link[p];
            }
        }
        if (p == kNil) {
            link[c] = 0;
        } else if (len[p] + 1 == len[q]) {
            link[c] = q;
        } else {
            const uint32_t cl = new_state(len[p] + 1, link[q], endpos[q]);
            for (uint32_t j = head[q]; j != kNil; j = slots[j].w) {
                uint64_t empty_at = 0;
                probe(slots, n_buckets, cl, slots[j].token, &empty_at);
                put(empty_at, cl, slots[j].token, slots[j].dst);
            }
            // states further up the path that still point at q now point at the clone
            while (p != kNil) {
                if (p == 0) {
                    if (root[t].dst != q) break;
                    root[t].dst = cl;
                    p = kNil;
                } else {
                    if (at == kNil64) at = probe(slots, n_buckets, p, t, nullptr);
                    if (at == kNil64 || slots[at].dst != q) break;
                    slots[at].dst = cl;
                    p = link[p];
                    at = kNil64;
                }
            }
            link[q] = cl;
            link[c] = cl;
        }
        last = c;
        // the next token's walk continues at link(c): its bucket and its state fields
        if (i + 1 < n && link[c] != 0) {
            const uint32_t up = link[c];
            __builtin_prefetch(slots + bucket_of(hash_key(up, (uint32_t)tokens[i + 1]), n_buckets) *
                                           kBucketSlots, 0, 0);
            __builtin_prefetch(&st[up], 1, 0);
        }
    }

    // the device reads min_endpos(target) where the build kept the list chain
    if (progress) progress("finalize", 0, (int64_t)n_slots, user);
    parallel_ranges(n_slots, [&](uint64_t lo, uint64_t hi) {
        for (uint64_t j = lo; j < hi; j++)
            if (slots[j].state != kNil) slots[j].w = endpos[slots[j].dst];
    });
    for (int32_t t = 0; t < vocab; t++)
        if (root[t].dst) root[t].endpos = endpos[root[t].dst];
    return SAM_OK;
}

// Algorithm 3 without recursion and without per-state transition lists: a
// transition p -> q always has len(q) > len(p), so when the transitions are
// taken in order of decreasing len(p), freq(q) is final by the time it is added
// to freq(p).  freq starts at 1 for states made by expansion, 0 for clones (and
// for the root); a state is a clone iff its length differs from its min_endpos.
int HostSam::build_topk(int k, std::string &err, ProgressFn progress, void *user)
{
    if (k < 1 || k > kMaxTopK) {
        err = "sam_corpus_build_topk: k must be in 1 .. " + std::to_string(kMaxTopK);
        return SAM_EINVAL;
    }
    const uint64_t n_slots = n_buckets * kBucketSlots;
    std::vector<uint32_t> order;      // used slots, by decreasing length of the source state
    std::vector<uint64_t> start;      // counting sort over lengths 0 .. n_tokens
    std::vector<uint64_t> topf;       // freq of the entries of topk, while selecting
    try {
        freq.assign(n_states, 0);
        topk.assign((size_t)n_states * k, TopEnt{0, 0, 0.0f});
        topf.assign((size_t)n_states * k, 0);
        start.assign((size_t)n_tokens + 2, 0);
        order.resize(n_trans);
    } catch (const std::bad_alloc &) {
        err = "sam_corpus_build_topk: out of host memory";
        return SAM_ENOMEM;
    }
    for (uint32_t s = 1; s < n_states; s++) freq[s] = len[s] == endpos[s] ? 1 : 0;
    if (progress) progress("topk-sort", 0, 3, user);
    uint64_t used = 0;
    for (uint64_t j = 0; j < n_slots; j++)
        if (slots[j].state != kNil) { start[len[slots[j].state] + 1]++; used++; }
    for (size_t l = 1; l < start.size(); l++) start[l] += start[l - 1];
    for (uint64_t j = 0; j < n_slots; j++)
        if (slots[j].state != kNil) order[start[len[slots[j].state]]++] = (uint32_t)j;
    if (progress) progress("topk-freq", 1, 3, user);
    for (uint64_t i = used; i-- > 0;) {
        const Slot &e = slots[order[i]];
        freq[e.state] += freq[e.dst];
    }
    for (int32_t t = 0; t < vocab; t++)
        if (root[t].dst) freq[0] += freq[root[t].dst];
    if (progress) progress("topk-select", 2, 3, user);
    // keep the k best successors of each state by (freq desc, token asc)
    auto offer = [&](uint32_t state, uint32_t token, uint32_t dst) {
        TopEnt *e = &topk[(size_t)state * k];
        uint64_t *f = &topf[(size_t)state * k];
        const uint64_t fd = freq[dst];
        int pos = k;
        while (pos > 0 && (e[pos - 1].dst == 0 || fd > f[pos - 1] ||
                           (fd == f[pos - 1] && token < e[pos - 1].token)))
            pos--;
        if (pos == k) return;
        for (int i = k - 1; i > pos; i--) { e[i] = e[i - 1]; f[i] = f[i - 1]; }
        e[pos] = TopEnt{token, dst, 0.0f};
        f[pos] = fd;
    };
    for (uint64_t j = 0; j < n_slots; j++)
        if (slots[j].state != kNil) offer(slots[j].state, slots[j].token, slots[j].dst);
    for (int32_t t = 0; t < vocab; t++)
        if (root[t].dst) offer(0, (uint32_t)t, root[t].dst);
    for (uint32_t s = 0; s < n_states; s++)
        for (int i = 0; i < k; i++) {
            TopEnt &e = topk[(size_t)s * k + i];
            if (e.dst) e.prob = (float)((double)topf[(size_t)s * k + i] / (double)freq[s]);
        }
    top_k = k;
    return SAM_OK;
}

// ---- file format -----------------------------------------------------------
// header (64 bytes): magic "SAMCORP1", layout version, bucket width, n_tokens,
// vocab, n_states, n_trans, n_buckets; then the arrays in the order text, len,
// link, endpos, root, slots, each as raw bytes.

namespace {

struct FileHeader {
    char     magic[8];
    uint32_t version;
    uint32_t bucket_slots;
    int64_t  n_tokens;
    int64_t  vocab;
    uint64_t n_states;
    uint64_t n_trans;
    uint64_t n_buckets;
    uint64_t reserved;
};
static_assert(sizeof(FileHeader) == 64, "file header is 64 bytes");
constexpr char kMagic[8] = {'S', 'A', 'M', 'C', 'O', 'R', 'P', '1'};
constexpr uint32_t kFileVersion = 1;

bool write_all(FILE *f, const void *p, size_t bytes)
{
    const char *c = (const char *)p;
    while (bytes) {
        const size_t chunk = bytes < ((size_t)1 << 30) ? bytes : ((size_t)1 << 30);
        if (fwrite(c, 1, chunk, f) != chunk) return false;
        c += chunk;
        bytes -= chunk;
    }
    return true;
}

bool read_all(FILE *f, void *p, size_t bytes)
{
    char *c = (char *)p;
    while (bytes) {
        const size_t chunk = bytes < ((size_t)1 << 30) ? bytes : ((size_t)1 << 30);
        if (fread(c, 1, chunk, f) != chunk) return false;
        c += chunk;
        bytes -= chunk;
    }
    return true;
}

}  // namespace

int HostSam::save(const char *path, std::string &err) const
{
    FILE *f = fopen(path, "wb");
    if (!f) { err = std::string("sam_corpus_save: cannot open ") + path; return SAM_EINVAL; }
    FileHeader h = {};
    memcpy(h.magic, kMagic, 8);
    h.version = kFileVersion;
    h.bucket_slots = kBucketSlots;
    h.n_tokens = n_tokens; h.vocab = vocab; h.n_states = n_states; h.n_trans = n_trans;
    h.n_buckets = n_buckets;
    // the file keeps length, link and end position as three arrays
    auto write_field = [&](uint32_t HostState::*field) {
        std::vector<uint32_t> chunk;
        for (uint64_t lo = 0; lo < n_states; lo += 1u << 20) {
            const uint64_t hi = lo + (1u << 20) < n_states ? lo + (1u << 20) : n_states;
            chunk.resize((size_t)(hi - lo));
            for (uint64_t s = lo; s < hi; s++) chunk[(size_t)(s - lo)] = st[s].*field;
            if (!write_all(f, chunk.data(), chunk.size() * sizeof(uint32_t))) return false;
        }
        return true;
    };
    const bool ok = write_all(f, &h, sizeof(h)) &&
                    write_all(f, text.data(), (size_t)n_tokens * sizeof(int32_t)) &&
                    write_field(&HostState::len) && write_field(&HostState::link) &&
                    write_field(&HostState::endpos) &&
                    write_all(f, root.data(), (size_t)vocab * sizeof(RootEnt)) &&
                    write_all(f, slots, (size_t)n_buckets * kBucketSlots * sizeof(Slot));
    const bool closed = fclose(f) == 0;
    if (!ok || !closed) { err = std::string("sam_corpus_save: write failed on ") + path; return SAM_EINVAL; }
    return SAM_OK;
}

int HostSam::load(const char *path, std::string &err)
{
    FILE *f = fopen(path, "rb");
    if (!f) { err = std::string("sam_corpus_load: cannot open ") + path; return SAM_EINVAL; }
    FileHeader h;
    int rc = SAM_OK;
    if (!read_all(f, &h, sizeof(h)) || memcmp(h.magic, kMagic, 8) != 0 ||
        h.version != kFileVersion || h.bucket_slots != (uint32_t)kBucketSlots) {
        err = std::string("sam_corpus_load: ") + path + " is not an automaton file of this library version";
        rc = SAM_EINVAL;
    } else if (h.n_tokens < 1 || h.n_tokens > 0x7FFFFFFELL || h.vocab < 1 || h.vocab > 0x7FFFFFFFLL ||
               h.n_states < 2 || h.n_states > 2 * (uint64_t)h.n_tokens + 1 ||
               h.n_buckets < static_buckets_for(h.n_tokens) ||
               h.n_buckets * kBucketSlots >= 0xFFFFFFFFull) {
        err = std::string("sam_corpus_load: inconsistent header in ") + path;
        rc = SAM_EINVAL;
    }
    if (rc == SAM_OK) {
        n_tokens = h.n_tokens; vocab = (int32_t)h.vocab; n_states = (uint32_t)h.n_states;
        n_trans = h.n_trans; n_buckets = h.n_buckets;
        const size_t n_slots = (size_t)n_buckets * kBucketSlots;
        try {
            text.resize((size_t)n_tokens);
            root.resize((size_t)vocab);
        } catch (const std::bad_alloc &) {
            rc = SAM_ENOMEM;
        }
        free(slots);
        slots = nullptr;
        if (rc == SAM_OK && (!st.reserve(n_states) ||
                             !(slots = (Slot *)huge_alloc(n_slots * sizeof(Slot)))))
            rc = SAM_ENOMEM;
        if (rc != SAM_OK) {
            err = "sam_corpus_load: out of host memory";
        } else {
            st.set_size(n_states);
            auto read_field = [&](uint32_t HostState::*field) {
                std::vector<uint32_t> chunk;
                for (uint64_t lo = 0; lo < n_states; lo += 1u << 20) {
                    const uint64_t hi = lo + (1u << 20) < n_states ? lo + (1u << 20) : n_states;
                    chunk.resize((size_t)(hi - lo));
                    if (!read_all(f, chunk.data(), chunk.size() * sizeof(uint32_t))) return false;
                    for (uint64_t s = lo; s < hi; s++) st[s].*field = chunk[(size_t)(s - lo)];
                }
                return true;
            };
            for (uint64_t s = 0; s < n_states; s++) st[s].head = kNil;
            const bool ok = read_all(f, text.data(), (size_t)n_tokens * sizeof(int32_t)) &&
                            read_field(&HostState::len) && read_field(&HostState::link) &&
                            read_field(&HostState::endpos) &&
                            read_all(f, root.data(), (size_t)vocab * sizeof(RootEnt)) &&
                            read_all(f, slots, n_slots * sizeof(Slot));
            char extra;
            if (!ok || fread(&extra, 1, 1, f) != 0) {
                err = std::string("sam_corpus_load: ") + path + " is truncated or has trailing bytes";
                rc = SAM_EINVAL;
            }
        }
    }
    fclose(f);
    if (rc != SAM_OK) return rc;
    // cheap structural checks, so that a damaged file cannot send a kernel out of bounds
    if (len[0] != 0 || link[0] != kNil) { err = "sam_corpus_load: bad root record"; return SAM_EINVAL; }
    for (uint32_t s = 1; s < n_states; s++)
        if (link[s] >= n_states || len[link[s]] >= len[s] || endpos[s] > (uint64_t)n_tokens ||
            len[s] > endpos[s]) {
            err = "sam_corpus_load: state " + std::to_string(s) + " is inconsistent";
            return SAM_EINVAL;
        }
    uint64_t used = 0;
    const uint64_t n_slots = n_buckets * kBucketSlots;
    for (uint64_t j = 0; j < n_slots; j++)
        if (slots[j].state != kNil) {
            used++;
            if (slots[j].state >= n_states || slots[j].dst == 0 || slots[j].dst >= n_states ||
                slots[j].token >= (uint32_t)vocab || slots[j].w != endpos[slots[j].dst]) {
                err = "sam_corpus_load: transition slot " + std::to_string(j) + " is inconsistent";
                return SAM_EINVAL;
            }
        }
    for (int32_t t = 0; t < vocab; t++)
        if (root[t].dst) {
            used++;
            if (root[t].dst >= n_states || root[t].endpos != endpos[root[t].dst]) {
                err = "sam_corpus_load: root transition " + std::to_string(t) + " is inconsistent";
                return SAM_EINVAL;
            }
        }
    if (used != n_trans) { err = "sam_corpus_load: transition count does not match"; return SAM_EINVAL; }
    if (n_slots - (used - 0) < 1) { err = "sam_corpus_load: transition table is full"; return SAM_EINVAL; }
    return SAM_OK;
}

uint32_t HostSam::find(uint32_t state, uint32_t token) const
{
    if (state >= n_states || token >= (uint32_t)vocab) return kNil;
    if (state == 0) return root[token].dst ? root[token].dst : kNil;
    uint64_t at = probe(slots, n_buckets, state, token, nullptr);
    return at == kNil64 ? kNil : slots[at].dst;
}

void HostSam::make_linkrec(std::vector<LinkPair> &out) const
{
    out.resize(n_states);
    parallel_ranges(n_states, [&](uint64_t lo, uint64_t hi) {
        for (uint64_t s = lo ? lo : 1; s < hi; s++) out[s] = LinkPair{link[s], len[link[s]]};
    });
    out[0] = LinkPair{0, 0};
}


}  // namespace sam
