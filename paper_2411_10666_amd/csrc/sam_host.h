// Host-side construction of the static suffix automaton (Build-SAM, Algorithm 2
// of arxiv 2411.10666) directly into the flat arrays the device kernels read.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>

#include "sam_layout.h"

namespace sam {

// Fixed-capacity array on 2 MB pages (the state arrays are read at random while
// building; small pages would make the host TLB the bottleneck).
template <class T>
class HugeArray {
public:
    HugeArray() = default;
    HugeArray(const HugeArray &) = delete;
    HugeArray &operator=(const HugeArray &) = delete;
    ~HugeArray() { release(); }
    bool reserve(size_t cap);            // false: out of memory
    void release();
    void push_back(const T &v) { p_[n_++] = v; }
    void set_size(size_t n) { n_ = n; }  // after reserve(), before filling by index
    T &operator[](size_t i) { return p_[i]; }
    const T &operator[](size_t i) const { return p_[i]; }
    size_t size() const { return n_; }
    const T *data() const { return p_; }

private:
    T *p_ = nullptr;
    size_t n_ = 0;
};

// The fields of one state, side by side: Build-SAM reads several of them whenever it
// comes to a state (length and link on the suffix path; link, end position and list head
// of a state it clones), and each such visit is a cache miss on the host.
struct HostState {
    uint32_t len, link, endpos;
    uint32_t head;   // newest slot of the state's transition list (build only)
};

// state_field[s]: one field of HostState as if it were an array of its own
template <uint32_t HostState::*F>
struct StateField {
    HugeArray<HostState> *a;
    uint32_t &operator[](size_t i) { return (*a)[i].*F; }
    const uint32_t &operator[](size_t i) const { return (*a)[i].*F; }
};

struct HostSam {
    int64_t  n_tokens = 0;
    int32_t  vocab = 0;
    uint32_t n_states = 0;
    uint64_t n_trans = 0;        // all transitions, the root's included
    uint64_t n_buckets = 0;

    std::vector<int32_t>  text;
    HugeArray<HostState>  st;
    StateField<&HostState::len>    len{&st};
    StateField<&HostState::link>   link{&st};
    StateField<&HostState::endpos> endpos{&st};
    StateField<&HostState::head>   head{&st};
    std::vector<RootEnt>  root;  // direct-indexed transitions of the root
    Slot *slots = nullptr;       // n_buckets * 8, 128-byte aligned

    ~HostSam();
    HostSam() = default;
    HostSam(const HostSam &) = delete;
    HostSam &operator=(const HostSam &) = delete;

    // returns SAM_OK or an error code; message in err.  `progress` (may be
    // null) is called now and then with a phase name and done/total counts.
    typedef void (*ProgressFn)(const char *phase, int64_t done, int64_t total, void *user);
    // min_buckets (testing): a transition table of at least that many buckets.
    int build(const int32_t *tokens, int64_t n, int32_t vocab_, std::string &err,
              ProgressFn progress = nullptr, void *user = nullptr, uint64_t min_buckets = 0);

    // Write the built automaton to a file / read it back (same machine byte
    // order, same library layout version).  The top-k table is not stored.
    int save(const char *path, std::string &err) const;
    int load(const char *path, std::string &err);

    // next(state)[token] or kNil
    uint32_t find(uint32_t state, uint32_t token) const;

    // Algorithm 3: freq per state, the k most frequent successors of every state
    // and their probabilities.  Fills freq and topk (n_states * k entries).
    int top_k = 0;
    std::vector<uint64_t> freq;
    std::vector<TopEnt>   topk;
    int build_topk(int k, std::string &err, ProgressFn progress = nullptr, void *user = nullptr);

    // {link, length(link)} per state, for the device
    void make_linkrec(std::vector<LinkPair> &out) const;

};

}  // namespace sam
