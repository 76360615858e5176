// Memory layout shared by the host builder and the gfx950 kernels.
//
// The paper keeps, per state, link / next / length / min_endpos (Appendix A.1)
// and leaves the storage open.  Here every automaton is a set of flat arrays:
//
//  static automaton (read-only on the device)
//    text[n]                 int32 corpus
//    linkrec[n_states]       {link, length(link)}                       8 B
//    root[vocab]             {target, min_endpos(target)}, target 0 = none  8 B
//    slots[n_buckets * 8]    {state, token, target, min_endpos(target)} 16 B
//                            open addressing, 128-byte buckets of 8 slots,
//                            linear over buckets; root's transitions are not
//                            in it (they are in root[]).
//
//  dynamic automaton (one private region per sequence)
//    text[max_seq_len]       int32
//    rec[2 * max_seq_len]    {length, link, min_endpos, head,
//                             itok, idst, -, -}                         32 B
//                            itok/idst: the state's first transition, kept
//                            inline; head: newest of its further transitions
//                            in slots[], chained through Slot::w.
//    slots[n_buckets * 8]    {state, token, target, next-in-state-list} 16 B
#pragma once
#include <stdint.h>

namespace sam {

constexpr uint32_t kNil   = 0xFFFFFFFFu;   // "no state" / "no slot" / empty key
constexpr int      kBucketSlots = 8;       // 8 x 16 B = one 128-byte line

struct Slot {            // 16 B
    uint32_t state;      // source state, kNil = empty slot
    uint32_t token;
    uint32_t dst;
    uint32_t w;          // static: min_endpos(dst); dynamic and host build: next slot of `state`
};

struct LinkRec {         // 8 B, static automaton
    uint32_t link;
    uint32_t lenlink;
};

struct RootEnt {         // 8 B, static automaton; dst == 0 means no transition
    uint32_t dst;
    uint32_t endpos;
};

struct DynRec {          // 32 B, dynamic automaton
    uint32_t len;
    uint32_t link;       // kNil for the root
    uint32_t endpos;
    uint32_t head;       // kNil = no transitions in slots[]
    uint32_t itok;       // kNil = no inline transition
    uint32_t idst;
    uint32_t pad0;
    uint32_t pad1;
};

// per-sequence bookkeeping, 64 B
struct SeqMeta {
    uint32_t s1, l1, e1;     // static cursor: state, match length, min_endpos(state)
    uint32_t s2, l2, e2;     // dynamic cursor = link(last): state, its length, its min_endpos
    uint32_t n;              // tokens in the sequence so far
    uint32_t n_states;
    uint32_t last;
    uint32_t n_trans;
    uint32_t status;
    uint32_t pad[5];
};

// (state, token) -> 32-bit hash; the same function on host and device
#if defined(__HIPCC__) || defined(__CUDACC__)
__host__ __device__
#endif
inline uint32_t hash_key(uint32_t state, uint32_t token)
{
    uint32_t h = state * 0x9E3779B1u + token * 0x85EBCA77u;
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 12;
    h *= 0x297A2D39u;
    h ^= h >> 15;
    return h;
}

// map a 32-bit hash onto [0, n_buckets) without a modulo
#if defined(__HIPCC__) || defined(__CUDACC__)
__host__ __device__
#endif
inline uint64_t bucket_of(uint32_t h, uint64_t n_buckets)
{
    return ((uint64_t)h * n_buckets) >> 32;
}

inline uint64_t static_buckets_for(int64_t n_tokens)
{
    // transitions <= 3n; sized so that the usual ~2.1n gives a load near 0.5
    uint64_t slots = (uint64_t)((double)n_tokens * 3.0 / 0.70) + 64;
    return (slots + kBucketSlots - 1) / kBucketSlots;
}

inline uint64_t dynamic_buckets_for(int64_t max_seq_len)
{
    // <= 3T transitions in the worst case -> load <= 0.75
    uint64_t slots = (uint64_t)max_seq_len * 4 + 64;
    return (slots + kBucketSlots - 1) / kBucketSlots;
}

}  // namespace sam
