// Memory layout shared by the host builder and the gfx950 kernels.
//
// The paper keeps, per state, link / next / length / min_endpos (Appendix A.1)
// and leaves the storage open.  Here every automaton is a set of flat arrays:
//
//  static automaton (read-only on the device)
//    text[n]                 int32 corpus
//    linkrec[n_states]       {two transitions inline, link, length(link)} 32 B
//    root[vocab]             {target, min_endpos(target)}, target 0 = none  8 B
//    slots[n_buckets * 8]    {state, token, target, min_endpos(target)} 16 B
//                            open addressing, 128-byte buckets of 8 slots,
//                            linear over buckets; root's transitions are not
//                            in it (they are in root[]).
//    Every min_endpos(target) and every length(link) on the device carries, in
//    bit 31, whether the state it leads to is WIDE: has more than the two
//    transitions its record repeats.  Only a wide state's lookups need a bucket.
//    topk[n_states * k]      {token, target, probability}, optional     12 B
//                            (Algorithm 3; only for tree drafts)
//
//  dynamic automaton (one private region per sequence), two layouts:
//    text[max_seq_len]       int32
//   wide (any max_seq_len, any vocabulary)
//    rec[2 * max_seq_len+2]  {length, link, min_endpos, head,
//                             itok, idst, -, -}                         32 B
//    slots[n_buckets * 8]    {state, token, target, next-in-state-list} 16 B
//   compact (max_seq_len <= 16366 and vocab <= 2^17: 15-bit state ids)
//    rec[2 * max_seq_len+2]  {length:16, link:16, min_endpos:16, head:16,
//                             itok:32, idst:16, -:16}                   16 B
//    slots[n_buckets * 16]   {key = state << 17 | token : 32,
//                             target:16, next:16}                        8 B
//   itok/idst: the state's first transition, kept inline; head: newest of its
//   further transitions in slots[], chained through the slot's `next`.
//   A sequence of T tokens has at most T - 1 transitions outside the records
//   (transitions <= states + T - 2, and every state but the newest has one
//   inline), so 2T slots keep the table at most half full.
#pragma once
#include <stdint.h>

namespace sam {

constexpr uint32_t kNil   = 0xFFFFFFFFu;   // "no state" / "no slot" / empty key
constexpr int      kBucketSlots = 8;       // 8 x 16 B = one 128-byte line

struct Slot {            // 16 B
    uint32_t state;      // source state, kNil = empty slot
    uint32_t token;
    uint32_t dst;
    uint32_t w;          // static: min_endpos(dst) (on the device | wide(dst) << 31);
                         // dynamic and host build: next slot of `state`
};

struct LinkPair {        // 8 B: what the host hands over per state
    uint32_t link;
    uint32_t lenlink;    // len(link)
};

// 32 B per state of the static automaton, built on the device from the link
// pairs and the slot table.  Besides the suffix link it repeats TWO of the
// state's transitions: first those to states created after it, nearest first,
// then those to older states, lowest id first.  For a state that stands for a
// prefix of the corpus the first one is the transition to the next prefix, whose
// record is the next or next-but-one in this array -- so while a sequence follows
// a stretch of the corpus, its lookups read consecutive records (four to a cache
// line) instead of one random bucket each.  A state with at most two transitions
// (most states: the deep ones) is answered by its record alone, hit or miss, and
// the slot table the device keeps holds the transitions of the other states only.
struct LinkRec {
    uint32_t itok;       // token of the first repeated transition, kNil = none
    uint32_t idst;       // its target
    uint32_t iendpos;    // min_endpos(target) | wide(target) << 31
    uint32_t itok2;      // the second one, kNil = none
    uint32_t idst2;
    uint32_t iendpos2;
    uint32_t link;       // link(s) (0 for the root and for states of length 1)
    uint32_t lenlink;    // len(link(s)) | wide(link(s)) << 31
};

constexpr uint32_t kWideBit = 0x80000000u;   // see above; lengths and end positions are < 2^31

struct RootEnt {         // 8 B, static automaton; dst == 0 means no transition
    uint32_t dst;
    uint32_t endpos;     // on the device: | wide(dst) << 31
};

struct TopEnt {          // 12 B, static automaton, k per state; dst == 0 means unused
    uint32_t token;
    uint32_t dst;
    float    prob;       // freq(dst) / freq(state)
};

constexpr int kMaxTopK = 8;
constexpr int kMaxTreeSize = 128;

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
    uint32_t s1, l1, e1;     // static cursor: state, match length, min_endpos(state) | wide << 31
    uint32_t n;              // tokens in the sequence so far
    uint32_t n_states;
    uint32_t last;
    uint32_t n_trans;
    uint32_t status;
    // dynamic cursor = link(last) and a copy of that state's record, so the
    // next step starts without reading it back: s2 (kNil before the first
    // token), then len (= l2), link, min_endpos (= e2), head, itok, idst
    uint32_t s2, p_len, p_link, p_endpos, p_head, p_itok, p_idst;
    uint32_t pad;
};

// (state, token) -> 32-bit hash; the same function on host and device
#if defined(__HIPCC__)
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
#if defined(__HIPCC__)
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

// slots per sequence: at most max_seq_len - 1 are ever used -> load <= 0.5
inline uint64_t dynamic_slots_for(int64_t max_seq_len)
{
    return (((uint64_t)max_seq_len * 2 + 64) + 15) / 16 * 16;
}

constexpr int64_t kCompactMaxSeqLen = 16366;     // 2T+2 state ids below 0x7FFF
constexpr int32_t kCompactMaxVocab  = 1 << 17;

struct DynRecCompact {   // 16 B
    uint16_t len, link, endpos, head;   // 0xFFFF = none (link of the root, empty head)
    uint32_t itok;                      // kNil = no inline transition
    uint16_t idst, pad;
};

struct SlotCompact {     // 8 B
    uint32_t key;        // state << 17 | token, kNil = empty
    uint16_t dst, next;  // next: 0xFFFF = end of the state's list
};

}  // namespace sam
