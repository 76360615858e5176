// gfx950 kernels for batched suffix-automaton matching, online extension and
// draft gather (arxiv 2411.10666: Algorithm 1 Transfer, Algorithm 2 Expand,
// Section 3.2 draft read and source selection, Section 3.3 update order).
//
// Execution shape: one workgroup per sequence.
//   wave 0  walks the static automaton (read-only tables in HBM),
//   wave 1  extends the sequence's own dynamic automaton,
// both over the same accepted tokens and concurrently; the one that comes second
// selects the source and gathers the draft with coalesced reads.  For large
// batches the step kernel has two more waves per sequence, the scouts, which run
// ahead over the step's tokens and pull the records and buckets the two walks
// will fall back to into the caches (see "scout waves" below).
// Inside a walking wave all control flow is wave-uniform: the lanes
// are used to fetch a whole 128-byte hash bucket in one request and to resolve
// it with two ballots, so a lookup costs one memory round trip whatever the
// state's out-degree.  The path is bound by dependent memory round trips, so
// the code is organised around them: every load whose address is known is
// issued before the wave waits for any of them, and the first lookup of the
// next token is issued together with the last read of the current one.
// Sequence b is always served by workgroup b, so its private tables keep
// hitting the L2 of the same XCD from launch to launch.
//
// The two token loops exist twice: in C++ (static_transfer, dyn_expand: every
// layout, every size) and, for the compact per-sequence tables and corpora below
// 2^32 buckets, in gfx950 assembly (static_feed_asm, dyn_feed_compact), which is
// what the benchmark configurations run (template parameter kAsm of the kernels,
// chosen at launch).  What a token costs is one wavefront's
// chain of dependent instructions and memory round trips; the assembly needs
// under half the instructions of the compiled code and waits only for the loads
// it is about to use.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sam_device.h"

namespace sam {

namespace {

__device__ __forceinline__ uint32_t uni(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}

__device__ __forceinline__ uint32_t lane_get(uint32_t v, int src_lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src_lane);
}

// Keep a wave-uniform value materialised at this point of the program, so the
// load that produced it cannot be moved below.
__device__ __forceinline__ void pin_s(uint32_t &v)
{
    asm volatile("" : "+s"(v));
}

// Same for a per-lane value.  Used on the step's token vector: once the load has
// landed before the token loop, reading a lane of it inside the loop no longer
// makes the wave wait for the stores of the previous token.
__device__ __forceinline__ void pin_v(uint32_t &v)
{
    asm volatile("" : "+v"(v));
}

__device__ __forceinline__ void order_memory()
{
    // stores and later loads of one wavefront reach memory in program order;
    // this only stops the compiler from moving them across each other
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

// ---- static automaton: Transfer (Algorithm 1) -----------------------------

// Feed one token.  (s, l) is the cursor, e = min_endpos(s) with the wide flag of s
// in bit 31 (a state is wide if it has transitions beyond the two in its record).
__device__ __forceinline__ void static_transfer(const StaticView &S, uint32_t t, int lane,
                                                uint32_t &s, uint32_t &l, uint32_t &e,
                                                uint32_t &fault)
{
    // every suffix-link hop shortens the match, so l + 1 rounds always suffice;
    // the bound only matters if the tables were corrupted
    for (uint32_t guard = l + 2; ; guard--) {
        if (guard == 0) { fault |= SAM_STATUS_INTERNAL_BIT; s = 0; l = 0; e = 0; return; }
        if (s == 0) {
            const uint2 r = reinterpret_cast<const uint2 *>(S.root)[t];
            uint32_t d = uni(r.x), ep = uni(r.y);
            pin_s(ep);
            if (d) { s = d; e = ep; l = 1; }
            else   { l = 0; e = 0; }
            return;
        }
        // the record answers for a state with at most two transitions; a wide state's
        // bucket is requested together with it
        const bool wide = (e & kWideBit) != 0;
        const LinkRec lr = S.linkrec[s];
        uint64_t b = 0;
        uint4 sl = make_uint4(kNil, kNil, 0, 0);
        if (wide) {
            b = bucket_of(hash_key(s, t), S.n_buckets);
            sl = reinterpret_cast<const uint4 *>(S.slots)[b * kBucketSlots + (lane & 7)];
        }
        if (uni(lr.itok) == t) {
            s = uni(lr.idst); e = uni(lr.iendpos); l += 1;
            return;
        }
        if (uni(lr.itok2) == t) {
            s = uni(lr.idst2); e = uni(lr.iendpos2); l += 1;
            return;
        }
        uint32_t nlink = uni(lr.link), nlen = uni(lr.lenlink);
        pin_s(nlink);
        bool hit = false;
        if (wide) {
            uint32_t mh = (uint32_t)__ballot(sl.x == s && sl.y == t) & 0xFFu;
            uint32_t me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
            pin_s(mh);
            for (uint64_t left = S.n_buckets; left; left--) {
                if (mh) {
                    const int j = __builtin_ctz(mh);
                    s = lane_get(sl.z, j);
                    e = lane_get(sl.w, j);
                    l += 1;
                    hit = true;
                    break;
                }
                if (me) break;
                b = (b + 1 == S.n_buckets) ? 0 : b + 1;
                sl = reinterpret_cast<const uint4 *>(S.slots)[b * kBucketSlots + (lane & 7)];
                mh = (uint32_t)__ballot(sl.x == s && sl.y == t) & 0xFFu;
                me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
            }
        }
        if (hit) return;
        s = nlink;
        l = nlen & ~kWideBit;
        e = nlen & kWideBit;
    }
}

// ---- dynamic automaton: the two table layouts ------------------------------

struct Rec {              // a state record held in wave-uniform registers
    uint32_t len, link, endpos, head, itok, idst;     // kNil = none
};

// 32-byte records, 16-byte slots, 8 slots per bucket: any length, any vocabulary
struct WideDyn {
    static constexpr int kSlots = 8;
    struct RawRec { uint4 a; uint2 b; };
    typedef uint4 RawSlot;

    static __device__ __forceinline__ RawRec issue_rec(const void *rec, uint32_t s)
    {
        const DynRec *r = reinterpret_cast<const DynRec *>(rec) + s;
        RawRec w;
        w.a = reinterpret_cast<const uint4 *>(r)[0];
        w.b = reinterpret_cast<const uint2 *>(r)[2];
        return w;
    }
    static __device__ __forceinline__ Rec finish_rec(const RawRec &w)
    {
        Rec R;
        R.len = uni(w.a.x); R.link = uni(w.a.y); R.endpos = uni(w.a.z); R.head = uni(w.a.w);
        R.itok = uni(w.b.x); R.idst = uni(w.b.y);
        return R;
    }
    static __device__ __forceinline__ void store_rec(void *rec, uint32_t s, const Rec &R)
    {
        DynRec *r = reinterpret_cast<DynRec *>(rec) + s;
        reinterpret_cast<uint4 *>(r)[0] = make_uint4(R.len, R.link, R.endpos, R.head);
        reinterpret_cast<uint2 *>(r)[2] = make_uint2(R.itok, R.idst);
    }
    static __device__ __forceinline__ void store_inline(void *rec, uint32_t s, uint32_t tok,
                                                        uint32_t dst)
    {
        reinterpret_cast<uint2 *>(reinterpret_cast<DynRec *>(rec) + s)[2] = make_uint2(tok, dst);
    }
    static __device__ __forceinline__ void store_head(void *rec, uint32_t s, uint32_t head)
    {
        (reinterpret_cast<DynRec *>(rec) + s)->head = head;
    }
    static __device__ __forceinline__ void store_link(void *rec, uint32_t s, uint32_t link)
    {
        (reinterpret_cast<DynRec *>(rec) + s)->link = link;
    }
    static __device__ __forceinline__ void store_idst(void *rec, uint32_t s, uint32_t dst)
    {
        (reinterpret_cast<DynRec *>(rec) + s)->idst = dst;
    }
    static __device__ __forceinline__ RawSlot issue_slot(const void *slots, uint32_t idx)
    {
        return reinterpret_cast<const uint4 *>(slots)[idx];
    }
    static __device__ __forceinline__ bool slot_is(const RawSlot &sl, uint32_t p, uint32_t t)
    {
        return sl.x == p && sl.y == t;
    }
    static __device__ __forceinline__ bool slot_empty(const RawSlot &sl) { return sl.x == kNil; }
    static __device__ __forceinline__ uint32_t slot_dst(const RawSlot &sl) { return sl.z; }
    static __device__ __forceinline__ uint32_t slot_token(const RawSlot &sl) { return sl.y; }
    static __device__ __forceinline__ uint32_t slot_next(const RawSlot &sl) { return sl.w; }
    static __device__ __forceinline__ void store_slot(void *slots, uint32_t idx, uint32_t p,
                                                      uint32_t t, uint32_t dst, uint32_t next)
    {
        reinterpret_cast<uint4 *>(slots)[idx] = make_uint4(p, t, dst, next);
    }
    static __device__ __forceinline__ void store_slot_dst(void *slots, uint32_t idx, uint32_t dst)
    {
        reinterpret_cast<Slot *>(slots)[idx].dst = dst;
    }
};

// 16-byte records, 8-byte slots, 16 slots per bucket: 15-bit state ids
struct CompactDyn {
    static constexpr int kSlots = 16;
    typedef uint4 RawRec;
    typedef uint2 RawSlot;

    static __device__ __forceinline__ uint32_t widen(uint32_t v16)
    {
        return v16 == 0xFFFFu ? kNil : v16;
    }
    static __device__ __forceinline__ RawRec issue_rec(const void *rec, uint32_t s)
    {
        return reinterpret_cast<const uint4 *>(rec)[s];
    }
    static __device__ __forceinline__ Rec finish_rec(const RawRec &w)
    {
        const uint32_t a = uni(w.x), b = uni(w.y);
        Rec R;
        R.len = a & 0xFFFFu; R.link = widen(a >> 16);
        R.endpos = b & 0xFFFFu; R.head = widen(b >> 16);
        R.itok = uni(w.z); R.idst = uni(w.w) & 0xFFFFu;
        return R;
    }
    static __device__ __forceinline__ void store_rec(void *rec, uint32_t s, const Rec &R)
    {
        reinterpret_cast<uint4 *>(rec)[s] =
            make_uint4((R.len & 0xFFFFu) | (R.link << 16), (R.endpos & 0xFFFFu) | (R.head << 16),
                       R.itok, R.idst & 0xFFFFu);
    }
    static __device__ __forceinline__ void store_inline(void *rec, uint32_t s, uint32_t tok,
                                                        uint32_t dst)
    {
        reinterpret_cast<uint2 *>(rec)[2 * s + 1] = make_uint2(tok, dst & 0xFFFFu);
    }
    static __device__ __forceinline__ void store_head(void *rec, uint32_t s, uint32_t head)
    {
        reinterpret_cast<uint16_t *>(rec)[8 * s + 3] = (uint16_t)head;
    }
    static __device__ __forceinline__ void store_link(void *rec, uint32_t s, uint32_t link)
    {
        reinterpret_cast<uint16_t *>(rec)[8 * s + 1] = (uint16_t)link;
    }
    static __device__ __forceinline__ void store_idst(void *rec, uint32_t s, uint32_t dst)
    {
        reinterpret_cast<uint16_t *>(rec)[8 * s + 6] = (uint16_t)dst;
    }
    static __device__ __forceinline__ RawSlot issue_slot(const void *slots, uint32_t idx)
    {
        return reinterpret_cast<const uint2 *>(slots)[idx];
    }
    static __device__ __forceinline__ bool slot_is(const RawSlot &sl, uint32_t p, uint32_t t)
    {
        return sl.x == ((p << 17) | t);
    }
    static __device__ __forceinline__ bool slot_empty(const RawSlot &sl) { return sl.x == kNil; }
    static __device__ __forceinline__ uint32_t slot_dst(const RawSlot &sl) { return sl.y & 0xFFFFu; }
    static __device__ __forceinline__ uint32_t slot_token(const RawSlot &sl) { return sl.x & 0x1FFFFu; }
    static __device__ __forceinline__ uint32_t slot_next(const RawSlot &sl) { return widen(sl.y >> 16); }
    static __device__ __forceinline__ void store_slot(void *slots, uint32_t idx, uint32_t p,
                                                      uint32_t t, uint32_t dst, uint32_t next)
    {
        reinterpret_cast<uint2 *>(slots)[idx] =
            make_uint2((p << 17) | t, (dst & 0xFFFFu) | (next << 16));
    }
    static __device__ __forceinline__ void store_slot_dst(void *slots, uint32_t idx, uint32_t dst)
    {
        reinterpret_cast<uint16_t *>(slots)[4 * idx + 2] = (uint16_t)dst;
    }
};

// ---- dynamic automaton: Expand (Algorithm 2) ------------------------------

struct DynSeq {
    int32_t *text;
    void    *rec;
    void    *slots;
    uint32_t n_buckets;
};

// A lookup of (p, t) in the slot table whose home bucket has been fetched and
// reduced to two lane masks: mh = slots holding the key, me = empty slots.
template <class L>
struct Probe {
    uint32_t b;
    typename L::RawSlot sl;
    uint32_t mh, me;
};

// Home bucket of (p, t) in a sequence's private table.  The tables are small
// and at most half full, so a short mix is enough; one multiply-high maps the
// hash onto the bucket count.
__device__ __forceinline__ uint32_t dyn_bucket(const DynSeq &D, uint32_t p, uint32_t t)
{
    uint32_t h = (p * 0x9E3779B1u) ^ (t * 0x85EBCA77u);
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    return __umulhi(h, D.n_buckets);
}

template <class L>
__device__ __forceinline__ typename L::RawSlot issue_bucket(const DynSeq &D, uint32_t b, int lane)
{
    return L::issue_slot(D.slots, b * L::kSlots + (lane & (L::kSlots - 1)));
}

template <class L>
__device__ __forceinline__ void reduce_bucket(Probe<L> &P, uint32_t p, uint32_t t)
{
    constexpr uint32_t kMask = (1u << L::kSlots) - 1u;
    P.mh = (uint32_t)__ballot(L::slot_is(P.sl, p, t)) & kMask;
    P.me = (uint32_t)__ballot(L::slot_empty(P.sl)) & kMask;
}

// Finish a lookup.  Hit: returns true, `at` = slot index, `dst` = target.
// Miss: returns false, `at` = first empty slot on the probe path (where an
// insert of this key goes; kNil if a full sweep found none, which the sizing
// of the table excludes).
template <class L>
__device__ __forceinline__ bool resolve_probe(const DynSeq &D, Probe<L> P, uint32_t p, uint32_t t,
                                              int lane, uint32_t &at, uint32_t &dst)
{
    for (uint32_t left = D.n_buckets; ; left--) {
        if (P.mh) {
            const int j = __builtin_ctz(P.mh);
            at = P.b * L::kSlots + j;
            dst = lane_get(L::slot_dst(P.sl), j);
            return true;
        }
        if (P.me) {
            at = P.b * L::kSlots + __builtin_ctz(P.me);
            return false;
        }
        if (left == 0) { at = kNil; return false; }
        P.b = (P.b + 1 == D.n_buckets) ? 0 : P.b + 1;
        P.sl = issue_bucket<L>(D, P.b, lane);
        reduce_bucket<L>(P, p, t);
    }
}

// Record of p and the home bucket of (p, t) in one round trip: both loads are
// issued, then both are consumed in the same straight-line block, so neither
// can be sunk behind a branch that depends on the other.
template <class L>
__device__ __forceinline__ void rec_and_probe(const DynSeq &D, uint32_t p, uint32_t t, int lane,
                                              Rec &R, Probe<L> &P)
{
    const typename L::RawRec raw = L::issue_rec(D.rec, p);
    P.b = dyn_bucket(D, p, t);
    P.sl = issue_bucket<L>(D, P.b, lane);
    reduce_bucket<L>(P, p, t);
    R = L::finish_rec(raw);
    pin_s(R.itok);
    pin_s(P.mh);
}

constexpr uint32_t kInline = 0xFFFFFFFEu;   // "the transition sits in the record"

template <class L>
struct DynCursor {
    uint32_t n, n_states, last, n_trans;
    uint32_t P;               // link(last); kNil while the sequence is empty
    Rec      RP;              // record of P, kept in step with memory
    uint32_t rec_bytes;       // size of the sequence's record table
    bool     pf_ok;           // pf is the reduced home bucket of (P, next token)
    Probe<L> pf;
};

// Append token t (Algorithm 2); tn is the token after it (kNil if unknown).
// Afterwards P = link(last) is the state of the longest suffix of the sequence
// that also ends earlier in it, with length RP.len: what the paper's
// Transfer-then-Expand order leaves in the dynamic cursor.
template <class L>
__device__ __forceinline__ void dyn_expand(const DynSeq &D, uint32_t t, uint32_t tn, int lane,
                                           DynCursor<L> &c, uint32_t &fault)
{
    // Suffix links strictly shorten, so every chain below ends at the root after
    // fewer than n_states moves; `guard` turns a corrupted table into a status
    // bit instead of an endless loop.
    uint32_t guard = c.n_states + 4;
    const uint32_t k = c.n + 1;
    const uint32_t cur = c.n_states++;
    const uint32_t last = c.last;
    const bool writer = lane == 0;

    // `last` has no transition yet and its record has not been written yet:
    // write it now, with its first transition (t -> cur) inline
    Rec LR;
    LR.len = c.n; LR.link = c.P; LR.endpos = c.n; LR.head = kNil; LR.itok = t; LR.idst = cur;
    if (writer) L::store_rec(D.rec, last, LR);
    c.n_trans++;
    order_memory();

    uint32_t newP;
    Rec newRP;
    bool new_pf_ok = false;
    Probe<L> new_pf = c.pf;

    if (c.P == kNil) {
        // first token of the sequence: last is the root, which now has (t -> cur)
        newP = 0;
        newRP.len = 0; newRP.link = kNil; newRP.endpos = 0; newRP.head = kNil;
        newRP.itok = t; newRP.idst = cur;
    } else {
        uint32_t p = c.P;
        Rec R = c.RP;
        Probe<L> pr = c.pf;
        bool have_pr = c.pf_ok;
        uint32_t q = kNil, where = kNil;
        // give t-transitions to the states on last's suffix path that lack one
        for (;;) {
            if (--guard == 0) { fault |= SAM_STATUS_INTERNAL_BIT; p = kNil; break; }
            if (R.itok == t) { q = R.idst; where = kInline; break; }
            if (!have_pr) {
                // P's bucket was not prefetched (P is a fresh clone, or this is the first
                // token of a launch); it is only needed now that the inline transition
                // is a different token
                pr.b = dyn_bucket(D, p, t);
                pr.sl = issue_bucket<L>(D, pr.b, lane);
                reduce_bucket<L>(pr, p, t);
            }
            uint32_t at, dst;
            if (resolve_probe<L>(D, pr, p, t, lane, at, dst)) { q = dst; where = at; break; }
            if (R.itok == kNil) {
                if (writer) L::store_inline(D.rec, p, t, cur);
                R.itok = t; R.idst = cur;
            } else if (at == kNil) {
                fault |= SAM_STATUS_INTERNAL_BIT;
            } else {
                if (writer) {
                    L::store_slot(D.slots, at, p, t, cur, R.head);
                    L::store_head(D.rec, p, at);
                }
                R.head = at;
            }
            c.n_trans++;
            order_memory();
            if (R.link == kNil) { p = kNil; break; }   // R stays the root's record
            p = R.link;
            rec_and_probe<L>(D, p, t, lane, R, pr);
            have_pr = true;
        }

        if (p == kNil) {
            newP = 0;
            newRP = R;
        } else {
            // q's record, and with it the next token's first lookup (at q)
            const typename L::RawRec rawq = L::issue_rec(D.rec, q);
            if (tn != kNil) {
                new_pf.b = dyn_bucket(D, q, tn);
                new_pf.sl = issue_bucket<L>(D, new_pf.b, lane);
                reduce_bucket<L>(new_pf, q, tn);
                pin_s(new_pf.mh);
            }
            Rec Q = L::finish_rec(rawq);
            pin_s(Q.len);
            if (q == last) Q = LR;
            if (R.len + 1 == Q.len) {
                newP = q;
                newRP = Q;
                new_pf_ok = tn != kNil;
            } else {
                const uint32_t cl = c.n_states++;
                Rec CL;
                CL.len = R.len + 1; CL.link = Q.link; CL.endpos = Q.endpos;
                CL.head = kNil; CL.itok = Q.itok; CL.idst = Q.idst;
                if (Q.itok != kNil) c.n_trans++;
                // copy q's further transitions
                for (uint32_t j = Q.head; j != kNil;) {
                    if (--guard == 0 || j >= D.n_buckets * L::kSlots) {
                        fault |= SAM_STATUS_INTERNAL_BIT;
                        break;
                    }
                    const typename L::RawSlot sl = L::issue_slot(D.slots, j);
                    const uint32_t tok = uni(L::slot_token(sl)), d = uni(L::slot_dst(sl));
                    j = uni(L::slot_next(sl));
                    Probe<L> pc;
                    pc.b = dyn_bucket(D, cl, tok);
                    pc.sl = issue_bucket<L>(D, pc.b, lane);
                    reduce_bucket<L>(pc, cl, tok);
                    uint32_t at, dummy;
                    resolve_probe<L>(D, pc, cl, tok, lane, at, dummy);
                    if (at == kNil) { fault |= SAM_STATUS_INTERNAL_BIT; break; }
                    if (writer) L::store_slot(D.slots, at, cl, tok, d, CL.head);
                    CL.head = at;
                    c.n_trans++;
                    order_memory();
                }
                if (writer) L::store_rec(D.rec, cl, CL);
                order_memory();
                // states further up the path that still lead to q now lead to the clone
                for (;;) {
                    if (writer) {
                        if (where == kInline) L::store_idst(D.rec, p, cl);
                        else L::store_slot_dst(D.slots, where, cl);
                    }
                    order_memory();
                    p = R.link;
                    if (p == kNil) break;
                    if (--guard == 0) { fault |= SAM_STATUS_INTERNAL_BIT; break; }
                    rec_and_probe<L>(D, p, t, lane, R, pr);
                    if (R.itok == t) {
                        if (R.idst != q) break;
                        where = kInline;
                    } else {
                        uint32_t at, dst;
                        if (!resolve_probe<L>(D, pr, p, t, lane, at, dst) || dst != q) break;
                        where = at;
                    }
                }
                if (writer) L::store_link(D.rec, q, cl);
                newP = cl;
                newRP = CL;
            }
        }
    }
    // the record of `cur` is written by the next call (or by flush_last)
    c.n = k; c.last = cur; c.P = newP; c.RP = newRP; c.pf_ok = new_pf_ok; c.pf = new_pf;
}

// Write the record of `last` (no transition yet) at the end of a launch.
template <class L>
__device__ __forceinline__ void flush_last(const DynSeq &D, const DynCursor<L> &c, int lane)
{
    Rec LR;
    LR.len = c.n; LR.link = c.P; LR.endpos = c.n; LR.head = kNil; LR.itok = kNil; LR.idst = 0;
    if (lane == 0) L::store_rec(D.rec, c.last, LR);
}

// ---- compact layout: Expand (Algorithm 2) in gfx950 assembly ----------------
//
// The same algorithm as dyn_expand above, for the compact tables, written out by
// hand: one wavefront's dependent instruction chain is what a token costs, and
// this form needs about half the instructions of the compiled one (records stay
// packed as stored, no copies between paths, stores under a one-lane exec mask
// without a branch).  The wide layout takes the C++ path; the kernels are
// instantiated with one form or the other, never both, because the mere presence
// of the C++ loop costs the assembly one 2 % (registers, code size).  Every table access goes through a buffer resource whose size is
// the table's, so an index outside a table reads zeros or is dropped instead of
// touching foreign memory, and every loop that follows table contents counts
// down a guard.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 table_rsrc(const void *base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)base;
    u32x4 r;
    r.x = uni((uint32_t)a);
    r.y = uni((uint32_t)(a >> 32)) & 0xFFFFu;   // stride 0: raw buffer
    r.z = bytes;
    r.w = 0x00020000u;                          // 32-bit data format
    return r;
}

// Append tokens tv[i .. m) to a sequence (P = -1: it is still empty).  i: index of the next token (in/out); on return i == m,
// or tv[i] is outside the vocabulary, or `flt` carries the internal-error bit.
// r0..r3 are the record of P as stored in the table.
//
// Register use inside (all named registers are scratch for this block):
//   s64 t        s65 next token (-1: none)   s66 t * c2
//   s68 q        s69..s71 scratch            s72 probe bucket (-1: no probe held)
//   s73 probe hit mask   s74 probe empty mask   s75 bucket of (q, next token)
//   s76..s79 record of q        s80 s81 words 0, 1 of last's record   s82 cur
//   s83 where the transition to q sits (slot index, -2: inline)   s84 slot index
//   s85 key      s86 loop guard   s87 last before this token   s88 clone
//   s89..s92 record of the clone  s93 list cursor  s94 token of a copied slot
//   s95 its target   s67 key of a requested, not yet reduced bucket (-1: none)   s98 scratch (slot bit, address)   s99 the next state up the path
//   v40 v41 addresses   v42:43 probe bucket   v44:45 next token's bucket
//   v46:49 record load  v50:53 store data  v54 store data of 16-bit fields   s96:97 exec on entry
// The probe of a bucket: lanes 0..15 load its 16 slots; hit mask = lanes whose
// key matches, empty mask = lanes whose key is the empty key.
#define SAM_HASH(dst, state, tokmul)                                                  \
        "s_mul_i32 s69, " state ", 0x9e3779b1\n\t"                                    \
        "s_xor_b32 s69, s69, " tokmul "\n\t"                                          \
        "s_lshr_b32 s70, s69, 15\n\t"                                                 \
        "s_xor_b32 s69, s69, s70\n\t"                                                 \
        "s_mul_i32 s69, s69, 0x2c1b3c6d\n\t"                                          \
        "s_mul_hi_u32 " dst ", s69, %[nb]\n\t"
#define SAM_LOAD_BUCKET(vdst, bucket)                                                 \
        "s_lshl_b32 s69, " bucket ", 7\n\t"                                           \
        "v_add_u32 v41, s69, %[lo]\n\t"                                               \
        "buffer_load_dwordx2 " vdst ", v41, %[rslt], 0 offen\n\t"
#define SAM_NEXT_BUCKET(bucket)                                                       \
        "s_add_u32 " bucket ", " bucket ", 1\n\t"                                     \
        "s_cmp_eq_u32 " bucket ", %[nb]\n\t"                                          \
        "s_cselect_b32 " bucket ", 0, " bucket "\n\t"
#define SAM_GUARD(label)                                                              \
        "s_sub_u32 s86, s86, 1\n\t"                                                   \
        "s_cbranch_scc1 " label "\n\t"
// last's record {n | P << 16, n | none << 16, t, cur} -> table (one lane)
#define SAM_STORE_LAST                                                                \
        "s_lshl_b32 s69, s87, 4\n\t"                                                 \
        "s_mov_b64 exec, 1\n\t"                                                      \
        "v_mov_b32 v40, s69\n\t"                                                     \
        "v_mov_b32 v50, s80\n\t"                                                     \
        "v_mov_b32 v51, s81\n\t"                                                     \
        "v_mov_b32 v52, s64\n\t"                                                     \
        "v_mov_b32 v53, s82\n\t"                                                     \
        "buffer_store_dwordx4 v[50:53], v40, %[rrec], 0 offen\n\t"                   \
        "s_mov_b64 exec, 0xffff\n\t"

__device__ __forceinline__ void dyn_feed_compact(u32x4 rrec, u32x4 rslt, uint32_t nb, uint32_t m,
                                                 uint32_t vocab, uint32_t tv, uint32_t lo,
                                                 uint32_t &i, uint32_t &n, uint32_t &ns,
                                                 uint32_t &last, uint32_t &nt, uint32_t &P,
                                                 uint32_t &r0, uint32_t &r1, uint32_t &r2,
                                                 uint32_t &r3, uint32_t &flt)
{
    asm volatile(
        "s_mov_b64 s[96:97], exec\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_mov_b32 s67, -1\n\t"
        "s_mov_b32 s72, -1\n"
        // ---- one token ---------------------------------------------------------
        "L_token_%=:\n\t"
        "v_readlane_b32 s64, %[tv], %[i]\n\t"
        "s_add_u32 s69, %[i], 1\n\t"
        "s_mov_b32 s65, -1\n\t"
        "s_cmp_ge_u32 s64, %[vocab]\n\t"
        "s_cbranch_scc1 L_exit_%=\n\t"
        "s_mul_i32 s66, s64, 0x85ebca77\n\t"
        "s_cmp_lt_u32 s69, %[m]\n\t"
        "s_cbranch_scc0 L_notn_%=\n\t"
        "v_readlane_b32 s65, %[tv], s69\n\t"
        "s_cmp_lt_u32 s65, %[vocab]\n\t"
        "s_cselect_b32 s65, s65, -1\n"
        "L_notn_%=:\n\t"
        // new state cur; last's record {n | P << 16, n | none << 16, t, cur}
        "s_mov_b32 s82, %[ns]\n\t"
        "s_lshl_b32 s80, %[P], 16\n\t"
        "s_or_b32 s80, s80, %[n]\n\t"
        "s_or_b32 s81, %[n], 0xffff0000\n\t"
        // (stored once the loads this token waits for are in flight, so that the
        // wave never waits for the store itself)
        "s_add_u32 %[ns], %[ns], 1\n\t"
        "s_add_u32 %[nt], %[nt], 1\n\t"
        "s_add_u32 %[n], %[n], 1\n\t"
        "s_mov_b32 s87, %[last]\n\t"
        "s_mov_b32 %[last], s82\n\t"
        // guard: suffix-link and list chains take fewer than n_states moves in all, sweeps
        // past full buckets fewer than n_buckets
        "s_add_u32 s86, %[ns], 4\n\t"
        "s_add_u32 s86, s86, %[nb]\n\t"
        "s_cmp_eq_u32 %[P], -1\n\t"
        "s_cbranch_scc0 L_walk_%=\n\t"
        // the sequence's very first token: last is the root, which now has (t -> cur)
        // as its inline transition; the cursor is the root
        "s_mov_b32 %[P], 0\n\t"
        "s_mov_b32 %[r0], 0xffff0000\n\t"
        "s_mov_b32 %[r1], 0xffff0000\n\t"
        "s_mov_b32 %[r2], s64\n\t"
        "s_mov_b32 %[r3], s82\n\t"
        "s_branch L_atroot_%=\n"
        // ---- walk last's suffix path: states without a t-transition get one ----
        "L_walk_%=:\n\t"
        SAM_GUARD("L_corrupt_%=")
        "s_cmp_eq_u32 %[r2], s64\n\t"
        "s_cbranch_scc1 L_inline_%=\n\t"
        "s_cmp_eq_u32 s72, -1\n\t"
        "s_cbranch_scc1 L_probe_%=\n\t"
        "s_cmp_eq_u32 s67, -1\n\t"
        "s_cbranch_scc1 L_resolve_%=\n\t"
        // the bucket was requested at the end of the last token and not looked at yet
        "s_waitcnt vmcnt(0)\n\t"
        "v_mov_b32 v42, v44\n\t"
        "v_mov_b32 v43, v45\n\t"
        "v_cmp_eq_u32 vcc, s67, v44\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v44\n\t"
        "s_mov_b32 s67, -1\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n\t"
        "s_branch L_resolve_%=\n"
        "L_probe_%=:\n\t"
        // no probe held for (P, t): fetch and reduce its home bucket
        SAM_HASH("s72", "%[P]", "s66")
        SAM_LOAD_BUCKET("v[42:43]", "s72")
        "s_lshl_b32 s85, %[P], 17\n\t"
        "s_or_b32 s85, s85, s64\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "v_cmp_eq_u32 vcc, s85, v42\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v42\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n"
        "L_resolve_%=:\n\t"
        "s_cmp_lg_u32 s73, 0\n\t"
        "s_cbranch_scc1 L_hit_%=\n\t"
        "s_cmp_lg_u32 s74, 0\n\t"
        "s_cbranch_scc1 L_miss_%=\n\t"
        // bucket full of other keys: go on in the next one
        SAM_GUARD("L_corrupt_%=")
        SAM_NEXT_BUCKET("s72")
        SAM_LOAD_BUCKET("v[42:43]", "s72")
        "s_lshl_b32 s85, %[P], 17\n\t"
        "s_or_b32 s85, s85, s64\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "v_cmp_eq_u32 vcc, s85, v42\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v42\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n\t"
        "s_branch L_resolve_%=\n"
        "L_hit_%=:\n\t"
        "s_ff1_i32_b32 s69, s73\n\t"
        "v_readlane_b32 s68, v43, s69\n\t"
        "s_lshl_b32 s83, s72, 4\n\t"
        "s_add_u32 s83, s83, s69\n\t"
        "s_and_b32 s68, s68, 0xffff\n\t"
        "s_branch L_found_%=\n"
        "L_inline_%=:\n\t"
        "s_mov_b32 s68, %[r3]\n\t"
        "s_mov_b32 s83, -2\n\t"
        "s_mov_b32 s67, -1\n\t"               // a bucket still on the way is not needed
        "s_branch L_found_%=\n"
        "L_miss_%=:\n\t"
        // (P, t) is missing.  The next state up the path is known from P's record, so
        // its record and its bucket for t are requested first; the stores that give P
        // its transition follow and are not waited for.
        "s_add_u32 %[nt], %[nt], 1\n\t"
        "s_lshr_b32 s99, %[r0], 16\n\t"
        "s_cmp_eq_u32 s99, 0xffff\n\t"
        "s_cbranch_scc1 L_ins_%=\n\t"
        "s_lshl_b32 s70, s99, 4\n\t"
        "v_mov_b32 v40, s70\n\t"
        "buffer_load_dwordx4 v[46:49], v40, %[rrec], 0 offen\n\t"
        SAM_HASH("s75", "s99", "s66")
        SAM_LOAD_BUCKET("v[44:45]", "s75")
        "L_ins_%=:\n\t"
        // (P, t) -> cur: inline if P has no transition yet, else into the empty slot
        "s_cmp_eq_u32 %[r2], -1\n\t"
        "s_cbranch_scc1 L_ins_inline_%=\n\t"
        "s_ff1_i32_b32 s98, s74\n\t"
        "s_lshl_b32 s84, s72, 4\n\t"
        "s_add_u32 s84, s84, s98\n\t"
        "s_lshl_b32 s85, %[P], 17\n\t"
        "s_or_b32 s85, s85, s64\n\t"
        "s_and_b32 s70, %[r1], 0xffff0000\n\t"
        "s_or_b32 s70, s70, s82\n\t"
        "s_lshl_b32 s69, s84, 3\n\t"
        "s_lshl_b32 s71, %[P], 4\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v40, s69\n\t"
        "v_mov_b32 v50, s85\n\t"
        "v_mov_b32 v51, s70\n\t"
        "buffer_store_dwordx2 v[50:51], v40, %[rslt], 0 offen\n\t"
        "v_mov_b32 v41, s71\n\t"
        "v_mov_b32 v52, s84\n\t"
        "buffer_store_short v52, v41, %[rrec], 0 offen offset:6\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_and_b32 %[r1], %[r1], 0xffff\n\t"
        "s_lshl_b32 s69, s84, 16\n\t"
        "s_or_b32 %[r1], %[r1], s69\n\t"
        "s_cmp_eq_u32 s99, 0xffff\n\t"
        "s_cbranch_scc1 L_atroot_%=\n\t"        // P is the root: it stays the cursor
        // the slot just taken still reads as empty in a bucket fetched before the
        // store: if the next state's bucket is the same one, take it out of the mask
        "s_lshl_b32 s98, 1, s98\n\t"
        "s_cmp_eq_u32 s72, s75\n\t"
        "s_cselect_b32 s98, s98, 0\n\t"
        "s_waitcnt vmcnt(2)\n\t"
        "s_branch L_advance_%=\n"
        "L_ins_inline_%=:\n\t"
        "s_lshl_b32 s71, %[P], 4\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v41, s71\n\t"
        "v_mov_b32 v50, s64\n\t"
        "v_mov_b32 v51, s82\n\t"
        "buffer_store_dwordx2 v[50:51], v41, %[rrec], 0 offen offset:8\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_mov_b32 %[r2], s64\n\t"
        "s_mov_b32 %[r3], s82\n\t"
        "s_cmp_eq_u32 s99, 0xffff\n\t"
        "s_cbranch_scc1 L_atroot_%=\n\t"
        "s_mov_b32 s98, 0\n\t"
        "s_waitcnt vmcnt(1)\n"
        "L_advance_%=:\n\t"
        // one state up: its record and the reduced bucket become the current ones
        "s_mov_b32 %[P], s99\n\t"
        "s_lshl_b32 s85, s99, 17\n\t"
        "s_or_b32 s85, s85, s64\n\t"
        "v_cmp_eq_u32 vcc, s85, v44\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v44\n\t"
        "v_readfirstlane_b32 %[r0], v46\n\t"
        "v_readfirstlane_b32 %[r1], v47\n\t"
        "v_readfirstlane_b32 %[r2], v48\n\t"
        "v_readfirstlane_b32 %[r3], v49\n\t"
        "v_mov_b32 v42, v44\n\t"
        "v_mov_b32 v43, v45\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_andn2_b32 s74, s70, s98\n\t"
        "s_mov_b32 s72, s75\n\t"
        "s_branch L_walk_%=\n"
        // ---- q = next(P)[t] exists -----------------------------------------------
        "L_found_%=:\n\t"
        "s_lshl_b32 s69, s68, 4\n\t"
        "v_mov_b32 v40, s69\n\t"
        "buffer_load_dwordx4 v[46:49], v40, %[rrec], 0 offen\n\t"
        "s_cmp_eq_u32 s65, -1\n\t"
        "s_cbranch_scc1 L_noprefetch_%=\n\t"
        // with it, the next token's first lookup (at q)
        "s_mul_i32 s71, s65, 0x85ebca77\n\t"
        SAM_HASH("s75", "s68", "s71")
        SAM_LOAD_BUCKET("v[44:45]", "s75")
        SAM_STORE_LAST
        "s_waitcnt vmcnt(2)\n\t"
        "s_branch L_qrec_%=\n"
        "L_noprefetch_%=:\n\t"
        SAM_STORE_LAST
        "s_waitcnt vmcnt(1)\n"
        "L_qrec_%=:\n\t"
        "v_readfirstlane_b32 s76, v46\n\t"
        "v_readfirstlane_b32 s77, v47\n\t"
        "v_readfirstlane_b32 s78, v48\n\t"
        "v_readfirstlane_b32 s79, v49\n\t"
        "s_cmp_lg_u32 s68, s87\n\t"
        "s_cbranch_scc1 L_qok_%=\n\t"
        "s_mov_b32 s76, s80\n\t"                // q is the old last: its record as just written
        "s_mov_b32 s77, s81\n\t"
        "s_mov_b32 s78, s64\n\t"
        "s_mov_b32 s79, s82\n"
        "L_qok_%=:\n\t"
        "s_and_b32 s69, %[r0], 0xffff\n\t"
        "s_add_u32 s69, s69, 1\n\t"             // len(P) + 1
        "s_and_b32 s70, s76, 0xffff\n\t"
        "s_cmp_eq_u32 s69, s70\n\t"
        "s_cbranch_scc0 L_clone_%=\n\t"
        "s_mov_b32 %[P], s68\n\t"
        "s_mov_b32 %[r0], s76\n\t"
        "s_mov_b32 %[r1], s77\n\t"
        "s_mov_b32 %[r2], s78\n\t"
        "s_mov_b32 %[r3], s79\n\t"
        "s_mov_b32 s72, -1\n\t"
        "s_cmp_eq_u32 s65, -1\n\t"
        "s_cbranch_scc1 L_next_%=\n\t"
        "s_lshl_b32 s85, s68, 17\n\t"
        "s_or_b32 s85, s85, s65\n\t"
        "s_mov_b32 s72, s75\n\t"
        "s_waitcnt vmcnt(1)\n\t"
        "v_mov_b32 v42, v44\n\t"
        "v_mov_b32 v43, v45\n\t"
        "v_cmp_eq_u32 vcc, s85, v44\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v44\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n\t"
        "s_branch L_next_%=\n"
        // ---- clone q at length len(P) + 1 ------------------------------------------
        "L_clone_%=:\n\t"
        "s_mov_b32 s88, %[ns]\n\t"
        "s_add_u32 %[ns], %[ns], 1\n\t"
        "s_and_b32 s89, s76, 0xffff0000\n\t"
        "s_or_b32 s89, s89, s69\n\t"            // len = len(P) + 1, link = link(q)
        "s_or_b32 s90, s77, 0xffff0000\n\t"     // endpos(q), empty list
        "s_mov_b32 s91, s78\n\t"
        "s_mov_b32 s92, s79\n\t"
        "s_lshr_b32 s93, s77, 16\n\t"           // head of q's list
        "s_waitcnt vmcnt(0)\n\t"
        "s_cmp_eq_u32 s78, -1\n\t"
        "s_cbranch_scc1 L_copy_%=\n\t"
        "s_add_u32 %[nt], %[nt], 1\n"
        "L_copy_%=:\n\t"
        "s_cmp_eq_u32 s93, 0xffff\n\t"
        "s_cbranch_scc1 L_copied_%=\n\t"
        SAM_GUARD("L_corrupt_%=")
        "s_lshl_b32 s69, s93, 3\n\t"
        "v_mov_b32 v40, s69\n\t"
        "buffer_load_dwordx2 v[46:47], v40, %[rslt], 0 offen\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "v_readfirstlane_b32 s94, v46\n\t"
        "v_readfirstlane_b32 s95, v47\n\t"
        "s_and_b32 s94, s94, 0x1ffff\n\t"
        "s_lshr_b32 s93, s95, 16\n\t"
        "s_and_b32 s95, s95, 0xffff\n\t"
        "s_mul_i32 s71, s94, 0x85ebca77\n\t"
        SAM_HASH("s84", "s88", "s71")
        "L_copy_probe_%=:\n\t"
        SAM_LOAD_BUCKET("v[42:43]", "s84")
        "s_waitcnt vmcnt(0)\n\t"
        "v_cmp_eq_u32 vcc, -1, v42\n\t"
        "s_nop 1\n\t"
        "s_cmp_lg_u32 vcc_lo, 0\n\t"
        "s_cbranch_scc1 L_copy_put_%=\n\t"
        SAM_GUARD("L_corrupt_%=")
        SAM_NEXT_BUCKET("s84")
        "s_branch L_copy_probe_%=\n"
        "L_copy_put_%=:\n\t"
        "s_ff1_i32_b32 s69, vcc_lo\n\t"
        "s_lshl_b32 s84, s84, 4\n\t"
        "s_add_u32 s84, s84, s69\n\t"           // slot index
        "s_lshl_b32 s85, s88, 17\n\t"
        "s_or_b32 s85, s85, s94\n\t"
        "s_and_b32 s70, s90, 0xffff0000\n\t"
        "s_or_b32 s70, s70, s95\n\t"
        "s_lshl_b32 s69, s84, 3\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v40, s69\n\t"
        "v_mov_b32 v50, s85\n\t"
        "v_mov_b32 v51, s70\n\t"
        "buffer_store_dwordx2 v[50:51], v40, %[rslt], 0 offen\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_and_b32 s90, s90, 0xffff\n\t"
        "s_lshl_b32 s69, s84, 16\n\t"
        "s_or_b32 s90, s90, s69\n\t"
        "s_add_u32 %[nt], %[nt], 1\n\t"
        "s_branch L_copy_%=\n"
        "L_copied_%=:\n\t"
        "s_lshl_b32 s69, s88, 4\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v40, s69\n\t"
        "v_mov_b32 v50, s89\n\t"
        "v_mov_b32 v51, s90\n\t"
        "v_mov_b32 v52, s91\n\t"
        "v_mov_b32 v53, s92\n\t"
        "buffer_store_dwordx4 v[50:53], v40, %[rrec], 0 offen\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        // the next token starts at the clone: request its bucket there now that the
        // clone's transitions are all stored (a request before them could miss one)
        "s_cmp_eq_u32 s65, -1\n\t"
        "s_cbranch_scc1 L_redirect_%=\n\t"
        "s_mul_i32 s71, s65, 0x85ebca77\n\t"
        SAM_HASH("s75", "s88", "s71")
        SAM_LOAD_BUCKET("v[44:45]", "s75")
        // states further up the path that still lead to q now lead to the clone
        "L_redirect_%=:\n\t"
        "s_lshr_b32 s99, %[r0], 16\n\t"
        "s_lshl_b32 s98, %[P], 4\n\t"           // where the store below goes, if inline
        "s_cmp_eq_u32 s99, 0xffff\n\t"
        "s_cbranch_scc1 L_red_store_%=\n\t"
        SAM_GUARD("L_corrupt_%=")
        // the next state's record and bucket first, then the store (not waited for)
        "s_mov_b32 %[P], s99\n\t"
        "s_lshl_b32 s70, %[P], 4\n\t"
        "v_mov_b32 v40, s70\n\t"
        "buffer_load_dwordx4 v[46:49], v40, %[rrec], 0 offen\n\t"
        SAM_HASH("s72", "%[P]", "s66")
        SAM_LOAD_BUCKET("v[42:43]", "s72")
        "s_lshl_b32 s85, %[P], 17\n\t"
        "s_or_b32 s85, s85, s64\n"
        "L_red_store_%=:\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v54, s88\n\t"
        "s_cmp_eq_u32 s83, -2\n\t"
        "s_cbranch_scc0 L_red_slot_%=\n\t"
        "v_mov_b32 v40, s98\n\t"
        "buffer_store_short v54, v40, %[rrec], 0 offen offset:12\n\t"
        "s_branch L_red_up_%=\n"
        "L_red_slot_%=:\n\t"
        "s_lshl_b32 s69, s83, 3\n\t"
        "v_mov_b32 v40, s69\n\t"
        "buffer_store_short v54, v40, %[rslt], 0 offen offset:4\n"
        "L_red_up_%=:\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_cmp_eq_u32 s99, 0xffff\n\t"
        "s_cbranch_scc1 L_redirected_%=\n\t"
        "s_waitcnt vmcnt(1)\n\t"
        "v_cmp_eq_u32 vcc, s85, v42\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v42\n\t"
        "v_readfirstlane_b32 %[r0], v46\n\t"
        "v_readfirstlane_b32 %[r1], v47\n\t"
        "v_readfirstlane_b32 %[r2], v48\n\t"
        "v_readfirstlane_b32 %[r3], v49\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n\t"
        "s_cmp_eq_u32 %[r2], s64\n\t"
        "s_cbranch_scc0 L_red_resolve_%=\n\t"
        "s_cmp_eq_u32 %[r3], s68\n\t"
        "s_cbranch_scc0 L_redirected_%=\n\t"
        "s_mov_b32 s83, -2\n\t"
        "s_branch L_redirect_%=\n"
        "L_red_resolve_%=:\n\t"
        "s_cmp_lg_u32 s73, 0\n\t"
        "s_cbranch_scc1 L_red_hit_%=\n\t"
        "s_cmp_lg_u32 s74, 0\n\t"
        "s_cbranch_scc1 L_redirected_%=\n\t"
        SAM_GUARD("L_corrupt_%=")
        SAM_NEXT_BUCKET("s72")
        SAM_LOAD_BUCKET("v[42:43]", "s72")
        "s_waitcnt vmcnt(0)\n\t"
        "v_cmp_eq_u32 vcc, s85, v42\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v42\n\t"
        "s_mov_b32 s73, vcc_lo\n\t"
        "s_mov_b32 s74, s70\n\t"
        "s_branch L_red_resolve_%=\n"
        "L_red_hit_%=:\n\t"
        "s_ff1_i32_b32 s69, s73\n\t"
        "v_readlane_b32 s70, v43, s69\n\t"
        "s_lshl_b32 s83, s72, 4\n\t"
        "s_add_u32 s83, s83, s69\n\t"
        "s_and_b32 s70, s70, 0xffff\n\t"
        "s_cmp_eq_u32 s70, s68\n\t"
        "s_cbranch_scc1 L_redirect_%=\n"
        "L_redirected_%=:\n\t"
        "s_lshl_b32 s69, s68, 4\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 v40, s69\n\t"
        "v_mov_b32 v54, s88\n\t"
        "buffer_store_short v54, v40, %[rrec], 0 offen offset:2\n\t"
        "s_mov_b64 exec, 0xffff\n\t"
        "s_mov_b32 %[P], s88\n\t"
        "s_mov_b32 %[r0], s89\n\t"
        "s_mov_b32 %[r1], s90\n\t"
        "s_mov_b32 %[r2], s91\n\t"
        "s_mov_b32 %[r3], s92\n\t"
        "s_mov_b32 s72, -1\n\t"
        "s_cmp_eq_u32 s65, -1\n\t"
        "s_cbranch_scc1 L_next_%=\n\t"
        // its bucket is on the way; it is waited for and reduced only if the next
        // token does not take the clone's inline transition
        "s_lshl_b32 s67, s88, 17\n\t"
        "s_or_b32 s67, s67, s65\n\t"
        "s_mov_b32 s72, s75\n\t"
        "s_branch L_next_%=\n"
        "L_atroot_%=:\n\t"
        "s_mov_b32 s72, -1\n\t"
        SAM_STORE_LAST
        // ---- next token -------------------------------------------------------------
        "L_next_%=:\n\t"
        "s_add_u32 %[i], %[i], 1\n\t"
        "s_cmp_lt_u32 %[i], %[m]\n\t"
        "s_cbranch_scc1 L_token_%=\n\t"
        "s_branch L_exit_%=\n"
        "L_corrupt_%=:\n\t"
        "s_or_b32 %[flt], %[flt], 8\n"
        "L_exit_%=:\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "s_mov_b64 exec, s[96:97]\n\t"
        : [i] "+s"(i), [n] "+s"(n), [ns] "+s"(ns), [last] "+s"(last), [nt] "+s"(nt), [P] "+s"(P),
          [r0] "+s"(r0), [r1] "+s"(r1), [r2] "+s"(r2), [r3] "+s"(r3), [flt] "+s"(flt)
        : [rrec] "s"(rrec), [rslt] "s"(rslt), [nb] "s"(nb), [m] "s"(m), [vocab] "s"(vocab),
          [tv] "v"(tv), [lo] "v"(lo)
        : "memory", "vcc", "scc",
          "s64", "s65", "s66", "s67", "s68", "s69", "s70", "s71", "s72", "s73", "s74", "s75",
          "s76", "s77", "s78", "s79", "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87",
          "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95", "s96", "s97", "s98", "s99",
          "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", "v50", "v51",
          "v52", "v53", "v54");
}
#undef SAM_HASH
#undef SAM_STORE_LAST
#undef SAM_LOAD_BUCKET
#undef SAM_NEXT_BUCKET
#undef SAM_GUARD

// ---- per-wave work shared by the step, ingest and replay kernels -------------

// Transfer (Algorithm 1) over tokens tv[i .. m) in gfx950 assembly: the same
// steps as static_transfer, about a third of the instructions.  Lanes 0..7 fetch
// the 8 slots of a bucket, the suffix-link record travels with the bucket.  i:
// index of the next token (in/out); on return i == m or tv[i] is outside the
// vocabulary.  Needs n_buckets < 2^32.
//   s64 t   s65 t * c2   s66 link-hop guard   s67 bucket-sweep guard
//   s68:69 s70:71 addresses / compare results   s72 hash   s73 bucket
//   s74 hit mask   s75 empty mask   s76:77 compare result   s78 s79 scratch
//   v41 zero   v42:45 slot {state, token, dst, endpos}   s88..s95 state record   v46:47 root entry
__device__ __forceinline__ void static_feed_asm(uint32_t slots_lo, uint32_t slots_hi,
                                                uint32_t lr_lo, uint32_t lr_hi, uint32_t root_lo,
                                                uint32_t root_hi, uint32_t nb, uint32_t m,
                                                uint32_t vocab, uint32_t tv, uint32_t lane16,
                                                uint32_t &i, uint32_t &st, uint32_t &l,
                                                uint32_t &e, uint32_t &flt)
{
    asm volatile(
        "s_mov_b64 s[96:97], exec\n\t"
        "s_mov_b64 exec, 0xff\n\t"
        "v_mov_b32 v41, 0\n"
        "L_stok_%=:\n\t"
        "v_readlane_b32 s64, %[tv], %[i]\n\t"
        "s_add_u32 s66, %[l], 2\n\t"            // every link hop shortens the match
        "s_cmp_ge_u32 s64, %[vocab]\n\t"
        "s_cbranch_scc1 L_sexit_%=\n\t"
        "s_mul_i32 s65, s64, 0x85ebca77\n"
        "L_stry_%=:\n\t"
        "s_sub_u32 s66, s66, 1\n\t"
        "s_cbranch_scc1 L_scorrupt_%=\n\t"
        "s_cmp_eq_u32 %[st], 0\n\t"
        "s_cbranch_scc1 L_sroot_%=\n\t"
        // the state's record {itok, idst, iendpos, itok2, idst2, iendpos2, link, lenlink}.
        // It comes through the scalar cache (the table is read-only), which has its own
        // counter: vector loads return in order, so a record behind a bucket in the same
        // queue could not arrive before it.  Bit 31 of e says whether the state is wide;
        // if not, its record holds all its transitions and no bucket is requested.
        "s_lshl_b32 s68, %[st], 5\n\t"
        "s_lshr_b32 s69, %[st], 27\n\t"
        "s_add_u32 s68, s68, %[lr_lo]\n\t"
        "s_addc_u32 s69, s69, %[lr_hi]\n\t"
        "s_load_dwordx8 s[88:95], s[68:69], 0x0\n\t"
        "s_bitcmp1_b32 %[e], 31\n\t"
        "s_cbranch_scc0 L_srec_%=\n\t"
        "s_mul_i32 s72, %[st], 0x9e3779b1\n\t"
        "s_add_u32 s72, s72, s65\n\t"
        "s_lshr_b32 s79, s72, 15\n\t"
        "s_xor_b32 s72, s72, s79\n\t"
        "s_mul_i32 s72, s72, 0x2c1b3c6d\n\t"
        "s_lshr_b32 s79, s72, 12\n\t"
        "s_xor_b32 s72, s72, s79\n\t"
        "s_mul_i32 s72, s72, 0x297a2d39\n\t"
        "s_lshr_b32 s79, s72, 15\n\t"
        "s_xor_b32 s72, s72, s79\n\t"
        "s_mul_hi_u32 s73, s72, %[nb]\n\t"
        "s_mov_b32 s67, %[nb]\n\t"
        "s_lshl_b32 s70, s73, 7\n\t"
        "s_lshr_b32 s71, s73, 25\n\t"
        "s_add_u32 s70, s70, %[slots_lo]\n\t"
        "s_addc_u32 s71, s71, %[slots_hi]\n\t"
        "global_load_dwordx4 v[42:45], %[lane16], s[70:71]\n\t"
        // the record is here before the bucket (often from a line the last token
        // already brought in): if it repeats the transition asked for, the bucket is
        // not waited for at all
        "s_waitcnt lgkmcnt(0)\n\t"
        "s_cmp_eq_u32 s88, s64\n\t"
        "s_cbranch_scc1 L_sinline_%=\n\t"
        "s_cmp_eq_u32 s91, s64\n\t"
        "s_cbranch_scc1 L_sinline2_%=\n\t"
        "s_branch L_swait_%=\n"
        "L_srec_%=:\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "s_cmp_eq_u32 s88, s64\n\t"
        "s_cbranch_scc1 L_sinline_%=\n\t"
        "s_cmp_eq_u32 s91, s64\n\t"
        "s_cbranch_scc1 L_sinline2_%=\n\t"
        "s_branch L_smiss_%=\n"
        "L_sload_%=:\n\t"
        "s_lshl_b32 s70, s73, 7\n\t"
        "s_lshr_b32 s71, s73, 25\n\t"
        "s_add_u32 s70, s70, %[slots_lo]\n\t"
        "s_addc_u32 s71, s71, %[slots_hi]\n\t"
        "global_load_dwordx4 v[42:45], %[lane16], s[70:71]\n"
        "L_swait_%=:\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "v_cmp_eq_u32 vcc, %[st], v42\n\t"
        "v_cmp_eq_u32 s[76:77], s64, v43\n\t"
        "v_cmp_eq_u32 s[70:71], -1, v42\n\t"
        "s_and_b32 s74, vcc_lo, s76\n\t"
        "s_mov_b32 s75, s70\n\t"
        "s_cmp_lg_u32 s74, 0\n\t"
        "s_cbranch_scc1 L_shit_%=\n\t"
        "s_cmp_lg_u32 s75, 0\n\t"
        "s_cbranch_scc1 L_smiss_%=\n\t"
        // bucket full of other keys: go on in the next one
        "s_sub_u32 s67, s67, 1\n\t"
        "s_cbranch_scc1 L_scorrupt_%=\n\t"
        "s_add_u32 s73, s73, 1\n\t"
        "s_cmp_eq_u32 s73, %[nb]\n\t"
        "s_cselect_b32 s73, 0, s73\n\t"
        "s_branch L_sload_%=\n"
        "L_shit_%=:\n\t"
        "s_ff1_i32_b32 s78, s74\n\t"
        "s_add_u32 %[l], %[l], 1\n\t"
        "v_readlane_b32 %[st], v44, s78\n\t"
        "v_readlane_b32 %[e], v45, s78\n\t"
        "s_branch L_sdone_%=\n"
        "L_sinline_%=:\n\t"
        "s_add_u32 %[l], %[l], 1\n\t"
        "s_mov_b32 %[st], s89\n\t"
        "s_mov_b32 %[e], s90\n\t"
        "s_branch L_sdone_%=\n"
        "L_sinline2_%=:\n\t"
        "s_add_u32 %[l], %[l], 1\n\t"
        "s_mov_b32 %[st], s92\n\t"
        "s_mov_b32 %[e], s93\n\t"
        "s_branch L_sdone_%=\n"
        "L_smiss_%=:\n\t"
        "s_mov_b32 %[st], s94\n\t"              // follow the suffix link
        "s_and_b32 %[l], s95, 0x7fffffff\n\t"
        "s_and_b32 %[e], s95, 0x80000000\n\t"   // its wide flag; its end position is not needed
        "s_branch L_stry_%=\n"
        "L_sroot_%=:\n\t"
        "s_lshl_b32 s68, s64, 3\n\t"
        "s_add_u32 s68, s68, %[root_lo]\n\t"
        "s_addc_u32 s69, %[root_hi], 0\n\t"
        "global_load_dwordx2 v[46:47], v41, s[68:69]\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "v_readfirstlane_b32 s78, v46\n\t"
        "v_readfirstlane_b32 s79, v47\n\t"
        "s_cmp_eq_u32 s78, 0\n\t"
        "s_cbranch_scc1 L_snone_%=\n\t"
        "s_mov_b32 %[st], s78\n\t"
        "s_mov_b32 %[e], s79\n\t"
        "s_mov_b32 %[l], 1\n\t"
        "s_branch L_sdone_%=\n"
        "L_snone_%=:\n\t"
        "s_mov_b32 %[l], 0\n\t"
        "s_mov_b32 %[e], 0\n"
        "L_sdone_%=:\n\t"
        "s_add_u32 %[i], %[i], 1\n\t"
        "s_cmp_lt_u32 %[i], %[m]\n\t"
        "s_cbranch_scc1 L_stok_%=\n\t"
        "s_branch L_sexit_%=\n"
        "L_scorrupt_%=:\n\t"
        "s_or_b32 %[flt], %[flt], 8\n\t"
        "s_mov_b32 %[st], 0\n\t"
        "s_mov_b32 %[l], 0\n\t"
        "s_mov_b32 %[e], 0\n"
        "L_sexit_%=:\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "s_mov_b64 exec, s[96:97]\n\t"
        : [i] "+s"(i), [st] "+s"(st), [l] "+s"(l), [e] "+s"(e), [flt] "+s"(flt)
        : [slots_lo] "s"(slots_lo), [slots_hi] "s"(slots_hi), [lr_lo] "s"(lr_lo),
          [lr_hi] "s"(lr_hi), [root_lo] "s"(root_lo), [root_hi] "s"(root_hi), [nb] "s"(nb),
          [m] "s"(m), [vocab] "s"(vocab), [tv] "v"(tv), [lane16] "v"(lane16)
        : "memory", "vcc", "scc",
          "s64", "s65", "s66", "s67", "s68", "s69", "s70", "s71", "s72", "s73", "s74", "s75",
          "s76", "s77", "s78", "s79", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95",
          "s96", "s97",
          "v41", "v42", "v43", "v44", "v45", "v46", "v47");
}

// Wave 0: feed `count` tokens to the static cursor; stops in front of a token
// outside the vocabulary (wave 1 reports it).
__device__ __forceinline__ void static_feed(const StaticView &S, const int32_t *tok, int64_t count,
                                            uint32_t vocab, int lane, uint32_t &s, uint32_t &l,
                                            uint32_t &e, uint32_t &fault, bool use_asm,
                                            bool have_first = false, uint32_t first = 0)
{
    bool stop = false;
    const bool in_asm = use_asm;          // the launcher sends corpora beyond 2^32 buckets to C++
    for (int64_t base = 0; base < count && !stop; base += 64) {
        const int m = (int)((count - base) < 64 ? (count - base) : 64);
        uint32_t tv;
        if (have_first && base == 0) tv = first;     // fetched by the caller with its other loads
        else tv = lane < m ? (uint32_t)tok[base + lane] : 0u;
        pin_v(tv);
        if (in_asm) {
            const uint64_t a_sl = (uint64_t)S.slots, a_lr = (uint64_t)S.linkrec,
                           a_rt = (uint64_t)S.root;
            uint32_t i = 0, flt = 0;
            uint32_t a_s = uni(s), a_l = uni(l), a_e = uni(e);
            static_feed_asm(uni((uint32_t)a_sl), uni((uint32_t)(a_sl >> 32)), uni((uint32_t)a_lr),
                            uni((uint32_t)(a_lr >> 32)), uni((uint32_t)a_rt),
                            uni((uint32_t)(a_rt >> 32)), uni((uint32_t)S.n_buckets),
                            uni((uint32_t)m), uni(vocab), tv, (uint32_t)(lane & 7) * 16u, i, a_s,
                            a_l, a_e, flt);
            s = a_s; l = a_l; e = a_e;
            fault |= flt;
            if ((int)i < m) stop = true;
        } else {
            for (int i = 0; i < m; i++) {
                const uint32_t t = lane_get(tv, i);
                if (t >= vocab) { stop = true; break; }
                static_transfer(S, t, lane, s, l, e, fault);
            }
        }
    }
}

// Wave 1: append `count` tokens to the sequence's dynamic automaton and text.
template <class L>
__device__ __forceinline__ void dyn_feed(const DynSeq &D, const int32_t *tok, int64_t count,
                                         uint32_t vocab, int lane, DynCursor<L> &c,
                                         uint32_t &fault, bool use_asm, bool have_first = false,
                                         uint32_t first = 0)
{
    bool stop = false;
    for (int64_t base = 0; base < count && !stop; base += 64) {
        const int m = (int)((count - base) < 64 ? (count - base) : 64);
        uint32_t tv;
        if (have_first && base == 0) tv = first;     // fetched by the caller with its other loads
        else tv = lane < m ? (uint32_t)tok[base + lane] : 0u;
        pin_v(tv);
        c.pf_ok = false;
        const uint32_t n_chunk = c.n;
        int fed = 0;
        bool in_asm = false;
        if constexpr (L::kSlots == 16) in_asm = use_asm;
        if constexpr (L::kSlots == 16) if (in_asm) {
            // values the two waves of a workgroup hold jointly count as per-lane for
            // the compiler; the assembly wants them in scalar registers
            const uint32_t nbk = uni(D.n_buckets), m_u = uni((uint32_t)m), vocab_u = uni(vocab);
            const u32x4 rrec = table_rsrc(D.rec, uni(c.rec_bytes));
            const u32x4 rslt = table_rsrc(D.slots, nbk * 128u);
            c.n = uni(c.n); c.n_states = uni(c.n_states); c.last = uni(c.last);
            c.n_trans = uni(c.n_trans); c.P = uni(c.P);
            const uint32_t lo = (uint32_t)(lane & 15) * 8u;
            if (!stop && fed < m) {
                uint32_t i = uni((uint32_t)fed), flt = 0;
                uint32_t r0 = uni((c.RP.len & 0xFFFFu) | (c.RP.link << 16));
                uint32_t r1 = uni((c.RP.endpos & 0xFFFFu) | (c.RP.head << 16));
                uint32_t r2 = uni(c.RP.itok), r3 = uni(c.RP.idst & 0xFFFFu);
                uint32_t a_n = uni(c.n), a_ns = uni(c.n_states), a_last = uni(c.last);
                uint32_t a_nt = uni(c.n_trans), a_P = uni(c.P);
                dyn_feed_compact(rrec, rslt, nbk, m_u, vocab_u, tv, lo, i, a_n, a_ns, a_last,
                                 a_nt, a_P, r0, r1, r2, r3, flt);
                c.n = a_n; c.n_states = a_ns; c.last = a_last; c.n_trans = a_nt; c.P = a_P;
                c.RP.len = r0 & 0xFFFFu; c.RP.link = L::widen(r0 >> 16);
                c.RP.endpos = r1 & 0xFFFFu; c.RP.head = L::widen(r1 >> 16);
                c.RP.itok = r2; c.RP.idst = r3;
                fed = (int)i;
                fault |= flt;
                if (fed < m) {
                    stop = true;
                    if (!flt) fault |= SAM_STATUS_TOKEN_BIT;
                }
            }
        }
        if (!in_asm) {
            for (; fed < m; fed++) {
                const uint32_t t = lane_get(tv, fed);
                if (t >= vocab) { stop = true; fault |= SAM_STATUS_TOKEN_BIT; break; }
                uint32_t tn = kNil;
                if (fed + 1 < m) {
                    tn = lane_get(tv, fed + 1);
                    if (tn >= vocab) tn = kNil;
                }
                dyn_expand<L>(D, t, tn, lane, c, fault);
            }
        }
        // the sequence's text, one coalesced store per chunk
        if (lane < fed) D.text[n_chunk + lane] = (int32_t)tv;
    }
}

template <class L>
__device__ __forceinline__ DynSeq dyn_region(const BatchView &B, int b)
{
    DynSeq D;
    D.text = B.dyn_text + (size_t)b * B.max_seq_len;
    D.rec = reinterpret_cast<char *>(B.dyn_rec) +
            (size_t)b * B.max_states * (B.compact ? sizeof(DynRecCompact) : sizeof(DynRec));
    D.slots = reinterpret_cast<char *>(B.dyn_slots) + (size_t)b * B.dyn_buckets * 128;
    D.n_buckets = B.dyn_buckets;
    return D;
}

template <class L>
__device__ __forceinline__ void load_cursor(const SeqMeta *meta, DynCursor<L> &c)
{
    c.n = uni(meta->n); c.n_states = uni(meta->n_states); c.last = uni(meta->last);
    c.n_trans = uni(meta->n_trans);
    c.P = uni(meta->s2);
    c.RP.len = uni(meta->p_len); c.RP.link = uni(meta->p_link);
    c.RP.endpos = uni(meta->p_endpos); c.RP.head = uni(meta->p_head);
    c.RP.itok = uni(meta->p_itok); c.RP.idst = uni(meta->p_idst);
    c.rec_bytes = 0;
    c.pf_ok = false;
    c.pf.b = 0; c.pf.mh = 0; c.pf.me = 0;
    c.pf.sl = typename L::RawSlot();
}

// The same from the 16 words of the block held one per lane (lane i = word i).
template <class L>
__device__ __forceinline__ void cursor_from_lanes(uint32_t mv, DynCursor<L> &c)
{
    c.n = lane_get(mv, 3); c.n_states = lane_get(mv, 4); c.last = lane_get(mv, 5);
    c.n_trans = lane_get(mv, 6);
    c.P = lane_get(mv, 8);
    c.RP.len = lane_get(mv, 9); c.RP.link = lane_get(mv, 10);
    c.RP.endpos = lane_get(mv, 11); c.RP.head = lane_get(mv, 12);
    c.RP.itok = lane_get(mv, 13); c.RP.idst = lane_get(mv, 14);
    c.rec_bytes = 0;
    c.pf_ok = false;
    c.pf.b = 0; c.pf.mh = 0; c.pf.me = 0;
    c.pf.sl = typename L::RawSlot();
}

// all of the dynamic cursor except meta->n (see the kernels for why)
template <class L>
__device__ __forceinline__ void store_cursor(SeqMeta *meta, const DynCursor<L> &c)
{
    meta->n_states = c.n_states; meta->last = c.last; meta->n_trans = c.n_trans;
    meta->s2 = c.P;
    meta->p_len = c.RP.len; meta->p_link = c.RP.link; meta->p_endpos = c.RP.endpos;
    meta->p_head = c.RP.head; meta->p_itok = c.RP.itok; meta->p_idst = c.RP.idst;
}

// Wave 0 after the barrier: choose the source (Section 3.2) and gather the draft.
__device__ __forceinline__ void emit_draft(const StaticView &S, const BatchView &B, int b, int lane,
                                           uint32_t l1, uint32_t e1, uint32_t l2, uint32_t e2,
                                           uint32_t n1, int32_t *match_len, int32_t *draft,
                                           int32_t *draft_len, int32_t *source)
{
    const bool use_static = B.has_static && ((int64_t)l1 > (int64_t)l2 + (int64_t)B.l_bias);
    const uint32_t ml = use_static ? l1 : l2;
    const uint32_t p = use_static ? (e1 & ~kWideBit) : e2;
    const int32_t *T = use_static ? S.text : B.dyn_text + (size_t)b * B.max_seq_len;
    const uint32_t Tn = use_static ? S.n_tokens : n1;
    const int Ld = B.draft_len;
    int dl = 0;
    if (ml > 0) {
        const uint32_t room = Tn - p;
        dl = room < (uint32_t)Ld ? (int)room : Ld;
    }
    for (int i = lane; i < Ld; i += 64)
        draft[(size_t)b * Ld + i] = i < dl ? T[p + i] : -1;
    if (lane == 0) {
        match_len[b] = (int32_t)ml;
        draft_len[b] = dl;
        int src = ml == 0 ? 0 : (use_static ? 2 : 1);
        if (B.l_threshold >= 0 && (int64_t)ml <= (int64_t)B.l_threshold) src = 3;
        source[b] = src;
    }
}

// ---- scout waves: memory-level parallelism for the two walks -----------------
//
// A walk is one chain of dependent loads, so a sequence keeps one or two memory
// requests in flight while the device could serve thousands.  What the chain will
// touch is largely predictable, though: after a mismatch both walks fall back to
// short suffixes of the text, i.e. to the states reached from the root by the
// strings x[j..k] for start positions j shortly before the position k being fed.
// A scout wave follows those strings for the start positions inside the step's row
// of tokens, several at a time, a few steps deep, and throws the results away: all it does is
// pull the records and buckets into the cache the walking wave reads through,
// where the walk then finds them in a fraction of the time of a miss.  Nothing the
// scouts read influences the result; they never write.

// How far each start position is followed.  Measured on the benchmark shapes: three
// transitions deep is the best trade between what the walks then find in the cache
// and what the scouts' own requests cost them in the queues they share; start
// positions before the step's first token (which need a dependent read of the
// sequence's text before the scouts can start) cost more than they bring.
constexpr int kScoutDepth = 3;

// Token of every start position, one per lane: lane j holds the step's token j, kNil
// beyond the row's end (or for a token outside the vocabulary).
__device__ __forceinline__ uint32_t scout_tokens(uint32_t tv, int count, uint32_t vocab, int lane)
{
    return (lane < count && tv < vocab) ? tv : kNil;
}

// Corpus automaton.  A bucket is fetched by 8 lanes (one slot each, one request per
// bucket, as in the walk), so the wave follows 8 start positions at a time and
// kRounds batches of 8 per transition depth; all their loads are in flight together.
__device__ __forceinline__ void scout_static(const StaticView &S, uint32_t tk, int n_starts, int lane)
{
    constexpr int kRounds = 3;                  // start positions 0 .. 23
    const int g = lane >> 3, i = lane & 7;
    uint32_t st[kRounds], ep[kRounds];          // state, its end position word (wide flag in bit 31)
    uint32_t acc = 0;
#pragma unroll
    for (int r = 0; r < kRounds; r++) {
        const int j = g + 8 * r;
        const uint32_t t0 = (uint32_t)__shfl((int)tk, j);
        st[r] = 0; ep[r] = 0;
        if (j < n_starts && t0 != kNil) {
            const uint2 re = reinterpret_cast<const uint2 *>(S.root)[t0];
            st[r] = re.x; ep[r] = re.y;
        }
    }
    for (int d = 1; d <= kScoutDepth; d++) {
        uint4 ra[kRounds], rb[kRounds];
        uint4 sl[kRounds];
        uint32_t tt[kRounds];
        bool on[kRounds];
        bool any = false;
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            const int j = g + 8 * r + d;
            tt[r] = (uint32_t)__shfl((int)tk, j & 63);
            on[r] = st[r] != 0 && st[r] < S.n_states && j < n_starts && tt[r] != kNil;
            ra[r] = make_uint4(kNil, 0, 0, kNil);
            rb[r] = make_uint4(0, 0, 0, 0);
            sl[r] = make_uint4(kNil, kNil, 0, 0);
            if (on[r]) {
                const uint4 *rec = reinterpret_cast<const uint4 *>(S.linkrec + st[r]);
                ra[r] = rec[0];                  // itok, idst, iendpos, itok2
                rb[r] = rec[1];                  // idst2, iendpos2, link, lenlink
                if (ep[r] & kWideBit) {
                    const uint64_t b = bucket_of(hash_key(st[r], tt[r]), S.n_buckets);
                    sl[r] = reinterpret_cast<const uint4 *>(S.slots)[b * kBucketSlots + i];
                }
            }
            any |= on[r];
        }
        if (!__any(any)) break;
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            const bool hit = on[r] && sl[r].x == st[r] && sl[r].y == tt[r];
            const uint32_t gm = (uint32_t)(__ballot(hit) >> (g * 8)) & 0xFFu;
            const int from = g * 8 + (gm ? __builtin_ctz(gm) : 0);
            const uint32_t sd = (uint32_t)__shfl((int)sl[r].z, from);
            const uint32_t se = (uint32_t)__shfl((int)sl[r].w, from);
            uint32_t nxt = 0, nep = 0;
            if (on[r]) {
                if (ra[r].x == tt[r]) { nxt = ra[r].y; nep = ra[r].z; }
                else if (ra[r].w == tt[r]) { nxt = rb[r].x; nep = rb[r].y; }
                else if (gm) { nxt = sd; nep = se; }
            }
            acc ^= rb[r].w;
            st[r] = nxt; ep[r] = nep;
        }
    }
    asm volatile("" :: "v"(acc), "v"(st[0]), "v"(st[1]), "v"(st[2]));
}

// The same over a sequence's own automaton in the compact layout (16-byte records,
// buckets of 16 slots of 8 bytes, fetched by 16 lanes: 4 start positions at a time).
// The tables change under the scout's eyes (wave 1 is extending them), so every index
// read from them is checked before it is used.
__device__ __forceinline__ void scout_dynamic_compact(const DynSeq &D, uint32_t max_states,
                                                      uint32_t tk, int n_starts, int lane)
{
    constexpr int kRounds = 5;                  // start positions 0 .. 19
    const uint4 *rec_t = reinterpret_cast<const uint4 *>(D.rec);
    const uint2 *slot_t = reinterpret_cast<const uint2 *>(D.slots);
    const int g = lane >> 4, i = lane & 15;
    uint32_t st[kRounds];                       // kNil: this start position is finished
    uint32_t acc = 0;
#pragma unroll
    for (int r = 0; r < kRounds; r++) st[r] = 0;                // the root
    for (int d = 0; d <= kScoutDepth; d++) {
        uint4 rec[kRounds];
        uint2 sl[kRounds];
        uint32_t tt[kRounds];
        bool on[kRounds];
        bool any = false;
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            const int j = g + 4 * r + d;
            tt[r] = (uint32_t)__shfl((int)tk, j & 63);
            on[r] = st[r] < max_states && j < n_starts && tt[r] != kNil;
            rec[r] = make_uint4(0, 0, kNil, 0);
            sl[r] = make_uint2(kNil, 0);
            if (on[r]) {
                rec[r] = rec_t[st[r]];
                sl[r] = slot_t[(size_t)dyn_bucket(D, st[r], tt[r]) * 16 + i];
            }
            any |= on[r];
        }
        if (!__any(any)) break;
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            const bool hit = on[r] && sl[r].x == ((st[r] << 17) | tt[r]);
            const uint32_t gm = (uint32_t)(__ballot(hit) >> (g * 16)) & 0xFFFFu;
            const uint32_t from = (uint32_t)__shfl((int)sl[r].y, g * 16 + (gm ? __builtin_ctz(gm) : 0));
            uint32_t nxt = kNil;
            if (on[r]) {
                if (rec[r].z == tt[r]) nxt = rec[r].w & 0xFFFFu;
                else if (gm) nxt = from & 0xFFFFu;
            }
            acc ^= rec[r].x;
            st[r] = nxt;
        }
    }
    asm volatile("" :: "v"(acc), "v"(st[0]), "v"(st[1]), "v"(st[2]), "v"(st[3]), "v"(st[4]));
}

}  // namespace

// One workgroup per sequence: two walking waves, and with kScout two scouts.  kIngest: sequence b is fed
// tokens[offsets[b] : offsets[b+1]) and nothing is written to the draft
// outputs.  Otherwise: sequence b is fed the first counts[b] tokens of
// tokens[b * max_accept ...], then source selection and draft gather.
template <class L, bool kIngest, bool kAsm, bool kScout>
__global__ __launch_bounds__(kScout ? 256 : 128) void sam_feed_kernel(StaticView S, BatchView B,
                                                        const int32_t *__restrict__ seq_map,
                                                        const int32_t *__restrict__ tokens,
                                                        const int64_t *__restrict__ offsets,
                                                        const int32_t *__restrict__ counts,
                                                        int32_t *__restrict__ match_len,
                                                        int32_t *__restrict__ draft,
                                                        int32_t *__restrict__ draft_len,
                                                        int32_t *__restrict__ source)
{
    __shared__ uint32_t sh[8];
    // ingest may address a subset of the batch: workgroup i serves sequence seq_map[i]
    const int b = (kIngest && seq_map) ? seq_map[blockIdx.x] : (int)blockIdx.x;
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    static_assert(!(kIngest && kScout), "scouts belong to the step kernel");
    if (kScout) {
        // the arrival counter of the two walking waves (see the end of the kernel)
        if (threadIdx.x == 0) sh[7] = 0;
        __syncthreads();
    }

    // Kernel arguments span three cache lines; named together here, they are all
    // requested before the first of them is waited for.
    {
        const uint32_t a0 = (uint32_t)(uintptr_t)S.slots, a1 = (uint32_t)(uintptr_t)B.meta,
                       a2 = (uint32_t)(uintptr_t)B.dyn_slots, a3 = (uint32_t)(uintptr_t)tokens,
                       a4 = (uint32_t)(uintptr_t)source;
        asm volatile("" :: "s"(a0), "s"(a1), "s"(a2), "s"(a3), "s"(a4));
    }
    SeqMeta *meta = &B.meta[b];

    // A step's first round trip fetches everything it needs before its first token
    // at once: the cursor block (16 words, one per lane), the count and the row of
    // accepted tokens.  Read one after the other they cost a launch three to five
    // dependent misses, which is a tenth of a whole step.
    static_assert(sizeof(SeqMeta) == 64, "the cursor block is read as 16 words");
    uint32_t mv = reinterpret_cast<const uint32_t *>(meta)[lane & 15];
    const int32_t *tok;
    int64_t count;
    uint32_t fault = 0;
    uint32_t first = 0;
    if (kIngest) {
        const int64_t o0 = offsets[blockIdx.x], o1 = offsets[blockIdx.x + 1];
        tok = tokens + o0;
        count = o1 - o0;
    } else {
        tok = tokens + (int64_t)b * B.max_accept;
        uint32_t raw = (uint32_t)counts[b];
        first = lane < B.max_accept ? (uint32_t)tok[lane] : 0u;   // the row exists whatever the count
        asm volatile("" : "+v"(mv), "+v"(first), "+s"(raw));      // all three in flight before any is used
        count = (int32_t)raw;
        if (count < 0 || count > B.max_accept) { fault |= SAM_STATUS_COUNT_BIT; count = 0; }
    }
    pin_v(mv);
    const uint32_t n0 = lane_get(mv, 3);
    count = (int64_t)uni((uint32_t)count);
    if ((int64_t)n0 + count > (int64_t)B.max_seq_len) { fault |= SAM_STATUS_CAPACITY_BIT; count = 0; }
    const uint32_t vocab = (uint32_t)B.vocab;

    if (kScout && wave >= 2) {
        // the step's scouts (waves 2 and 3): prefetch, then leave; the barrier below
        // waits for the two walking waves only
        if (count > 0) {
            const DynSeq D = dyn_region<L>(B, b);
            const uint32_t tk = scout_tokens(first, (int)count, vocab, lane);
            const int n_starts = count < 64 ? (int)count : 64;
            if (wave == 2) {
                if (B.has_static) scout_static(S, tk, n_starts, lane);
            } else {
                if (L::kSlots == 16) scout_dynamic_compact(D, B.max_states, tk, n_starts, lane);
            }
        }
        return;
    }

    if (wave == 0) {
        uint32_t s = lane_get(mv, 0), l = lane_get(mv, 1), e = lane_get(mv, 2);
        if (B.has_static) static_feed(S, tok, count, vocab, lane, s, l, e, fault, kAsm, !kIngest, first);
        if (lane == 0) { sh[0] = s; sh[1] = l; sh[2] = e; sh[6] = fault & SAM_STATUS_INTERNAL_BIT; }
    } else {
        const DynSeq D = dyn_region<L>(B, b);
        DynCursor<L> c;
        cursor_from_lanes<L>(mv, c);
        c.rec_bytes = (uint32_t)B.max_states * 16u;
        // The first token of a step finds nothing of the sequence's tables in the caches,
        // and its lookups come one after the other: the bucket at P, then record and
        // bucket one suffix link up, then at the root.  Their addresses are all known
        // now, so they are requested here at once and not waited for (the value is only
        // named again after the token loop); the loop's own requests then meet them on
        // the way or in the cache.
        uint32_t warm = 0;
        if (kScout && L::kSlots == 16 && count > 0 && c.P != kNil) {
            const uint32_t t0 = lane_get(first, 0);
            if (t0 < vocab) {
                const uint32_t up = c.RP.link == kNil ? 0u : c.RP.link;
                const uint32_t at = lane < 16 ? c.P : (lane < 32 ? up : 0u);
                const uint2 *slots = reinterpret_cast<const uint2 *>(D.slots);
                if (lane < 48 && at < B.max_states)
                    warm = slots[(size_t)dyn_bucket(D, at, t0) * 16 + (lane & 15)].y;
                else if (lane < 50 && up < B.max_states)
                    warm = reinterpret_cast<const uint4 *>(D.rec)[lane == 48 ? up : 0u].x;
            }
        }
        dyn_feed<L>(D, tok, count, vocab, lane, c, fault, kAsm, !kIngest, first);
        asm volatile("" :: "v"(warm));
        if (c.n != n0) flush_last<L>(D, c, lane);
        if (lane == 0) {
            sh[3] = c.P == kNil ? 0u : c.RP.len;
            sh[4] = c.P == kNil ? 0u : c.RP.endpos;
            sh[5] = c.n;
            store_cursor<L>(meta, c);
            if (fault) {
                meta->status |= fault;
                atomicOr(B.status, fault);
            }
        }
    }
    if (!kScout) {
        __syncthreads();
        if (wave == 1) return;
    } else {
        // The step's workgroup also holds the scouts, which a barrier would wait for, and
        // neither walking wave should wait for the other.  Each of the two counts itself
        // in when its words above (and, for wave 1, its text stores) are written; the one
        // that comes second sees both halves and finishes the step, the first one leaves.
        uint32_t before = 0;
        if (lane == 0)
            before = __hip_atomic_fetch_add(&sh[7], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (uni(before) == 0u) {
            // first to arrive: nothing left to do -- except, for the static walk, to ask
            // for the corpus text its draft would be read from, so that the wave that
            // finishes the step finds it on the way
            if (wave == 0 && B.has_static && sh[1] > 0) {
                const uint32_t at = (sh[2] & ~kWideBit) + 32u * (uint32_t)lane;
                if (32 * lane < B.draft_len + 32 && at < S.n_tokens) {
                    const int32_t v = S.text[at];
                    asm volatile("" :: "v"(v));
                }
            }
            return;
        }
    }
    // meta->n is read by both waves at the top, long before either gets here
    const uint32_t s1 = sh[0], l1 = sh[1], e1 = sh[2];
    if (lane == 0) {
        meta->n = sh[5];
        meta->s1 = s1; meta->l1 = l1; meta->e1 = e1;
        if (sh[6]) atomicOr(B.status, sh[6]);
    }
    if (kIngest) return;
    emit_draft(S, B, b, lane, l1, e1, sh[3], sh[4], sh[5], match_len, draft, draft_len, source);
}

// The same work for a whole schedule of steps in one launch: workgroup b runs
// sequence b through steps 0 .. n_steps-1 on its own, so no sequence waits for
// the longest row of another and nothing is launched in between.  Step s reads
// accepted[s, b, :] and counts[s, b] and writes row (s, b) of the outputs.  The
// cursors stay in registers from step to step.
template <class L, bool kAsm>
__global__ __launch_bounds__(128) void sam_replay_kernel(StaticView S, BatchView B, int n_steps,
                                                          const int32_t *__restrict__ accepted,
                                                          const int32_t *__restrict__ counts,
                                                          int32_t *__restrict__ match_len,
                                                          int32_t *__restrict__ draft,
                                                          int32_t *__restrict__ draft_len,
                                                          int32_t *__restrict__ source)
{
    __shared__ uint32_t sh[8];
    const int b = blockIdx.x;
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    SeqMeta *meta = &B.meta[b];
    const uint32_t vocab = (uint32_t)B.vocab;
    const size_t nb = (size_t)B.batch;
    uint32_t fault = 0;
    uint32_t n_cur = uni(meta->n);

    uint32_t s = 0, l = 0, e = 0;
    DynSeq D = dyn_region<L>(B, b);
    DynCursor<L> c;
    if (wave == 0) { s = uni(meta->s1); l = uni(meta->l1); e = uni(meta->e1); }
    load_cursor<L>(meta, c);
    c.rec_bytes = (uint32_t)B.max_states * 16u;
    const uint32_t n_first = n_cur;

    for (int step = 0; step < n_steps; step++) {
        const int32_t *tok = accepted + ((size_t)step * nb + b) * B.max_accept;
        int64_t count = counts[(size_t)step * nb + b];
        if (count < 0 || count > B.max_accept) { fault |= SAM_STATUS_COUNT_BIT; count = 0; }
        count = (int64_t)uni((uint32_t)count);
        if ((int64_t)n_cur + count > (int64_t)B.max_seq_len) { fault |= SAM_STATUS_CAPACITY_BIT; count = 0; }
        if (wave == 0) {
            if (B.has_static) static_feed(S, tok, count, vocab, lane, s, l, e, fault, kAsm);
        } else {
            dyn_feed<L>(D, tok, count, vocab, lane, c, fault, kAsm);
            if (lane == 0) {
                sh[3] = c.P == kNil ? 0u : c.RP.len;
                sh[4] = c.P == kNil ? 0u : c.RP.endpos;
                sh[5] = c.n;
            }
        }
        __syncthreads();                 // the step's text and wave 1's cursor are visible
        n_cur = sh[5];
        if (wave == 0)
            emit_draft(S, B, b, lane, l, e, sh[3], sh[4], n_cur, match_len + (size_t)step * nb,
                       draft + (size_t)step * nb * B.draft_len, draft_len + (size_t)step * nb,
                       source + (size_t)step * nb);
        __syncthreads();                 // sh is rewritten by the next step
    }

    if (wave == 0) {
        if (lane == 0) {
            meta->s1 = s; meta->l1 = l; meta->e1 = e;
            if (fault & SAM_STATUS_INTERNAL_BIT) atomicOr(B.status, SAM_STATUS_INTERNAL_BIT);
        }
    } else {
        if (c.n != n_first) flush_last<L>(D, c, lane);
        if (lane == 0) {
            store_cursor<L>(meta, c);
            meta->n = c.n;
            if (fault) {
                meta->status |= fault;
                atomicOr(B.status, fault);
            }
        }
    }
}

// Fresh sequences: root record, empty cursors.  The slot tables are filled with
// the empty key by the caller.
__global__ void sam_reset_kernel(BatchView B, const int32_t *seq_map, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int b = seq_map ? seq_map[i] : i;
    Rec r;
    r.len = 0; r.link = kNil; r.endpos = 0; r.head = kNil; r.itok = kNil; r.idst = 0;
    if (B.compact) {
        CompactDyn::store_rec(reinterpret_cast<char *>(B.dyn_rec) +
                                  (size_t)b * B.max_states * sizeof(DynRecCompact), 0, r);
    } else {
        void *base = reinterpret_cast<char *>(B.dyn_rec) + (size_t)b * B.max_states * sizeof(DynRec);
        WideDyn::store_rec(base, 0, r);
        DynRec *d = reinterpret_cast<DynRec *>(base);
        d->pad0 = 0; d->pad1 = 0;
    }
    SeqMeta m = {};
    m.n_states = 1;
    m.s2 = kNil;
    m.p_link = kNil; m.p_head = kNil; m.p_itok = kNil;
    B.meta[b] = m;
    if (!seq_map && b == 0) *B.status = 0;
}

// Empty the slot tables of the listed sequences (every key = kNil).
__global__ void sam_clear_slots_kernel(BatchView B, const int32_t *seq_map)
{
    const int b = seq_map[blockIdx.x];
    uint4 *base = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(B.dyn_slots) +
                                           (size_t)b * B.dyn_buckets * 128);
    const size_t n16 = (size_t)B.dyn_buckets * 8;
    for (size_t i = (size_t)blockIdx.y * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.y * blockDim.x)
        base[i] = make_uint4(kNil, kNil, kNil, kNil);
}

// Fill a 16-byte aligned region with the empty key (every byte 0xFF).
__global__ void sam_fill_empty_kernel(uint4 *base, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * blockDim.x)
        base[i] = make_uint4(kNil, kNil, kNil, kNil);
}

__global__ void sam_debug_kernel(BatchView B, int32_t *s1, int32_t *l1, int32_t *s2, int32_t *l2,
                                 int32_t *text_len, int32_t *n_states, int32_t *n_trans)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B.batch) return;
    const SeqMeta m = B.meta[b];
    if (s1) s1[b] = (int32_t)m.s1;
    if (l1) l1[b] = (int32_t)m.l1;
    if (s2) s2[b] = m.s2 == kNil ? 0 : (int32_t)m.s2;
    if (l2) l2[b] = m.s2 == kNil ? 0 : (int32_t)m.p_len;
    if (text_len) text_len[b] = (int32_t)m.n;
    if (n_states) n_states[b] = (int32_t)m.n_states;
    if (n_trans) n_trans[b] = (int32_t)m.n_trans;
}

// ---- the static state records, built once per corpus ------------------------
//
// While the passes below run, the fields of a record hold intermediate values:
// word 0 the number of transitions seen, words 2-3 and 4-5 two 64-bit keys.
// A transition's key is (0 if its target was created after the state, else 1) in
// the upper half and the target in the lower: the smallest key is the transition
// the record repeats first, the next one the second.

__device__ __forceinline__ unsigned long long staterec_key(const Slot &sl)
{
    return ((unsigned long long)(sl.dst > sl.state ? 0u : 1u) << 32) | sl.dst;
}

__global__ void sam_staterec_init_kernel(const LinkPair *pairs, LinkRec *rec, uint32_t n_states)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; s < n_states; s += stride) {
        LinkRec r;
        r.itok = 0;                                            // transitions seen
        r.idst = kNil;
        r.iendpos = kNil; r.itok2 = kNil;                      // first key
        r.idst2 = kNil; r.iendpos2 = kNil;                     // second key
        r.link = pairs[s].link; r.lenlink = pairs[s].lenlink;
        rec[s] = r;
    }
}

// pass 0: count, smallest key; pass 1: smallest key but the first
__global__ void sam_staterec_pick_kernel(const Slot *slots, LinkRec *rec, uint64_t n_slots, int pass)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_slots; i += stride) {
        const Slot sl = slots[i];
        if (sl.state == kNil) continue;
        LinkRec *r = &rec[sl.state];
        unsigned long long *k0 = reinterpret_cast<unsigned long long *>(&r->iendpos);
        unsigned long long *k1 = reinterpret_cast<unsigned long long *>(&r->idst2);
        const unsigned long long key = staterec_key(sl);
        if (pass == 0) {
            atomicAdd(&r->itok, 1u);
            atomicMin(k0, key);
        } else if (key != *k0) {
            atomicMin(k1, key);
        }
    }
}

// wide[s / 32] bit s % 32: the state has more transitions than its record repeats;
// the record's targets move to their places, tokens and end positions follow in the
// next pass
__global__ void sam_staterec_settle_kernel(LinkRec *rec, uint32_t *wide, uint32_t n_states)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; s < n_states; s += stride) {
        LinkRec r = rec[s];
        if (r.itok > 2) atomicOr(&wide[s >> 5], 1u << (s & 31));
        const uint32_t d0 = r.iendpos, d1 = r.idst2;           // lower halves of the two keys
        r.itok = kNil; r.idst = d0; r.iendpos = 0;
        r.itok2 = kNil; r.idst2 = d1; r.iendpos2 = 0;
        rec[s] = r;
    }
}

__device__ __forceinline__ uint32_t wide_flag(const uint32_t *wide, uint32_t s)
{
    return ((wide[s >> 5] >> (s & 31)) & 1u) ? kWideBit : 0u;
}

// tokens and end positions of the repeated transitions; every slot's end position
// gets the wide flag of its target
__global__ void sam_staterec_fill_kernel(Slot *slots, LinkRec *rec, const uint32_t *wide,
                                         uint64_t n_slots)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_slots; i += stride) {
        const Slot sl = slots[i];
        if (sl.state == kNil) continue;
        const uint32_t w = sl.w | wide_flag(wide, sl.dst);
        slots[i].w = w;
        LinkRec *r = &rec[sl.state];
        if (r->idst == sl.dst) { r->itok = sl.token; r->iendpos = w; }
        else if (r->idst2 == sl.dst) { r->itok2 = sl.token; r->iendpos2 = w; }
    }
}

// the wide flag of the suffix link's state, and of the root's targets
__global__ void sam_staterec_links_kernel(LinkRec *rec, RootEnt *root, const uint32_t *wide,
                                          uint32_t n_states, uint32_t vocab)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; s < n_states; s += stride) {
        rec[s].lenlink |= wide_flag(wide, rec[s].link);
        if (s < vocab && root[s].dst) root[s].endpos |= wide_flag(wide, root[s].dst);
    }
    // a vocabulary larger than the state count (tiny corpora)
    for (uint64_t t = n_states + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < vocab; t += stride)
        if (root[t].dst) root[t].endpos |= wide_flag(wide, root[t].dst);
}

// ---- the device's transition table: wide states only --------------------------
//
// A narrow state (at most two transitions) is answered by its record, so no lookup
// ever asks the table for one of its transitions.  The table the walks probe is
// therefore rebuilt on the device with the transitions of wide states alone, at
// load 0.5: a fraction of the host's table, which holds every transition.

__global__ void sam_count_wide_kernel(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                                      unsigned long long *count)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_slots; i += stride) {
        const uint32_t st = slots[i].state;
        if (st != kNil && wide_flag(wide, st)) mine++;
    }
    if (mine) atomicAdd(count, mine);
}

// Insert every transition of a wide state into the new table (all keys kNil before):
// a slot is claimed by an atomic exchange of its state word, the other words follow;
// nothing looks the table up before this kernel has finished.
__global__ void sam_compact_slots_kernel(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                                         Slot *out, uint64_t n_buckets)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_slots; i += stride) {
        const Slot sl = slots[i];
        if (sl.state == kNil || !wide_flag(wide, sl.state)) continue;
        uint64_t b = bucket_of(hash_key(sl.state, sl.token), n_buckets);
        bool placed = false;
        for (uint64_t left = n_buckets; left && !placed; left--) {
            for (int j = 0; j < kBucketSlots && !placed; j++) {
                Slot *dst = out + b * kBucketSlots + j;
                if (dst->state == kNil && atomicCAS(&dst->state, kNil, sl.state) == kNil) {
                    dst->token = sl.token;
                    dst->dst = sl.dst;
                    dst->w = sl.w;
                    placed = true;
                }
            }
            b = (b + 1 == n_buckets) ? 0 : b + 1;
        }
    }
}

// ---- launchers (called from the C ABI) ------------------------------------

hipError_t launch_staterec(const LinkPair *pairs, Slot *slots, RootEnt *root, LinkRec *linkrec,
                           uint32_t *wide, uint32_t n_states, uint64_t n_slots, uint32_t vocab,
                           hipStream_t stream)
{
    hipLaunchKernelGGL(sam_staterec_init_kernel, dim3(4096), dim3(256), 0, stream, pairs, linkrec,
                       n_states);
    hipLaunchKernelGGL(sam_staterec_pick_kernel, dim3(8192), dim3(256), 0, stream, slots, linkrec,
                       n_slots, 0);
    hipLaunchKernelGGL(sam_staterec_pick_kernel, dim3(8192), dim3(256), 0, stream, slots, linkrec,
                       n_slots, 1);
    hipLaunchKernelGGL(sam_staterec_settle_kernel, dim3(4096), dim3(256), 0, stream, linkrec, wide,
                       n_states);
    hipLaunchKernelGGL(sam_staterec_fill_kernel, dim3(8192), dim3(256), 0, stream, slots, linkrec,
                       wide, n_slots);
    hipLaunchKernelGGL(sam_staterec_links_kernel, dim3(4096), dim3(256), 0, stream, linkrec, root,
                       wide, n_states, vocab);
    return hipGetLastError();
}

hipError_t launch_count_wide(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                             unsigned long long *count, hipStream_t stream)
{
    hipLaunchKernelGGL(sam_count_wide_kernel, dim3(8192), dim3(256), 0, stream, slots, wide,
                       n_slots, count);
    return hipGetLastError();
}

hipError_t launch_compact_slots(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                                Slot *out, uint64_t n_buckets, hipStream_t stream)
{
    hipLaunchKernelGGL(sam_compact_slots_kernel, dim3(8192), dim3(256), 0, stream, slots, wide,
                       n_slots, out, n_buckets);
    return hipGetLastError();
}

hipError_t launch_feed(const StaticView &S, const BatchView &B, const int32_t *seq_map,
                       int n_seqs, const int32_t *tokens, const int64_t *offsets,
                       const int32_t *counts, int32_t *match_len, int32_t *draft,
                       int32_t *draft_len, int32_t *source, hipStream_t stream)
{
    const bool scout = !offsets && B.scout;
    const dim3 grid(n_seqs), block(scout ? 256 : 128);
#define SAM_LAUNCH_FEED(LAYOUT, INGEST, ASM, SCOUT)                                            \
    hipLaunchKernelGGL((sam_feed_kernel<LAYOUT, INGEST, ASM, SCOUT>), grid, block, 0, stream,  \
                       S, B, seq_map, tokens, offsets, counts, match_len, draft, draft_len,    \
                       source)
    const int which = (B.compact ? 4 : 0) | (offsets ? 2 : 0) | ((B.no_asm || (S.n_buckets >> 32)) ? 0 : 1);
    switch (which) {
    case 7: SAM_LAUNCH_FEED(CompactDyn, true, true, false); break;
    case 6: SAM_LAUNCH_FEED(CompactDyn, true, false, false); break;
    case 5: if (scout) SAM_LAUNCH_FEED(CompactDyn, false, true, true);
            else SAM_LAUNCH_FEED(CompactDyn, false, true, false);
            break;
    case 4: if (scout) SAM_LAUNCH_FEED(CompactDyn, false, false, true);
            else SAM_LAUNCH_FEED(CompactDyn, false, false, false);
            break;
    case 3: SAM_LAUNCH_FEED(WideDyn, true, true, false); break;
    case 2: SAM_LAUNCH_FEED(WideDyn, true, false, false); break;
    case 1: if (scout) SAM_LAUNCH_FEED(WideDyn, false, true, true);
            else SAM_LAUNCH_FEED(WideDyn, false, true, false);
            break;
    default: if (scout) SAM_LAUNCH_FEED(WideDyn, false, false, true);
             else SAM_LAUNCH_FEED(WideDyn, false, false, false);
             break;
    }
#undef SAM_LAUNCH_FEED
    return hipGetLastError();
}

hipError_t launch_replay(const StaticView &S, const BatchView &B, int n_steps,
                         const int32_t *accepted, const int32_t *counts, int32_t *match_len,
                         int32_t *draft, int32_t *draft_len, int32_t *source, hipStream_t stream)
{
    const dim3 grid(B.batch), block(128);
#define SAM_LAUNCH_REPLAY(LAYOUT, ASM)                                                         \
    hipLaunchKernelGGL((sam_replay_kernel<LAYOUT, ASM>), grid, block, 0, stream, S, B, n_steps, \
                       accepted, counts, match_len, draft, draft_len, source)
    const bool cxx = B.no_asm || (S.n_buckets >> 32);
    if (B.compact) {
        if (cxx) SAM_LAUNCH_REPLAY(CompactDyn, false); else SAM_LAUNCH_REPLAY(CompactDyn, true);
    } else {
        if (cxx) SAM_LAUNCH_REPLAY(WideDyn, false); else SAM_LAUNCH_REPLAY(WideDyn, true);
    }
#undef SAM_LAUNCH_REPLAY
    return hipGetLastError();
}

hipError_t launch_reset(const BatchView &B, const int32_t *seq_map, int n_seqs,
                        hipStream_t stream)
{
    if (seq_map) {
        hipLaunchKernelGGL(sam_clear_slots_kernel, dim3(n_seqs, 16), dim3(256), 0, stream, B,
                           seq_map);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(sam_reset_kernel, dim3((n_seqs + 127) / 128), dim3(128), 0, stream, B,
                       seq_map, n_seqs);
    return hipGetLastError();
}

hipError_t launch_fill_empty(void *base, size_t bytes, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 255) / 256;
    hipLaunchKernelGGL(sam_fill_empty_kernel, dim3((unsigned)(want < 4096 ? want : 4096)), dim3(256),
                       0, stream, reinterpret_cast<uint4 *>(base), n16);
    return hipGetLastError();
}

hipError_t launch_debug(const BatchView &B, int32_t *s1, int32_t *l1, int32_t *s2, int32_t *l2,
                        int32_t *text_len, int32_t *n_states, int32_t *n_trans,
                        hipStream_t stream)
{
    hipLaunchKernelGGL(sam_debug_kernel, dim3((B.batch + 127) / 128), dim3(128), 0, stream, B,
                       s1, l1, s2, l2, text_len, n_states, n_trans);
    return hipGetLastError();
}

}  // namespace sam
