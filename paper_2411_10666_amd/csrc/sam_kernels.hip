// gfx950 kernels for batched suffix-automaton matching, online extension and
// draft gather (arxiv 2411.10666: Algorithm 1 Transfer, Algorithm 2 Expand,
// Section 3.2 draft read and source selection, Section 3.3 update order).
//
// Execution shape: one workgroup of two 64-lane wavefronts per sequence.
//   wave 0  walks the static automaton (read-only tables in HBM),
//   wave 1  extends the sequence's own dynamic automaton,
// both over the same accepted tokens and concurrently; they meet at one
// barrier, after which wave 0 selects the source and gathers the draft with
// coalesced reads.  Inside a wave all control flow is wave-uniform: the lanes
// are used to fetch a whole 128-byte hash bucket (8 slots) in one request and
// to resolve it with a ballot, so a lookup costs one memory round trip whatever
// the state's out-degree.  Sequence b is always served by workgroup b, so its
// private tables keep hitting the L2 of the same XCD from launch to launch.
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

__device__ __forceinline__ void order_memory()
{
    // stores and later loads of one wavefront reach memory in program order;
    // this only stops the compiler from moving them across each other
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

// ---- static automaton: Transfer (Algorithm 1) -----------------------------

// Feed one token.  (s, l) is the cursor, e = min_endpos(s).
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
        // fetch the suffix-link record together with the bucket: it is only
        // needed on a miss, but then it is already here
        const LinkRec lr = S.linkrec[s];
        uint64_t b = bucket_of(hash_key(s, t), S.n_buckets);
        uint4 sl = reinterpret_cast<const uint4 *>(S.slots)[b * kBucketSlots + (lane & 7)];
        uint32_t mh = (uint32_t)__ballot(sl.x == s && sl.y == t) & 0xFFu;
        uint32_t me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
        uint32_t nlink = uni(lr.link), nlen = uni(lr.lenlink);
        pin_s(nlink);
        pin_s(mh);
        bool hit = false;
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
        if (hit) return;
        s = nlink;
        l = nlen;
    }
}

// ---- dynamic automaton: Expand (Algorithm 2) ------------------------------

struct DynSeq {
    int32_t *text;
    DynRec  *rec;
    Slot    *slots;
    uint32_t n_buckets;
};

struct Rec {              // a DynRec held in wave-uniform registers
    uint32_t len, link, endpos, head, itok, idst;
};

struct RawRec { uint4 a; uint2 b; };

__device__ __forceinline__ RawRec issue_rec(const DynRec *r)
{
    RawRec w;
    w.a = reinterpret_cast<const uint4 *>(r)[0];
    w.b = reinterpret_cast<const uint2 *>(r)[2];
    return w;
}

__device__ __forceinline__ Rec finish_rec(const RawRec &w)
{
    const uint4 a = w.a;
    const uint2 b = w.b;
    Rec R;
    R.len = uni(a.x); R.link = uni(a.y); R.endpos = uni(a.z); R.head = uni(a.w);
    R.itok = uni(b.x); R.idst = uni(b.y);
    return R;
}

__device__ __forceinline__ Rec load_rec(const DynRec *r) { return finish_rec(issue_rec(r)); }

__device__ __forceinline__ void store_rec(DynRec *r, const Rec &R, int lane)
{
    if (lane == 0) {
        reinterpret_cast<uint4 *>(r)[0] = make_uint4(R.len, R.link, R.endpos, R.head);
        reinterpret_cast<uint2 *>(r)[2] = make_uint2(R.itok, R.idst);
    }
}

// Look (p, t) up in the sequence's slot table.  Hit: returns true, `at` = slot
// index, `dst` = target.  Miss: returns false, `at` = first empty slot on the
// probe path (where an insert of this key goes).  `sl` is the already issued
// load of the key's home bucket (see issue_bucket).
__device__ __forceinline__ uint4 issue_bucket(const DynSeq &D, uint32_t b, int lane)
{
    return reinterpret_cast<const uint4 *>(D.slots)[b * kBucketSlots + (lane & 7)];
}

__device__ __forceinline__ bool resolve_probe(const DynSeq &D, uint32_t p, uint32_t t, int lane,
                                              uint32_t b, uint4 sl, uint32_t &at, uint32_t &dst)
{
    // the table always has empty slots (at most 3/4 full), so this ends long
    // before the bound; a full sweep reports "absent, nowhere to insert"
    for (uint32_t left = D.n_buckets; ; left--) {
        if (left == 0) { at = kNil; return false; }
        const uint32_t mh = (uint32_t)__ballot(sl.x == p && sl.y == t) & 0xFFu;
        if (mh) {
            const int j = __builtin_ctz(mh);
            at = b * kBucketSlots + j;
            dst = lane_get(sl.z, j);
            return true;
        }
        const uint32_t me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
        if (me) {
            at = b * kBucketSlots + __builtin_ctz(me);
            return false;
        }
        b = (b + 1 == D.n_buckets) ? 0 : b + 1;
        sl = issue_bucket(D, b, lane);
    }
}

__device__ __forceinline__ bool dyn_probe(const DynSeq &D, uint32_t p, uint32_t t, int lane,
                                          uint32_t &at, uint32_t &dst)
{
    const uint32_t b = (uint32_t)bucket_of(hash_key(p, t), D.n_buckets);
    return resolve_probe(D, p, t, lane, b, issue_bucket(D, b, lane), at, dst);
}

// Record of p and the bucket of (p, t) fetched in one round trip: both loads are
// issued, then both are consumed in the same straight-line block (the first
// ballots and the record's words), so neither can be sunk behind a branch that
// depends on the other.
__device__ __forceinline__ bool rec_and_probe(const DynSeq &D, uint32_t p, uint32_t t, int lane,
                                              Rec &R, uint32_t &at, uint32_t &dst)
{
    const RawRec raw = issue_rec(&D.rec[p]);
    uint32_t b = (uint32_t)bucket_of(hash_key(p, t), D.n_buckets);
    uint4 sl = issue_bucket(D, b, lane);
    uint32_t mh = (uint32_t)__ballot(sl.x == p && sl.y == t) & 0xFFu;
    uint32_t me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
    R = finish_rec(raw);
    pin_s(R.itok);
    pin_s(mh);
    for (uint32_t left = D.n_buckets; ; left--) {
        if (mh) {
            const int j = __builtin_ctz(mh);
            at = b * kBucketSlots + j;
            dst = lane_get(sl.z, j);
            return true;
        }
        if (me) {
            at = b * kBucketSlots + __builtin_ctz(me);
            return false;
        }
        if (left == 0) { at = kNil; return false; }
        b = (b + 1 == D.n_buckets) ? 0 : b + 1;
        sl = issue_bucket(D, b, lane);
        mh = (uint32_t)__ballot(sl.x == p && sl.y == t) & 0xFFu;
        me = (uint32_t)__ballot(sl.x == kNil) & 0xFFu;
    }
}

constexpr uint32_t kInline = 0xFFFFFFFEu;   // "the transition sits in the record"

struct DynCursor {
    uint32_t n, n_states, last, n_trans;
    uint32_t s2, l2, e2;      // link(last), its length, its min_endpos
};

// Append token t (Algorithm 2).  Afterwards (s2, l2) is the state and length of
// the longest suffix of the sequence that also ends earlier in it, which is
// what the paper's Transfer-then-Expand order leaves in the dynamic cursor.
__device__ __forceinline__ void dyn_expand(const DynSeq &D, uint32_t t, int lane, DynCursor &c,
                                           uint32_t &fault)
{
    // Suffix links strictly shorten, so every chain below ends at the root after
    // fewer than n_states moves; `guard` turns a corrupted table into a status
    // bit instead of an endless loop.
    uint32_t guard = c.n_states + 4;
    const uint32_t k = c.n + 1;
    const uint32_t cur = c.n_states++;
    const uint32_t last = c.last;

    // `last` never has a transition yet: its first one goes inline
    if (lane == 0)
        reinterpret_cast<uint2 *>(&D.rec[last])[2] = make_uint2(t, cur);
    c.n_trans++;
    order_memory();

    uint32_t p = c.s2;
    if (last == 0) p = kNil;               // root's link
    Rec R = {};
    uint32_t q = kNil, where = kNil;
    while (p != kNil) {
        if (--guard == 0) { fault |= SAM_STATUS_INTERNAL_BIT; p = kNil; break; }
        uint32_t at, dst;
        const bool hit = rec_and_probe(D, p, t, lane, R, at, dst);
        if (R.itok == t) { q = R.idst; where = kInline; break; }
        if (hit)         { q = dst;    where = at;      break; }
        if (R.itok == kNil) {
            if (lane == 0)
                reinterpret_cast<uint2 *>(&D.rec[p])[2] = make_uint2(t, cur);
        } else if (at == kNil) {
            fault |= SAM_STATUS_INTERNAL_BIT;
        } else {
            if (lane == 0) {
                reinterpret_cast<uint4 *>(D.slots)[at] = make_uint4(p, t, cur, R.head);
                D.rec[p].head = at;
            }
        }
        c.n_trans++;
        order_memory();
        p = R.link;
    }

    uint32_t linkc, l2, e2;
    if (p == kNil) {
        linkc = 0; l2 = 0; e2 = 0;
    } else {
        Rec Q = load_rec(&D.rec[q]);
        if (q == last) { Q.itok = t; Q.idst = cur; }
        if (R.len + 1 == Q.len) {
            linkc = q; l2 = Q.len; e2 = Q.endpos;
        } else {
            const uint32_t cl = c.n_states++;
            Rec CL;
            CL.len = R.len + 1; CL.link = Q.link; CL.endpos = Q.endpos;
            CL.head = kNil; CL.itok = Q.itok; CL.idst = Q.idst;
            if (Q.itok != kNil) c.n_trans++;
            // copy q's further transitions
            for (uint32_t j = Q.head; j != kNil;) {
                if (--guard == 0 || j >= D.n_buckets * kBucketSlots) {
                    fault |= SAM_STATUS_INTERNAL_BIT;
                    break;
                }
                const uint4 sl = reinterpret_cast<const uint4 *>(D.slots)[j];
                const uint32_t tok = uni(sl.y), d = uni(sl.z);
                j = uni(sl.w);
                uint32_t at, dummy;
                dyn_probe(D, cl, tok, lane, at, dummy);
                if (at == kNil) { fault |= SAM_STATUS_INTERNAL_BIT; break; }
                if (lane == 0)
                    reinterpret_cast<uint4 *>(D.slots)[at] = make_uint4(cl, tok, d, CL.head);
                CL.head = at;
                c.n_trans++;
                order_memory();
            }
            store_rec(&D.rec[cl], CL, lane);
            order_memory();
            // states further up the path that still lead to q now lead to the clone
            for (;;) {
                if (lane == 0) {
                    if (where == kInline) D.rec[p].idst = cl;
                    else D.slots[where].dst = cl;
                }
                order_memory();
                p = R.link;
                if (p == kNil) break;
                if (--guard == 0) { fault |= SAM_STATUS_INTERNAL_BIT; break; }
                uint32_t at, dst;
                const bool hit = rec_and_probe(D, p, t, lane, R, at, dst);
                if (R.itok == t) {
                    if (R.idst != q) break;
                    where = kInline;
                } else if (hit) {
                    if (dst != q) break;
                    where = at;
                } else {
                    break;
                }
            }
            if (lane == 0) D.rec[q].link = cl;
            linkc = cl; l2 = CL.len; e2 = CL.endpos;
        }
    }
    Rec C;
    C.len = k; C.link = linkc; C.endpos = k; C.head = kNil; C.itok = kNil; C.idst = 0;
    store_rec(&D.rec[cur], C, lane);
    if (lane == 0) D.text[c.n] = (int32_t)t;
    order_memory();
    c.n = k; c.last = cur; c.s2 = linkc; c.l2 = l2; c.e2 = e2;
}

}  // namespace

// One workgroup (2 waves) per sequence.  offsets != NULL: ingest mode, sequence
// b is fed tokens[offsets[b] : offsets[b+1]) and nothing is written to the
// draft outputs.  Otherwise step mode: sequence b is fed the first counts[b]
// tokens of tokens[b * max_accept ...], then source selection and draft gather.
__global__ __launch_bounds__(128) void sam_feed_kernel(StaticView S, BatchView B,
                                                        const int32_t *__restrict__ tokens,
                                                        const int64_t *__restrict__ offsets,
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
    const uint32_t n0 = uni(meta->n);

    // which tokens
    const int32_t *tok;
    int64_t count;
    uint32_t fault = 0;
    if (offsets) {
        const int64_t o0 = offsets[b], o1 = offsets[b + 1];
        tok = tokens + o0;
        count = o1 - o0;
    } else {
        tok = tokens + (int64_t)b * B.max_accept;
        count = counts[b];
        if (count < 0 || count > B.max_accept) { fault |= SAM_STATUS_COUNT_BIT; count = 0; }
    }
    count = (int64_t)uni((uint32_t)count);
    if ((int64_t)n0 + count > (int64_t)B.max_seq_len) { fault |= SAM_STATUS_CAPACITY_BIT; count = 0; }
    const uint32_t vocab = (uint32_t)B.vocab;

    if (wave == 0) {
        uint32_t s = uni(meta->s1), l = uni(meta->l1), e = uni(meta->e1);
        if (B.has_static) {
            bool stop = false;
            for (int64_t base = 0; base < count && !stop; base += 64) {
                const int m = (int)((count - base) < 64 ? (count - base) : 64);
                const uint32_t tv = lane < m ? (uint32_t)tok[base + lane] : 0u;
                for (int i = 0; i < m; i++) {
                    const uint32_t t = lane_get(tv, i);
                    if (t >= vocab) { stop = true; break; }
                    static_transfer(S, t, lane, s, l, e, fault);
                }
            }
        }
        if (lane == 0) { sh[0] = s; sh[1] = l; sh[2] = e; sh[6] = fault & SAM_STATUS_INTERNAL_BIT; }
    } else {
        DynSeq D;
        D.text = B.dyn_text + (size_t)b * B.max_seq_len;
        D.rec = B.dyn_rec + (size_t)b * B.max_states;
        D.slots = B.dyn_slots + (size_t)b * B.dyn_buckets * kBucketSlots;
        D.n_buckets = B.dyn_buckets;
        DynCursor c;
        c.n = n0; c.n_states = uni(meta->n_states); c.last = uni(meta->last);
        c.n_trans = uni(meta->n_trans);
        c.s2 = uni(meta->s2); c.l2 = uni(meta->l2); c.e2 = uni(meta->e2);
        bool stop = false;
        for (int64_t base = 0; base < count && !stop; base += 64) {
            const int m = (int)((count - base) < 64 ? (count - base) : 64);
            const uint32_t tv = lane < m ? (uint32_t)tok[base + lane] : 0u;
            for (int i = 0; i < m; i++) {
                const uint32_t t = lane_get(tv, i);
                if (t >= vocab) { stop = true; fault |= SAM_STATUS_TOKEN_BIT; break; }
                dyn_expand(D, t, lane, c, fault);
            }
        }
        if (lane == 0) {
            sh[3] = c.l2; sh[4] = c.e2; sh[5] = c.n;
            meta->s2 = c.s2; meta->l2 = c.l2; meta->e2 = c.e2;
            meta->n_states = c.n_states; meta->last = c.last; meta->n_trans = c.n_trans;
            if (fault) {
                meta->status |= fault;
                atomicOr(B.status, fault);
            }
        }
    }
    __syncthreads();
    // meta->n is read by both waves above, so it is written only after the barrier
    if (wave == 1) {
        if (lane == 0) meta->n = sh[5];
        return;
    }
    const uint32_t s1 = sh[0], l1 = sh[1], e1 = sh[2];
    const uint32_t l2 = sh[3], e2 = sh[4], n1 = sh[5];
    if (lane == 0) {
        meta->s1 = s1; meta->l1 = l1; meta->e1 = e1;
        if (sh[6]) atomicOr(B.status, sh[6]);
    }
    if (offsets) return;

    const bool use_static = B.has_static && ((int64_t)l1 > (int64_t)l2 + (int64_t)B.l_bias);
    const uint32_t ml = use_static ? l1 : l2;
    const uint32_t p = use_static ? e1 : e2;
    const int32_t *T = use_static ? S.text : B.dyn_text + (size_t)b * B.max_seq_len;
    const uint32_t Tn = use_static ? S.n_tokens : n1;
    const int L = B.draft_len;
    int dl = 0;
    if (ml > 0) {
        const uint32_t room = Tn - p;
        dl = room < (uint32_t)L ? (int)room : L;
    }
    for (int i = lane; i < L; i += 64)
        draft[(size_t)b * L + i] = i < dl ? T[p + i] : -1;
    if (lane == 0) {
        match_len[b] = (int32_t)ml;
        draft_len[b] = dl;
        source[b] = ml == 0 ? 0 : (use_static ? 2 : 1);
    }
}

// Fresh sequences: root record, empty cursors.  The slot tables are filled with
// the empty key by the caller.
__global__ void sam_reset_kernel(BatchView B)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B.batch) return;
    DynRec r;
    r.len = 0; r.link = kNil; r.endpos = 0; r.head = kNil; r.itok = kNil; r.idst = 0;
    r.pad0 = 0; r.pad1 = 0;
    B.dyn_rec[(size_t)b * B.max_states] = r;
    SeqMeta m = {};
    m.n_states = 1;
    B.meta[b] = m;
    if (b == 0) *B.status = 0;
}

__global__ void sam_debug_kernel(BatchView B, int32_t *s1, int32_t *l1, int32_t *s2, int32_t *l2,
                                 int32_t *text_len, int32_t *n_states, int32_t *n_trans)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B.batch) return;
    const SeqMeta m = B.meta[b];
    if (s1) s1[b] = (int32_t)m.s1;
    if (l1) l1[b] = (int32_t)m.l1;
    if (s2) s2[b] = (int32_t)m.s2;
    if (l2) l2[b] = (int32_t)m.l2;
    if (text_len) text_len[b] = (int32_t)m.n;
    if (n_states) n_states[b] = (int32_t)m.n_states;
    if (n_trans) n_trans[b] = (int32_t)m.n_trans;
}

// ---- launchers (called from the C ABI) ------------------------------------

hipError_t launch_feed(const StaticView &S, const BatchView &B, const int32_t *tokens,
                       const int64_t *offsets, const int32_t *counts, int32_t *match_len,
                       int32_t *draft, int32_t *draft_len, int32_t *source, hipStream_t stream)
{
    hipLaunchKernelGGL(sam_feed_kernel, dim3(B.batch), dim3(128), 0, stream, S, B, tokens,
                       offsets, counts, match_len, draft, draft_len, source);
    return hipGetLastError();
}

hipError_t launch_reset(const BatchView &B, hipStream_t stream)
{
    hipLaunchKernelGGL(sam_reset_kernel, dim3((B.batch + 127) / 128), dim3(128), 0, stream, B);
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
