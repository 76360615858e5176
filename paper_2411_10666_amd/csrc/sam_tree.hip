// gfx950 kernel for tree drafts from the static automaton (arxiv 2411.10666,
// Section 3.2 and Algorithm 4: best-first expansion over the top-k successors
// that Algorithm 3 computed on the host).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sam_device.h"

namespace sam {

namespace {

// Maximum of a value over the 64 lanes, the same in every lane.  Within a row of
// 16 lanes by four data-parallel-primitive moves (a butterfly would need the LDS
// crossbar, whose round trip is what a pop of the queue would then be spent on),
// across the four rows through the scalar unit.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
    uint32_t y;
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1, 0xF, 0xF, false);   // lanes i ^ 1
    x = x > y ? x : y;
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x4E, 0xF, 0xF, false);   // lanes i ^ 2
    x = x > y ? x : y;
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x141, 0xF, 0xF, false);  // 7 - i in each half row
    x = x > y ? x : y;
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x140, 0xF, 0xF, false);  // 15 - i in each row
    x = x > y ? x : y;
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0);
    const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
    const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

}  // namespace

// Tree draft by best-first expansion over the top-k successors (Algorithm 4),
// one wavefront per sequence.  The priority queue lives in LDS as an append-only
// array; an entry's key packs (probability bits, ~push index), so the maximum
// key is the largest probability and, among equals, the entry pushed first.  The
// k children of the popped state are fetched by k lanes in one request and appended
// in table order; while that request travels, the lanes scan the entries already
// queued and reduce them to their best (two 32-bit wave reductions), so that the next
// pop (that best, or the first of the new children) is known as soon as the children are.
// Probabilities are float products rounded once per edge.
__global__ __launch_bounds__(64) void sam_tree_kernel(StaticView S, BatchView B, int max_size,
                                                       int32_t *__restrict__ tokens,
                                                       int32_t *__restrict__ parents,
                                                       float *__restrict__ probs,
                                                       int32_t *__restrict__ sizes)
{
    constexpr int kQ = kMaxTreeSize * kMaxTopK + 1;
    __shared__ unsigned long long qkey[kQ];
    __shared__ uint32_t qstate[kQ];
    __shared__ int32_t qtok[kQ];
    __shared__ int32_t qpar[kQ];
    // the draft is collected here and written out once at the end: a store per pop would
    // sit in the same in-order queue as the pop's table read and be waited for with it
    __shared__ int32_t otok[kMaxTreeSize];
    __shared__ int32_t opar[kMaxTreeSize];
    __shared__ float   oprob[kMaxTreeSize];
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const SeqMeta m = B.meta[b];
    const int k = S.top_k;
    int dn = 0;
    if (m.n > 0) {
        if (lane == 0) {
            qkey[0] = ((unsigned long long)__float_as_uint(1.0f) << 32) | 0xFFFFFFFFull;
            qstate[0] = m.s1;
            qtok[0] = B.dyn_text[(size_t)b * B.max_seq_len + m.n - 1];
            qpar[0] = -1;
        }
        __syncthreads();
        int qn = 1;
        unsigned long long best = qkey[0];              // the next entry to pop (0: queue empty)
        while (dn < max_size && best != 0) {
            const uint32_t idx = 0xFFFFFFFFu - (uint32_t)best;
            const float p = __uint_as_float((uint32_t)(best >> 32));
            const uint32_t st = qstate[idx];
            // the children's table row is the one dependent memory read of a pop: request
            // it first, and look for the best of the entries already queued while it travels
            TopEnt e = {0, 0, 0.0f};
            if (lane < k) e = S.topk[(size_t)st * k + lane];
            if (lane == 0) {
                otok[dn] = qtok[idx];
                opar[dn] = qpar[idx];
                oprob[dn] = p;
            }
            unsigned long long mine = 0;
            for (int i = lane; i < qn; i += 256) {
                // four independent reads per round (clamped, then masked), one wait
                unsigned long long key[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int at = i + 64 * u;
                    key[u] = qkey[at < kQ ? at : kQ - 1];
                }
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int at = i + 64 * u;
                    if (at >= qn || (uint32_t)at == idx) key[u] = 0;
                    mine = key[u] > mine ? key[u] : mine;
                }
            }
            // the best of the entries already queued, still in the shadow of the request: the
            // largest 64-bit key is the largest upper half, then the largest lower half
            // among the lanes that hold that upper half
            const uint32_t hi = wave_max_u32((uint32_t)(mine >> 32));
            const uint32_t lo = wave_max_u32((uint32_t)(mine >> 32) == hi ? (uint32_t)mine : 0u);
            best = ((unsigned long long)hi << 32) | lo;
            // (the children are first looked at here, after the reductions: the empty
            // statement keeps the compiler from waiting for them in their middle)
            asm volatile("" : "+v"(e.dst) : "s"(hi), "s"(lo));
            const bool valid = e.dst != 0;
            const unsigned long long mask = __ballot(valid);
            unsigned long long mine_new = 0;
            if (valid) {
                const int pos = qn + __popcll(mask & ((1ull << lane) - 1ull));
                const float pn = __fmul_rn(p, e.prob);
                const unsigned long long key = ((unsigned long long)__float_as_uint(pn) << 32) |
                                               (unsigned long long)(0xFFFFFFFFu - (uint32_t)pos);
                qkey[pos] = key;
                qstate[pos] = e.dst;
                qtok[pos] = (int32_t)e.token;
                qpar[pos] = dn;
                mine_new = key;
            }
            if (lane == 0) qkey[idx] = 0;               // popped
            // A table row lists a state's successors by falling frequency, hence by falling
            // probability (the product with p rounds monotonically), and is filled from its
            // first entry on: the best of the new children is lane 0's, and among equal
            // products it is also the one pushed first.
            const unsigned long long first_new =
                ((unsigned long long)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(mine_new >> 32)) << 32) |
                (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)mine_new);
            best = first_new > best ? first_new : best;
            qn += __popcll(mask);
            dn++;
            __syncthreads();
        }
    }
    for (int i = lane; i < max_size; i += 64) {
        const bool have = i < dn;
        tokens[(size_t)b * max_size + i] = have ? otok[i] : -1;
        parents[(size_t)b * max_size + i] = have ? opar[i] : -1;
        probs[(size_t)b * max_size + i] = have ? oprob[i] : 0.0f;
    }
    if (lane == 0) sizes[b] = dn;
}

hipError_t launch_tree(const StaticView &S, const BatchView &B, int max_size, int32_t *tokens,
                       int32_t *parents, float *probs, int32_t *sizes, hipStream_t stream)
{
    hipLaunchKernelGGL(sam_tree_kernel, dim3(B.batch), dim3(64), 0, stream, S, B, max_size, tokens,
                       parents, probs, sizes);
    return hipGetLastError();
}

}  // namespace sam
