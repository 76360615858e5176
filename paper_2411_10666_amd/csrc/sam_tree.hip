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
// key is the largest probability and, among equals, the entry pushed first.  A
// pop is a strided scan plus two 32-bit wave reductions; the k children of the popped
// state are fetched by k lanes in one request and appended in table order.
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
        while (dn < max_size) {
            unsigned long long best = 0;
            for (int i = lane; i < qn; i += 64) {
                const unsigned long long key = qkey[i];
                best = key > best ? key : best;
            }
            // the largest 64-bit key: the largest upper half, then the largest lower
            // half among the lanes that hold that upper half
            const uint32_t hi = wave_max_u32((uint32_t)(best >> 32));
            const uint32_t lo = wave_max_u32((uint32_t)(best >> 32) == hi ? (uint32_t)best : 0u);
            best = ((unsigned long long)hi << 32) | lo;
            if (best == 0) break;                       // queue empty
            const uint32_t idx = 0xFFFFFFFFu - (uint32_t)best;
            const float p = __uint_as_float((uint32_t)(best >> 32));
            const uint32_t st = qstate[idx];
            if (lane == 0) {
                tokens[(size_t)b * max_size + dn] = qtok[idx];
                parents[(size_t)b * max_size + dn] = qpar[idx];
                probs[(size_t)b * max_size + dn] = p;
                qkey[idx] = 0;                          // popped
            }
            TopEnt e = {0, 0, 0.0f};
            if (lane < k) e = S.topk[(size_t)st * k + lane];
            const bool valid = e.dst != 0;
            const unsigned long long mask = __ballot(valid);
            if (valid) {
                const int pos = qn + __popcll(mask & ((1ull << lane) - 1ull));
                const float pn = __fmul_rn(p, e.prob);
                qkey[pos] = ((unsigned long long)__float_as_uint(pn) << 32) |
                            (unsigned long long)(0xFFFFFFFFu - (uint32_t)pos);
                qstate[pos] = e.dst;
                qtok[pos] = (int32_t)e.token;
                qpar[pos] = dn;
            }
            qn += __popcll(mask);
            dn++;
            __syncthreads();
        }
    }
    for (int i = dn + lane; i < max_size; i += 64) {
        tokens[(size_t)b * max_size + i] = -1;
        parents[(size_t)b * max_size + i] = -1;
        probs[(size_t)b * max_size + i] = 0.0f;
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
