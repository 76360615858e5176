// Measurement aids: what the memory system of the current device delivers for
// the access patterns of the draft-retrieval path (dependent loads of one
// 128-byte bucket per hop, independent random 16-byte slot reads, streaming
// copies) and what an empty launch costs.  None of this is on the path; the
// figures put the path's own throughput into proportion.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "../../include/sam.h"
#include "sam_membench.h"

namespace sam {
namespace {

constexpr uint32_t kLcgMul = 1664525u;      // = 1 (mod 4) and an odd increment:
constexpr uint32_t kLcgAdd = 1013904223u;   // full period on any power of two

// node i (128 bytes): word 0 = successor, the other words = filler
__global__ void chase_fill_kernel(uint32_t *nodes, uint32_t n_nodes)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t w = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; w < (uint64_t)n_nodes * 32;
         w += stride) {
        const uint32_t i = (uint32_t)(w >> 5);
        nodes[w] = (w & 31) ? i : ((i * kLcgMul + kLcgAdd) & (n_nodes - 1));
    }
}

// one wavefront: all lanes read the current node (one line), lane 0's word
// names the next one
__global__ void chase_kernel(const uint32_t *nodes, uint32_t start, int64_t hops, uint32_t *out)
{
    uint32_t p = start, acc = 0;
    for (int64_t i = 0; i < hops; ++i) {
        const uint32_t v = nodes[(size_t)p * 32 + (threadIdx.x & 31)];
        acc ^= v;
        p = __builtin_amdgcn_readfirstlane(v);
    }
    out[threadIdx.x] = acc ^ p;
}

// every lane: `per_lane` independent random 16-byte reads
__global__ void gather_kernel(const uint4 *table, uint64_t n_elems, int64_t per_lane, uint32_t *out)
{
    uint64_t x = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 0x9E3779B97F4A7C15ull + 1;
    uint32_t acc = 0;
    for (int64_t i = 0; i < per_lane; ++i) {
        x ^= x >> 12; x ^= x << 25; x ^= x >> 27;
        const uint64_t idx = __umul64hi(x * 0x2545F4914F6CDD1Dull, n_elems);
        const uint4 v = table[idx];
        acc += v.x + v.w;
    }
    if (acc == 0x12345678u) out[0] = acc;   // keeps the loads alive
}

__global__ void copy_kernel(const uint4 *src, uint4 *dst, uint64_t n)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = src[i];
}

__global__ void empty_kernel(uint32_t *) {}

struct Scope {                              // frees what a measurement allocated
    void *a = nullptr, *b = nullptr, *c = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Scope()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        if (a) (void)hipFree(a);
        if (b) (void)hipFree(b);
        if (c) (void)hipFree(c);
    }
};

bool ok(hipError_t e, const char *what, std::string &err)
{
    if (e == hipSuccess) return true;
    err = std::string("sam_membench: ") + what + ": " + hipGetErrorString(e);
    return false;
}

#define MB_TRY(call, what) do { if (!ok((call), what, err)) return SAM_EDEVICE; } while (0)

int elapsed(Scope &s, double *ms, std::string &err)
{
    MB_TRY(hipEventSynchronize(s.e1), "hipEventSynchronize");
    float f = 0.f;
    MB_TRY(hipEventElapsedTime(&f, s.e0, s.e1), "hipEventElapsedTime");
    *ms = f;
    return SAM_OK;
}

}  // namespace

int membench(int32_t kind, int64_t size, int64_t count, int32_t workgroups, double *result,
             std::string &err)
{
    Scope s;
    MB_TRY(hipEventCreate(&s.e0), "hipEventCreate");
    MB_TRY(hipEventCreate(&s.e1), "hipEventCreate");
    MB_TRY(hipMalloc(&s.c, 4096), "hipMalloc");
    uint32_t *out = (uint32_t *)s.c;
    double ms = 0.0;
    int rc;

    switch (kind) {
    case SAM_MEMBENCH_CHASE: {
        if (size < 4096 || size > ((int64_t)1 << 36) || (size & (size - 1)) || count < 1)
            { err = "sam_membench: chase needs a power-of-two footprint of 4 KiB .. 64 GiB and count >= 1"; return SAM_EINVAL; }
        const uint32_t n_nodes = (uint32_t)(size / 128);
        MB_TRY(hipMalloc(&s.a, (size_t)size), "hipMalloc");
        chase_fill_kernel<<<2048, 256>>>((uint32_t *)s.a, n_nodes);
        MB_TRY(hipGetLastError(), "launch");
        if (n_nodes <= (1u << 20)) {        // one whole cycle: what fits a cache is in it
            chase_kernel<<<1, 64>>>((const uint32_t *)s.a, 0u, (int64_t)n_nodes, out);
            MB_TRY(hipGetLastError(), "launch");
        }
        MB_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
        MB_TRY(hipEventRecord(s.e0, 0), "hipEventRecord");
        chase_kernel<<<1, 64>>>((const uint32_t *)s.a, 1u & (n_nodes - 1), count, out);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipEventRecord(s.e1, 0), "hipEventRecord");
        if ((rc = elapsed(s, &ms, err)) != SAM_OK) return rc;
        *result = ms * 1e6 / (double)count;             // ns per hop
        return SAM_OK;
    }
    case SAM_MEMBENCH_GATHER: {
        if (size < 4096 || size > ((int64_t)1 << 36) || count < 1 || workgroups < 1 ||
            workgroups > (1 << 20))
            { err = "sam_membench: gather needs 4 KiB .. 64 GiB, count >= 1, 1 .. 2^20 workgroups"; return SAM_EINVAL; }
        const uint64_t n_elems = (uint64_t)size / 16;
        MB_TRY(hipMalloc(&s.a, n_elems * 16), "hipMalloc");
        MB_TRY(hipMemset(s.a, 1, n_elems * 16), "hipMemset");
        gather_kernel<<<workgroups, 256>>>((const uint4 *)s.a, n_elems, 4, out);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
        MB_TRY(hipEventRecord(s.e0, 0), "hipEventRecord");
        gather_kernel<<<workgroups, 256>>>((const uint4 *)s.a, n_elems, count, out);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipEventRecord(s.e1, 0), "hipEventRecord");
        if ((rc = elapsed(s, &ms, err)) != SAM_OK) return rc;
        *result = (double)workgroups * 256.0 * (double)count / (ms * 1e-3);   // reads per second
        return SAM_OK;
    }
    case SAM_MEMBENCH_COPY: {
        if (size < 4096 || size > ((int64_t)1 << 35))
            { err = "sam_membench: copy needs 4 KiB .. 32 GiB"; return SAM_EINVAL; }
        const uint64_t n = (uint64_t)size / 16;
        MB_TRY(hipMalloc(&s.a, n * 16), "hipMalloc");
        MB_TRY(hipMalloc(&s.b, n * 16), "hipMalloc");
        MB_TRY(hipMemset(s.a, 1, n * 16), "hipMemset");
        copy_kernel<<<8192, 256>>>((const uint4 *)s.a, (uint4 *)s.b, n);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
        MB_TRY(hipEventRecord(s.e0, 0), "hipEventRecord");
        copy_kernel<<<8192, 256>>>((const uint4 *)s.a, (uint4 *)s.b, n);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipEventRecord(s.e1, 0), "hipEventRecord");
        if ((rc = elapsed(s, &ms, err)) != SAM_OK) return rc;
        *result = 2.0 * (double)(n * 16) / (ms * 1e-3);                       // bytes per second
        return SAM_OK;
    }
    case SAM_MEMBENCH_LAUNCH: {
        if (count < 1 || count > 1000000 || workgroups < 1 || workgroups > 65536)
            { err = "sam_membench: launch needs 1 .. 10^6 launches of 1 .. 65536 workgroups"; return SAM_EINVAL; }
        for (int i = 0; i < 64; ++i) empty_kernel<<<workgroups, 128>>>(out);
        MB_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
        MB_TRY(hipEventRecord(s.e0, 0), "hipEventRecord");
        for (int64_t i = 0; i < count; ++i) empty_kernel<<<workgroups, 128>>>(out);
        MB_TRY(hipGetLastError(), "launch");
        MB_TRY(hipEventRecord(s.e1, 0), "hipEventRecord");
        if ((rc = elapsed(s, &ms, err)) != SAM_OK) return rc;
        *result = ms * 1e3 / (double)count;                                   // microseconds per launch
        return SAM_OK;
    }
    default:
        err = "sam_membench: unknown kind";
        return SAM_EINVAL;
    }
}

}  // namespace sam
