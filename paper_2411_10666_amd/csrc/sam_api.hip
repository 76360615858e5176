// C ABI of the library (see include/sam.h): argument checks, device memory and
// kernel launches.  All arithmetic of the method runs in the kernels
// (sam_kernels.hip) and, for the corpus automaton, in the host builder
// (sam_host.cpp).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/sam.h"
#include "sam_device.h"
#include "sam_host.h"
#include "sam_membench.h"

using namespace sam;

namespace {

thread_local std::string g_err;
int g_layout_override = 0;   // bit 0: always the wide layout, bit 1: tight slot tables,
                             // bit 2: C++ token loops, bit 3: corpus table beyond 4 GiB,
                             // bit 4: scout waves whatever the batch size, bit 5: never
// Scout waves pay once the tables a step touches no longer stay in the caches from one
// launch to the next: the per-sequence tables when many sequences share the caches, the
// corpus automaton when it is larger than the last-level cache (256 MB).  Measured:
// 8 sequences over 12 MB of corpus tables +4.5 % per step with scouts, 64 over 1.2 GB
// -2 %, 256 over 12 GB -15 %.  They stop paying once the walking waves alone fill the
// chip: with more than six sequences per compute unit the scouts take wave slots and
// issue cycles from other sequences' walks (1024 sequences on 256 units over 6 GB of
// tables -9 % per step with scouts, 1536 -6 %, 2048 +9 %, 4096 +19 %, 8192 +27 %).
constexpr int     kScoutMinBatch = 128;
constexpr int     kScoutMaxSeqPerCu = 6;
constexpr int64_t kScoutMinCorpusBytes = 256ll << 20;
// buckets of 128 bytes that make a transition table of 4.5 GiB
constexpr uint64_t kHugeTableBuckets = (1ull << 25) + (1ull << 22);
HostSam::ProgressFn g_progress = nullptr;
void *g_progress_user = nullptr;

int fail(int code, const std::string &msg)
{
    g_err = msg;
    return code;
}

int fail_hip(const char *what, hipError_t e)
{
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? SAM_ENOMEM : SAM_EDEVICE;
}

#define HIP_TRY(expr)                                      \
    do {                                                   \
        hipError_t e_ = (expr);                            \
        if (e_ != hipSuccess) return fail_hip(#expr, e_);  \
    } while (0)

}  // namespace

// Table space of the batch made by sam_batch_init_noalloc: device memory that is
// part of the loaded code object, so no call ever has to allocate it.  Every GPU
// the library runs on holds its own copy at its own address for the life of the
// process.  In host code the name below is only a handle for hipGetSymbolAddress;
// the address kernels and fills receive is the one that call returns.
constexpr size_t kNoAllocBytes = (size_t)SAM_NOALLOC_MAX_BYTES;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoAllocBytes];

struct sam_corpus {
    HostSam    host;
    bool       on_device = false;
    int        device = -1;
    StaticView view = {};
    void      *d_text = nullptr, *d_linkrec = nullptr, *d_root = nullptr, *d_slots = nullptr;
    void      *d_topk = nullptr;
    int64_t    device_bytes = 0;
};

struct sam_batch {
    const sam_corpus *corpus = nullptr;
    BatchView         view = {};
    int64_t           device_bytes = 0;
    int               noalloc_device = -1;   // >= 0: lives in that device's fixed buffer
};

namespace {

// one fixed-buffer batch per device: its handle, the buffer's device address
// (looked up once per device) and whether the handle is handed out
constexpr int kMaxDevices = 64;
struct NoAllocSlot {
    sam_batch      handle;
    unsigned char *base = nullptr;
    bool           busy = false;
};
NoAllocSlot g_noalloc[kMaxDevices];
std::mutex  g_noalloc_mu;

}  // namespace

// Address of the current device's copy of the fixed buffer, looked up once per
// device with that device current (the first lookup makes the runtime load this
// file's device code on that GPU, which is when the buffer comes to exist there).
// Call with g_noalloc_mu held.
static hipError_t noalloc_base_locked(int dev, unsigned char **base)
{
    NoAllocSlot &slot = g_noalloc[dev];
    if (!slot.base) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        slot.base = (unsigned char *)p;
    }
    *base = slot.base;
    return hipSuccess;
}

extern "C" {

const char *sam_last_error(void) { return g_err.c_str(); }

#ifndef SAM_BUILD_ID
#define SAM_BUILD_ID "unknown"
#endif
const char *sam_build_id(void) { return SAM_BUILD_ID; }

static void corpus_release_device(sam_corpus *c)
{
    if (c->d_text) (void)hipFree(c->d_text);
    if (c->d_linkrec) (void)hipFree(c->d_linkrec);
    if (c->d_root) (void)hipFree(c->d_root);
    if (c->d_slots) (void)hipFree(c->d_slots);
    if (c->d_topk) (void)hipFree(c->d_topk);
    c->d_text = c->d_linkrec = c->d_root = c->d_slots = c->d_topk = nullptr;
}

static int corpus_upload(sam_corpus *c)
{
    const HostSam &h = c->host;
    std::vector<LinkPair> lr;
    try {
        h.make_linkrec(lr);
    } catch (const std::bad_alloc &) {
        return fail(SAM_ENOMEM, "sam_build: out of host memory for the link records");
    }
    const size_t b_text = (size_t)h.n_tokens * sizeof(int32_t);
    const size_t b_lr = (size_t)h.n_states * sizeof(LinkRec);
    const size_t b_root = (size_t)h.vocab * sizeof(RootEnt);
    const size_t b_slots = (size_t)h.n_buckets * kBucketSlots * sizeof(Slot);
    size_t b_slots_dev = b_slots;      // what stays on the device in the end
    HIP_TRY(hipGetDevice(&c->device));
    HIP_TRY(hipMalloc(&c->d_text, b_text));
    HIP_TRY(hipMalloc(&c->d_linkrec, b_lr));
    HIP_TRY(hipMalloc(&c->d_root, b_root));
    HIP_TRY(hipMalloc(&c->d_slots, b_slots));
    HIP_TRY(hipMemcpy(c->d_text, h.text.data(), b_text, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->d_root, h.root.data(), b_root, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->d_slots, h.slots, b_slots, hipMemcpyHostToDevice));
    {
        // link pairs -> 32-byte state records with two transitions inline
        void *d_pairs = nullptr, *d_wide = nullptr;
        const size_t b_pairs = (size_t)h.n_states * sizeof(LinkPair);
        const size_t b_wide = ((size_t)h.n_states + 31) / 32 * sizeof(uint32_t);
        HIP_TRY(hipMalloc(&d_pairs, b_pairs));
        hipError_t e = hipMalloc(&d_wide, b_wide);
        if (e == hipSuccess) e = hipMemset(d_wide, 0, b_wide);
        if (e == hipSuccess) e = hipMemcpy(d_pairs, lr.data(), b_pairs, hipMemcpyHostToDevice);
        if (e == hipSuccess)
            e = launch_staterec((const LinkPair *)d_pairs, (Slot *)c->d_slots, (RootEnt *)c->d_root,
                                (LinkRec *)c->d_linkrec, (uint32_t *)d_wide, h.n_states,
                                h.n_buckets * kBucketSlots, (uint32_t)h.vocab, nullptr);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        (void)hipFree(d_pairs);
        // The walks only ever look up transitions of wide states (a narrow state's record
        // holds all of its own): the table they probe is rebuilt with those alone, at load
        // 0.5, and the full one freed.  (Not in the testing mode that wants a table beyond
        // 4 GiB.)
        uint64_t n_buckets = h.n_buckets;
        if (e == hipSuccess && (g_layout_override & 8) == 0) {
            unsigned long long *d_count = nullptr, n_wide = 0;
            void *d_new = nullptr;
            e = hipMalloc((void **)&d_count, sizeof(*d_count));
            if (e == hipSuccess) e = hipMemset(d_count, 0, sizeof(*d_count));
            if (e == hipSuccess)
                e = launch_count_wide((const Slot *)c->d_slots, (const uint32_t *)d_wide,
                                      h.n_buckets * kBucketSlots, d_count, nullptr);
            if (e == hipSuccess) e = hipMemcpy(&n_wide, d_count, sizeof(n_wide), hipMemcpyDeviceToHost);
            if (d_count) (void)hipFree(d_count);
            const uint64_t nb_new = (2 * (uint64_t)n_wide + 64 + kBucketSlots - 1) / kBucketSlots;
            if (e == hipSuccess && nb_new < h.n_buckets) {
                const size_t b_new = (size_t)nb_new * kBucketSlots * sizeof(Slot);
                if (hipMalloc(&d_new, b_new) != hipSuccess) {
                    // no room for a second table beside the full one: the full one serves
                    (void)hipGetLastError();
                    d_new = nullptr;
                } else {
                    e = launch_fill_empty(d_new, b_new, nullptr);
                    if (e == hipSuccess)
                        e = launch_compact_slots((const Slot *)c->d_slots, (const uint32_t *)d_wide,
                                                 h.n_buckets * kBucketSlots, (Slot *)d_new, nb_new,
                                                 nullptr);
                    if (e == hipSuccess) e = hipDeviceSynchronize();
                    if (e == hipSuccess) {
                        (void)hipFree(c->d_slots);
                        c->d_slots = d_new;
                        n_buckets = nb_new;
                    } else {
                        (void)hipFree(d_new);
                    }
                }
            }
        }
        if (d_wide) (void)hipFree(d_wide);
        if (e != hipSuccess) return fail_hip("sam_build: state records", e);
        b_slots_dev = (size_t)n_buckets * kBucketSlots * sizeof(Slot);
        c->view.n_buckets = n_buckets;
    }
    c->view.text = (const int32_t *)c->d_text;
    c->view.linkrec = (const LinkRec *)c->d_linkrec;
    c->view.root = (const RootEnt *)c->d_root;
    c->view.slots = (const Slot *)c->d_slots;
    c->view.n_tokens = (uint32_t)h.n_tokens;
    c->view.n_states = h.n_states;
    c->device_bytes = (int64_t)(b_text + b_lr + b_root + b_slots_dev);
    c->on_device = true;
    if (c->device >= 0 && c->device < kMaxDevices) {
        // a set-up call: do the one-time lookup of the fixed buffer here, so that a later
        // sam_batch_init_noalloc on this device has nothing left to load
        std::lock_guard<std::mutex> lock(g_noalloc_mu);
        unsigned char *unused = nullptr;
        (void)noalloc_base_locked(c->device, &unused);
    }
    return SAM_OK;
}

static int build_common(const int32_t *tokens, int64_t n, int32_t vocab, bool upload,
                        sam_corpus **out)
{
    if (!out) return fail(SAM_EINVAL, "sam_build: out is NULL");
    *out = nullptr;
    sam_corpus *c = new (std::nothrow) sam_corpus;
    if (!c) return fail(SAM_ENOMEM, "sam_build: out of host memory");
    std::string err;
    int rc;
    try {
        rc = c->host.build(tokens, n, vocab, err, g_progress, g_progress_user,
                           (g_layout_override & 8) ? kHugeTableBuckets : 0);
    } catch (const std::bad_alloc &) {
        rc = SAM_ENOMEM;
        err = "sam_build: out of host memory";
    }
    if (rc != SAM_OK) {
        delete c;
        return fail(rc, err);
    }
    if (upload) {
        if (g_progress) g_progress("upload", 0, 1, g_progress_user);
        rc = corpus_upload(c);
        if (rc != SAM_OK) {
            corpus_release_device(c);
            delete c;
            return rc;
        }
    }
    *out = c;
    return SAM_OK;
}

int sam_build(const int32_t *corpus_tokens, int64_t n_tokens, int32_t vocab, sam_corpus **out)
{
    return build_common(corpus_tokens, n_tokens, vocab, true, out);
}

int sam_build_host_only(const int32_t *corpus_tokens, int64_t n_tokens, int32_t vocab,
                        sam_corpus **out)
{
    return build_common(corpus_tokens, n_tokens, vocab, false, out);
}

int sam_corpus_save(const sam_corpus *c, const char *path)
{
    if (!c || !path) return fail(SAM_EINVAL, "sam_corpus_save: NULL argument");
    std::string err;
    const int rc = c->host.save(path, err);
    return rc == SAM_OK ? SAM_OK : fail(rc, err);
}

static int load_common(const char *path, bool upload, sam_corpus **out)
{
    if (!out || !path) return fail(SAM_EINVAL, "sam_corpus_load: NULL argument");
    *out = nullptr;
    sam_corpus *c = new (std::nothrow) sam_corpus;
    if (!c) return fail(SAM_ENOMEM, "sam_corpus_load: out of host memory");
    std::string err;
    int rc;
    try {
        rc = c->host.load(path, err);
    } catch (const std::bad_alloc &) {
        rc = SAM_ENOMEM;
        err = "sam_corpus_load: out of host memory";
    }
    if (rc != SAM_OK) {
        delete c;
        return fail(rc, err);
    }
    if (upload) {
        rc = corpus_upload(c);
        if (rc != SAM_OK) {
            corpus_release_device(c);
            delete c;
            return rc;
        }
    }
    *out = c;
    return SAM_OK;
}

int sam_corpus_load(const char *path, sam_corpus **out) { return load_common(path, true, out); }

int sam_corpus_load_host_only(const char *path, sam_corpus **out)
{
    return load_common(path, false, out);
}

int sam_corpus_info(const sam_corpus *c, int64_t *n_states, int64_t *n_trans,
                    int64_t *device_bytes)
{
    if (!c) return fail(SAM_EINVAL, "sam_corpus_info: corpus is NULL");
    if (n_states) *n_states = c->host.n_states;
    if (n_trans) *n_trans = (int64_t)c->host.n_trans;
    if (device_bytes) *device_bytes = c->device_bytes;
    return SAM_OK;
}

int sam_corpus_export(const sam_corpus *c, int32_t *length, int32_t *link, int32_t *min_endpos)
{
    if (!c) return fail(SAM_EINVAL, "sam_corpus_export: corpus is NULL");
    const HostSam &h = c->host;
    for (uint32_t s = 0; s < h.n_states; s++) {
        if (length) length[s] = (int32_t)h.len[s];
        if (link) link[s] = h.link[s] == kNil ? -1 : (int32_t)h.link[s];
        if (min_endpos) min_endpos[s] = (int32_t)h.endpos[s];
    }
    return SAM_OK;
}

int sam_corpus_find(const sam_corpus *c, int64_t state, int32_t token, int64_t *target)
{
    if (!c || !target) return fail(SAM_EINVAL, "sam_corpus_find: NULL argument");
    if (state < 0 || state >= (int64_t)c->host.n_states || token < 0 || token >= c->host.vocab)
        return fail(SAM_EINVAL, "sam_corpus_find: state or token out of range");
    const uint32_t d = c->host.find((uint32_t)state, (uint32_t)token);
    *target = d == kNil ? -1 : (int64_t)d;
    return SAM_OK;
}

int sam_corpus_build_topk(sam_corpus *c, int32_t k)
{
    if (!c) return fail(SAM_EINVAL, "sam_corpus_build_topk: corpus is NULL");
    std::string err;
    int rc;
    try {
        rc = c->host.build_topk(k, err, g_progress, g_progress_user);
    } catch (const std::bad_alloc &) {
        rc = SAM_ENOMEM;
        err = "sam_corpus_build_topk: out of host memory";
    }
    if (rc != SAM_OK) return fail(rc, err);
    if (c->on_device) {
        int dev = -1;
        HIP_TRY(hipGetDevice(&dev));
        if (dev != c->device)
            return fail(SAM_EINVAL, "sam_corpus_build_topk: the corpus lives on another device");
        const size_t bytes = c->host.topk.size() * sizeof(TopEnt);
        HIP_TRY(hipDeviceSynchronize());     // no launch may still read the old table
        if (c->d_topk) {
            c->device_bytes -= (int64_t)((size_t)c->host.n_states * c->view.top_k * sizeof(TopEnt));
            (void)hipFree(c->d_topk);
            c->d_topk = nullptr;
            c->view.topk = nullptr;
            c->view.top_k = 0;
        }
        HIP_TRY(hipMalloc(&c->d_topk, bytes));
        HIP_TRY(hipMemcpy(c->d_topk, c->host.topk.data(), bytes, hipMemcpyHostToDevice));
        c->view.topk = (const TopEnt *)c->d_topk;
        c->view.top_k = k;
        c->device_bytes += (int64_t)bytes;
    }
    return SAM_OK;
}

int sam_corpus_export_topk(const sam_corpus *c, uint64_t *freq, int32_t *token, int32_t *target,
                           float *prob)
{
    if (!c) return fail(SAM_EINVAL, "sam_corpus_export_topk: corpus is NULL");
    const HostSam &h = c->host;
    if (h.top_k < 1) return fail(SAM_EINVAL, "sam_corpus_export_topk: no top-k table was built");
    const size_t n = (size_t)h.n_states * h.top_k;
    if (freq)
        for (uint32_t s = 0; s < h.n_states; s++) freq[s] = h.freq[s];
    for (size_t i = 0; i < n; i++) {
        const TopEnt &e = h.topk[i];
        if (token) token[i] = e.dst ? (int32_t)e.token : -1;
        if (target) target[i] = e.dst ? (int32_t)e.dst : -1;
        if (prob) prob[i] = e.prob;
    }
    return SAM_OK;
}

void sam_corpus_free(sam_corpus *c)
{
    if (!c) return;
    corpus_release_device(c);
    delete c;
}

static void batch_release(sam_batch *b)
{
    if (b->noalloc_device >= 0) {
        // nothing to free: the tables are the device's fixed buffer
        std::lock_guard<std::mutex> lock(g_noalloc_mu);
        g_noalloc[b->noalloc_device].busy = false;
        return;
    }
    if (b->view.dyn_text) (void)hipFree(b->view.dyn_text);
    if (b->view.dyn_rec) (void)hipFree(b->view.dyn_rec);
    if (b->view.dyn_slots) (void)hipFree(b->view.dyn_slots);
    if (b->view.meta) (void)hipFree(b->view.meta);
    if (b->view.status) (void)hipFree(b->view.status);
    delete b;
}

// Argument checks shared by the two init calls; resolves the vocabulary.
static int batch_check_args(const char *fn, const sam_corpus *corpus, const int32_t *prompt_tokens,
                            const int64_t *prompt_offsets, int32_t batch, int32_t &vocab,
                            int32_t max_seq_len, int32_t max_accept, int32_t draft_len)
{
    const std::string f(fn);
    if (!prompt_tokens || !prompt_offsets)
        return fail(SAM_EINVAL, f + ": prompt_tokens / prompt_offsets is NULL");
    if (batch < 1) return fail(SAM_EINVAL, f + ": batch must be >= 1");
    if (max_seq_len < 1 || max_seq_len > (1 << 28))
        return fail(SAM_EINVAL, f + ": max_seq_len must be in 1 .. 2^28");
    if (max_accept < 1 || max_accept > 4096)
        return fail(SAM_EINVAL, f + ": max_accept must be in 1 .. 4096");
    if (draft_len < 1 || draft_len > 1024)
        return fail(SAM_EINVAL, f + ": draft_len must be in 1 .. 1024");
    if (corpus && !corpus->on_device)
        return fail(SAM_EINVAL, f + ": corpus was built host-only");
    if (corpus) {
        int dev = -1;
        HIP_TRY(hipGetDevice(&dev));
        if (dev != corpus->device)
            return fail(SAM_EINVAL, f + ": the corpus lives on device " +
                                        std::to_string(corpus->device) + ", the current device is " +
                                        std::to_string(dev));
        vocab = corpus->host.vocab;
    }
    if (vocab < 1) return fail(SAM_EINVAL, f + ": vocab must be >= 1");
    return SAM_OK;
}

static int batch_check_offsets(const char *fn, const int64_t *offs, int32_t batch,
                               int32_t max_seq_len)
{
    const std::string f(fn);
    if (offs[0] < 0) return fail(SAM_EINVAL, f + ": prompt_offsets[0] < 0");
    for (int32_t b = 0; b < batch; b++) {
        const int64_t len = offs[b + 1] - offs[b];
        if (len < 0) return fail(SAM_EINVAL, f + ": prompt_offsets must not decrease");
        if (len > max_seq_len)
            return fail(SAM_ECAPACITY, f + ": prompt " + std::to_string(b) + " has " +
                                           std::to_string(len) + " tokens, max_seq_len is " +
                                           std::to_string(max_seq_len));
    }
    return SAM_OK;
}

// Sizes of the per-sequence tables for these parameters.
struct BatchBytes { size_t text, rec, slots, meta; };

static BatchBytes batch_configure(BatchView &v, const sam_corpus *corpus, int32_t batch,
                                  int32_t vocab, int32_t max_seq_len, int32_t max_accept,
                                  int32_t draft_len, int32_t l_bias)
{
    const bool has_static = corpus != nullptr;
    v.batch = batch;
    v.vocab = vocab;
    v.max_seq_len = (uint32_t)max_seq_len;
    v.max_states = 2u * (uint32_t)max_seq_len + 2u;
    v.compact = ((g_layout_override & 1) == 0 && max_seq_len <= kCompactMaxSeqLen &&
                 vocab <= kCompactMaxVocab) ? 1 : 0;
    // a sequence never holds more than max_seq_len - 1 transitions in its slots
    const uint64_t dyn_slots = (g_layout_override & 2)
                                   ? ((uint64_t)max_seq_len + 16 + 15) / 16 * 16
                                   : dynamic_slots_for(max_seq_len);
    const size_t slot_bytes = v.compact ? sizeof(SlotCompact) : sizeof(Slot);
    const size_t rec_bytes = v.compact ? sizeof(DynRecCompact) : sizeof(DynRec);
    v.dyn_buckets = (uint32_t)(dyn_slots * slot_bytes / 128);
    v.max_accept = max_accept;
    v.draft_len = draft_len;
    v.l_bias = l_bias;
    v.l_threshold = -1;
    v.no_asm = (g_layout_override & 4) ? 1 : 0;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        n_cu = 0;                          // unknown: no upper limit
    const bool scouts_fit = n_cu <= 0 || (int64_t)batch <= (int64_t)n_cu * kScoutMaxSeqPerCu;
    v.scout = ((g_layout_override & 32) == 0 &&
               ((g_layout_override & 16) ||
                (scouts_fit && (batch >= kScoutMinBatch ||
                                (corpus && corpus->device_bytes > kScoutMinCorpusBytes))))) ? 1 : 0;
    v.has_static = has_static ? 1 : 0;
    BatchBytes b;
    b.text = (size_t)batch * max_seq_len * sizeof(int32_t);
    b.rec = (size_t)batch * v.max_states * rec_bytes;
    b.slots = (size_t)batch * v.dyn_buckets * 128;
    b.meta = (size_t)batch * sizeof(SeqMeta);
    return b;
}

int sam_batch_init(const sam_corpus *corpus, const int32_t *prompt_tokens,
                   const int64_t *prompt_offsets, int32_t batch, int32_t vocab,
                   int32_t max_seq_len, int32_t max_accept, int32_t draft_len, int32_t l_bias,
                   void *hip_stream, sam_batch **out)
{
    if (!out) return fail(SAM_EINVAL, "sam_batch_init: out is NULL");
    *out = nullptr;
    int rc = batch_check_args("sam_batch_init", corpus, prompt_tokens, prompt_offsets, batch,
                              vocab, max_seq_len, max_accept, draft_len);
    if (rc != SAM_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;

    // the offsets decide how far each wave reads: check them before any launch
    std::vector<int64_t> offs;
    try {
        offs.resize((size_t)batch + 1);
    } catch (const std::bad_alloc &) {
        return fail(SAM_ENOMEM, "sam_batch_init: out of host memory");
    }
    HIP_TRY(hipMemcpyAsync(offs.data(), prompt_offsets, offs.size() * sizeof(int64_t),
                           hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    rc = batch_check_offsets("sam_batch_init", offs.data(), batch, max_seq_len);
    if (rc != SAM_OK) return rc;

    sam_batch *bt = new (std::nothrow) sam_batch;
    if (!bt) return fail(SAM_ENOMEM, "sam_batch_init: out of host memory");
    bt->corpus = corpus;
    BatchView &v = bt->view;
    const BatchBytes bb = batch_configure(v, corpus, batch, vocab, max_seq_len, max_accept,
                                          draft_len, l_bias);
    hipError_t e;
    if ((e = hipMalloc((void **)&v.dyn_text, bb.text)) != hipSuccess ||
        (e = hipMalloc((void **)&v.dyn_rec, bb.rec)) != hipSuccess ||
        (e = hipMalloc((void **)&v.dyn_slots, bb.slots)) != hipSuccess ||
        (e = hipMalloc((void **)&v.meta, bb.meta)) != hipSuccess ||
        (e = hipMalloc((void **)&v.status, 256)) != hipSuccess) {
        batch_release(bt);
        return fail_hip("sam_batch_init: hipMalloc", e);
    }
    bt->device_bytes = (int64_t)(bb.text + bb.rec + bb.slots + bb.meta + 256);
    StaticView S = corpus ? corpus->view : StaticView{};
    if ((e = hipMemsetAsync(v.dyn_slots, 0xFF, bb.slots, stream)) != hipSuccess ||
        (e = launch_reset(v, nullptr, batch, stream)) != hipSuccess ||
        (e = launch_feed(S, v, nullptr, batch, prompt_tokens, prompt_offsets, nullptr, nullptr,
                         nullptr, nullptr, nullptr, stream)) != hipSuccess ||
        (e = hipStreamSynchronize(stream)) != hipSuccess) {
        batch_release(bt);
        return fail_hip("sam_batch_init: prompt ingest", e);
    }
    uint32_t st = 0;
    if ((e = hipMemcpy(&st, v.status, sizeof(st), hipMemcpyDeviceToHost)) != hipSuccess) {
        batch_release(bt);
        return fail_hip("sam_batch_init: status read", e);
    }
    if (st & SAM_STATUS_TOKEN) {
        batch_release(bt);
        return fail(SAM_ETOKEN, "sam_batch_init: a prompt token is outside [0, vocab)");
    }
    *out = bt;
    return SAM_OK;
}

int sam_batch_init_noalloc(const sam_corpus *corpus, const int32_t *prompt_tokens,
                           const int64_t *prompt_offsets, const int64_t *prompt_offsets_host,
                           int32_t batch, int32_t vocab, int32_t max_seq_len, int32_t max_accept,
                           int32_t draft_len, int32_t l_bias, void *hip_stream, sam_batch **out)
{
    static const char *fn = "sam_batch_init_noalloc";
    if (!out) return fail(SAM_EINVAL, "sam_batch_init_noalloc: out is NULL");
    *out = nullptr;
    if (!prompt_offsets_host)
        return fail(SAM_EINVAL, "sam_batch_init_noalloc: prompt_offsets_host is NULL");
    int rc = batch_check_args(fn, corpus, prompt_tokens, prompt_offsets, batch, vocab, max_seq_len,
                              max_accept, draft_len);
    if (rc != SAM_OK) return rc;
    rc = batch_check_offsets(fn, prompt_offsets_host, batch, max_seq_len);
    if (rc != SAM_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(SAM_EINVAL, "sam_batch_init_noalloc: device index beyond " +
                                    std::to_string(kMaxDevices - 1));

    BatchView v = {};
    const BatchBytes bb = batch_configure(v, corpus, batch, vocab, max_seq_len, max_accept,
                                          draft_len, l_bias);
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const size_t o_text = 0, o_rec = o_text + up(bb.text), o_slots = o_rec + up(bb.rec),
                 o_meta = o_slots + up(bb.slots), o_status = o_meta + up(bb.meta),
                 need = o_status + 256;
    if (need > kNoAllocBytes)
        return fail(SAM_EINVAL, "sam_batch_init_noalloc: these sizes need " + std::to_string(need) +
                                    " bytes of table space, the fixed buffer holds " +
                                    std::to_string(kNoAllocBytes) +
                                    " (use sam_batch_init for larger batches)");

    NoAllocSlot &slot = g_noalloc[dev];
    unsigned char *base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_noalloc_mu);
        if (slot.busy)
            return fail(SAM_EINVAL, "sam_batch_init_noalloc: the fixed buffer of this device is in "
                                    "use by a batch that has not been freed");
        hipError_t e = noalloc_base_locked(dev, &base);
        if (e != hipSuccess) return fail_hip("sam_batch_init_noalloc: address of the fixed buffer", e);
        slot.busy = true;
    }
    v.dyn_text = (int32_t *)(base + o_text);
    v.dyn_rec = base + o_rec;
    v.dyn_slots = base + o_slots;
    v.meta = (SeqMeta *)(base + o_meta);
    v.status = (uint32_t *)(base + o_status);
    sam_batch *bt = &slot.handle;
    bt->corpus = corpus;
    bt->view = v;
    bt->device_bytes = (int64_t)need;
    bt->noalloc_device = dev;
    // the buffer keeps what the last batch left: empty the slot tables, then fresh
    // records, cursors and status word (the reset kernel), then the prompts
    StaticView S = corpus ? corpus->view : StaticView{};
    hipError_t e;
    if ((e = launch_fill_empty(v.dyn_slots, bb.slots, stream)) != hipSuccess ||
        (e = launch_reset(v, nullptr, batch, stream)) != hipSuccess ||
        (e = launch_feed(S, v, nullptr, batch, prompt_tokens, prompt_offsets, nullptr, nullptr,
                         nullptr, nullptr, nullptr, stream)) != hipSuccess) {
        batch_release(bt);
        return fail_hip("sam_batch_init_noalloc: launch", e);
    }
    *out = bt;
    return SAM_OK;
}

int sam_batch_step(sam_batch *bt, const int32_t *accepted, const int32_t *counts,
                   int32_t *match_len, int32_t *draft, int32_t *draft_len, int32_t *source,
                   void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_step: batch is NULL");
    if (!accepted || !counts || !match_len || !draft || !draft_len || !source)
        return fail(SAM_EINVAL, "sam_batch_step: NULL buffer");
    StaticView S = bt->corpus ? bt->corpus->view : StaticView{};
    hipError_t e = launch_feed(S, bt->view, nullptr, bt->view.batch, accepted, nullptr, counts,
                               match_len, draft, draft_len, source, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip("sam_batch_step: launch", e);
    return SAM_OK;
}

int sam_batch_replay(sam_batch *bt, int32_t n_steps, const int32_t *accepted, const int32_t *counts,
                     int32_t *match_len, int32_t *draft, int32_t *draft_len, int32_t *source,
                     void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_replay: batch is NULL");
    if (!accepted || !counts || !match_len || !draft || !draft_len || !source)
        return fail(SAM_EINVAL, "sam_batch_replay: NULL buffer");
    if (n_steps < 1) return fail(SAM_EINVAL, "sam_batch_replay: n_steps must be >= 1");
    StaticView S = bt->corpus ? bt->corpus->view : StaticView{};
    hipError_t e = launch_replay(S, bt->view, n_steps, accepted, counts, match_len, draft,
                                 draft_len, source, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip("sam_batch_replay: launch", e);
    return SAM_OK;
}

int sam_membench(int32_t kind, int64_t size, int64_t count, int32_t workgroups, double *result)
{
    if (!result) return fail(SAM_EINVAL, "sam_membench: result is NULL");
    std::string err;
    const int rc = membench(kind, size, count, workgroups, result, err);
    return rc == SAM_OK ? SAM_OK : fail(rc, err);
}

int sam_batch_tree_draft(sam_batch *bt, int32_t max_size, int32_t *tokens, int32_t *parents,
                         float *probs, int32_t *sizes, void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_tree_draft: batch is NULL");
    if (!tokens || !parents || !probs || !sizes)
        return fail(SAM_EINVAL, "sam_batch_tree_draft: NULL buffer");
    if (!bt->corpus || !bt->corpus->view.topk)
        return fail(SAM_EINVAL, "sam_batch_tree_draft: the batch has no corpus with a top-k "
                                "table (sam_corpus_build_topk)");
    if (max_size < 1 || max_size > kMaxTreeSize)
        return fail(SAM_EINVAL, "sam_batch_tree_draft: max_size must be in 1 .. " +
                                    std::to_string(kMaxTreeSize));
    hipError_t e = launch_tree(bt->corpus->view, bt->view, max_size, tokens, parents, probs,
                               sizes, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip("sam_batch_tree_draft: launch", e);
    return SAM_OK;
}

int sam_batch_reset(sam_batch *bt, const int32_t *slots, int32_t n_slots,
                    const int32_t *prompt_tokens, const int64_t *prompt_offsets, void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_reset: batch is NULL");
    if (!slots || !prompt_tokens || !prompt_offsets)
        return fail(SAM_EINVAL, "sam_batch_reset: NULL buffer");
    const BatchView &v = bt->view;
    if (n_slots < 1 || n_slots > v.batch)
        return fail(SAM_EINVAL, "sam_batch_reset: n_slots must be in 1 .. batch");
    hipStream_t stream = (hipStream_t)hip_stream;
    std::vector<int32_t> hs;
    std::vector<int64_t> offs;
    std::vector<char> seen;
    try {
        hs.resize((size_t)n_slots);
        offs.resize((size_t)n_slots + 1);
        seen.assign((size_t)v.batch, 0);
    } catch (const std::bad_alloc &) {
        return fail(SAM_ENOMEM, "sam_batch_reset: out of host memory");
    }
    HIP_TRY(hipMemcpyAsync(hs.data(), slots, hs.size() * sizeof(int32_t), hipMemcpyDeviceToHost,
                           stream));
    HIP_TRY(hipMemcpyAsync(offs.data(), prompt_offsets, offs.size() * sizeof(int64_t),
                           hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    if (offs[0] < 0) return fail(SAM_EINVAL, "sam_batch_reset: prompt_offsets[0] < 0");
    for (int32_t i = 0; i < n_slots; i++) {
        if (hs[i] < 0 || hs[i] >= v.batch)
            return fail(SAM_EINVAL, "sam_batch_reset: slot " + std::to_string(hs[i]) +
                                        " is outside the batch");
        if (seen[hs[i]])
            return fail(SAM_EINVAL, "sam_batch_reset: slot " + std::to_string(hs[i]) +
                                        " is listed twice");
        seen[hs[i]] = 1;
        const int64_t len = offs[i + 1] - offs[i];
        if (len < 0) return fail(SAM_EINVAL, "sam_batch_reset: prompt_offsets must not decrease");
        if (len > (int64_t)v.max_seq_len)
            return fail(SAM_ECAPACITY, "sam_batch_reset: prompt " + std::to_string(i) + " has " +
                                           std::to_string(len) + " tokens, max_seq_len is " +
                                           std::to_string(v.max_seq_len));
    }
    StaticView S = bt->corpus ? bt->corpus->view : StaticView{};
    hipError_t e;
    if ((e = launch_reset(v, slots, n_slots, stream)) != hipSuccess ||
        (e = launch_feed(S, v, slots, n_slots, prompt_tokens, prompt_offsets, nullptr, nullptr,
                         nullptr, nullptr, nullptr, stream)) != hipSuccess)
        return fail_hip("sam_batch_reset: launch", e);
    return SAM_OK;
}

int sam_batch_debug(const sam_batch *bt, int32_t *s1, int32_t *l1, int32_t *s2, int32_t *l2,
                    void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_debug: batch is NULL");
    hipError_t e = launch_debug(bt->view, s1, l1, s2, l2, nullptr, nullptr, nullptr,
                                (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip("sam_batch_debug: launch", e);
    return SAM_OK;
}

int sam_batch_sizes(const sam_batch *bt, int32_t *text_len, int32_t *n_states, int32_t *n_trans,
                    void *hip_stream)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_sizes: batch is NULL");
    hipError_t e = launch_debug(bt->view, nullptr, nullptr, nullptr, nullptr, text_len, n_states,
                                n_trans, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail_hip("sam_batch_sizes: launch", e);
    return SAM_OK;
}

int sam_batch_status(const sam_batch *bt, uint32_t *status, void *hip_stream)
{
    if (!bt || !status) return fail(SAM_EINVAL, "sam_batch_status: NULL argument");
    hipStream_t stream = (hipStream_t)hip_stream;
    HIP_TRY(hipMemcpyAsync(status, bt->view.status, sizeof(uint32_t), hipMemcpyDeviceToHost,
                           stream));
    HIP_TRY(hipStreamSynchronize(stream));
    return SAM_OK;
}

int sam_batch_set_threshold(sam_batch *bt, int32_t l_threshold)
{
    if (!bt) return fail(SAM_EINVAL, "sam_batch_set_threshold: batch is NULL");
    bt->view.l_threshold = l_threshold < 0 ? -1 : l_threshold;
    return SAM_OK;
}

int sam_set_progress_callback(sam_progress_fn fn, void *user)
{
    g_progress = fn;
    g_progress_user = user;
    return SAM_OK;
}

int sam_set_layout_override(int mode)
{
    if (mode < 0 || mode > 63) return fail(SAM_EINVAL, "sam_set_layout_override: mode is 0 .. 63");
    g_layout_override = mode;
    return SAM_OK;
}

int sam_batch_info(const sam_batch *bt, int64_t *device_bytes)
{
    if (!bt || !device_bytes) return fail(SAM_EINVAL, "sam_batch_info: NULL argument");
    *device_bytes = bt->device_bytes;
    return SAM_OK;
}

void sam_batch_free(sam_batch *bt)
{
    if (!bt) return;
    batch_release(bt);
}

}  // extern "C"
