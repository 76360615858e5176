// Kernel argument blocks and launcher prototypes (device side of the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sam_layout.h"

namespace sam {

constexpr uint32_t SAM_STATUS_CAPACITY_BIT = 1u;
constexpr uint32_t SAM_STATUS_TOKEN_BIT    = 2u;
constexpr uint32_t SAM_STATUS_COUNT_BIT    = 4u;
constexpr uint32_t SAM_STATUS_INTERNAL_BIT = 8u;

// Static automaton in device memory (all read-only for the kernels).
struct StaticView {
    const int32_t *text;
    const LinkRec *linkrec;
    const RootEnt *root;
    const Slot    *slots;
    uint64_t       n_buckets;
    uint32_t       n_tokens;
    uint32_t       n_states;
    const TopEnt  *topk;       // [n_states * top_k], NULL until sam_corpus_build_topk
    int32_t        top_k;
};

// A batch of sequences: per-sequence regions are laid out back to back.
struct BatchView {
    int32_t   batch;
    int32_t   vocab;
    uint32_t  max_seq_len;
    uint32_t  max_states;      // records per sequence (2 * max_seq_len + 2)
    uint32_t  dyn_buckets;     // 128-byte buckets per sequence
    int32_t   compact;         // 1: DynRecCompact / SlotCompact, 0: DynRec / Slot
    int32_t   max_accept;
    int32_t   draft_len;
    int32_t   l_bias;
    int32_t   l_threshold;     // < 0: no auxiliary drafter
    int32_t   has_static;
    int32_t   no_asm;          // testing: 1 = the C++ token loops instead of the assembly
    int32_t   scout;           // 1 = the step kernel runs with its two prefetching waves
    int32_t  *dyn_text;        // [batch, max_seq_len]
    void     *dyn_rec;         // [batch, max_states] records of the chosen layout
    void     *dyn_slots;       // [batch, dyn_buckets] buckets of 128 bytes
    SeqMeta  *meta;            // [batch]
    uint32_t *status;          // [1]
};

// seq_map (device, may be NULL): in ingest mode workgroup i serves sequence seq_map[i];
// n_seqs workgroups are launched.  Step mode always covers the whole batch.
hipError_t launch_feed(const StaticView &S, const BatchView &B, const int32_t *seq_map,
                       int n_seqs, const int32_t *tokens, const int64_t *offsets,
                       const int32_t *counts, int32_t *match_len, int32_t *draft,
                       int32_t *draft_len, int32_t *source, hipStream_t stream);
// A whole schedule of n_steps steps in one launch (rows [step, sequence] of every array).
// linkrec[s] from the link pairs and the (already uploaded) slot and root tables, whose end
// positions receive the wide flag of their targets.  wide: (n_states + 31) / 32 words of
// scratch, zeroed by the caller.
hipError_t launch_staterec(const LinkPair *pairs, Slot *slots, RootEnt *root, LinkRec *linkrec,
                           uint32_t *wide, uint32_t n_states, uint64_t n_slots, uint32_t vocab,
                           hipStream_t stream);
// Transitions of wide states among the n_slots slots (added to *count, device memory), and
// their insertion into a table of n_buckets buckets whose keys are all kNil.
hipError_t launch_count_wide(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                             unsigned long long *count, hipStream_t stream);
hipError_t launch_compact_slots(const Slot *slots, const uint32_t *wide, uint64_t n_slots,
                                Slot *out, uint64_t n_buckets, hipStream_t stream);
hipError_t launch_replay(const StaticView &S, const BatchView &B, int n_steps,
                         const int32_t *accepted, const int32_t *counts, int32_t *match_len,
                         int32_t *draft, int32_t *draft_len, int32_t *source, hipStream_t stream);
// seq_map NULL: fresh records and cursors for sequences 0 .. n_seqs-1 (slot tables
// are cleared by the caller).  Otherwise: the listed sequences, slot tables included.
hipError_t launch_reset(const BatchView &B, const int32_t *seq_map, int n_seqs,
                        hipStream_t stream);
// Every byte of [base, base + bytes) becomes 0xFF (the empty slot key); bytes is a
// multiple of 16.  A kernel, not a memset node, so that it may be captured in a graph.
hipError_t launch_fill_empty(void *base, size_t bytes, hipStream_t stream);
// Best-first tree drafts from the static cursor of every sequence (Algorithm 4).
hipError_t launch_tree(const StaticView &S, const BatchView &B, int max_size, int32_t *tokens,
                       int32_t *parents, float *probs, int32_t *sizes, hipStream_t stream);
hipError_t launch_debug(const BatchView &B, int32_t *s1, int32_t *l1, int32_t *s2, int32_t *l2,
                        int32_t *text_len, int32_t *n_states, int32_t *n_trans,
                        hipStream_t stream);

}  // namespace sam
