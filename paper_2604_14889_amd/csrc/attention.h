// Argument blocks shared by the attention kernels (internal).
#pragma once

#include <hip/hip_runtime.h>

#include "memosight.h"
#include "plan.h"

namespace ms {

constexpr int kMaxRowwaveSplits = 16;

// Per-call sequence ids and the cache lengths the host knows (lower bounds while device-side commits
// are outstanding), passed by value in the kernel argument block.
struct BatchMeta {
    int seq[MS_MAX_BATCH];
    int len[MS_MAX_BATCH];
};

struct AttnArgs {
    const void* pool_layer;  // first element of this layer's pages
    const int* d_pt;         // device page tables [max_seqs][max_pages]
    const int* d_len;        // device lengths [max_seqs]: what the kernels go by (the host's may lag behind device-side commits)
    const float* inv_freq;   // [head_dim / 2]
    const void* q;
    const void* k_new;
    const void* v_new;
    const int* pos;
    const int* ctx_new;      // may be null: default layout
    void* out;
    float* ws;
    int n_q, n_verify, n_q_heads, n_kv_heads, group, max_pages;
    long page_elems;
    int n_splits, chunk;
    float scale;
};

}  // namespace ms

struct ms_cache;

namespace ms {

// attention.hip
int static_scratch(int device, void** ptr);

// attention_mfma.hip
bool mfma_eligible(const ms_cache* c, int n_q);
size_t mfma_workspace_bytes(const ms_cache* c, int B, int n_q);
int reset_arrival_counters(ms_cache* c, int published, hipStream_t stream);
int launch_mfma(ms_cache* c, const AttnArgs& a, const BatchMeta& bm, int B, hipStream_t stream);

}  // namespace ms
