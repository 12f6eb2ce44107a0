// Internal declarations shared by the host-side translation units of libksa.
#ifndef KSA_INTERNAL_H_
#define KSA_INTERNAL_H_

#include <vector>

#include "ksa.h"
#include "ksa_schedule.h"

struct ksa_layout {
    ksa_params p;
    int64_t aug_len;      // L
    int32_t n_chunks;     // J
    std::vector<KsaWorkItem> items;   // one per query tile, heaviest first
    std::vector<KsaWgEntry> entries;  // one per workgroup: first those of the pipelined items, then the others
    int32_t n_pipelined_entries = 0;  // length of the first part (a multiple of 8)
    int32_t n_pipelined_items = 0;    // items with KsaWorkItem::pipelined set
    int32_t head_stack = 1;           // query heads per workgroup (1, 2 or 4)
    int32_t q_tile_rows = KSA_Q_TILE; // rows of a query tile = KSA_Q_TILE / head_stack
    // device copies (owned), valid on `device` once uploaded
    int device = -1;
    void *d_items = nullptr;
    void *d_entries = nullptr;
};

// Validates the problem statement; returns KSA_OK or the error.
int ksa_validate_params(const ksa_params *p);

// Launchers implemented in the .hip files.  All pointers device, strides in elements.
struct KsaPrefillLaunch {
    const void *q, *k, *v;
    void *o;
    float *lse;
    int64_t q_strides[3], kv_strides[3], o_strides[3];
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t n_entries;
    int32_t n_pipelined_entries;                  // entries [0, n_pipelined_entries): the pipelined kernel's; rest: the generic one's
    int32_t n_pipelined_items, n_generic_items;   // how many work items each of the two kernels owns
    int32_t head_stack;                           // query heads per workgroup
    ksa_params p;
    int64_t aug_len;
    void *workspace;          // key-major copy of V, written by the launch itself
    int32_t phases;           // bit 0: write the key-major copy of V; bit 1: run the attention kernels
    size_t workspace_bytes;
};
size_t ksa_prefill_workspace_size(const ksa_params &p);
int ksa_launch_prefill(const KsaPrefillLaunch &a, void *stream);

struct KsaPrefillBwdLaunch {
    const void *q, *k, *v, *o, *d_o;
    const float *lse;
    void *dq, *dk, *dv;
    int64_t q_strides[3], kv_strides[3], o_strides[3], dq_strides[3], dkv_strides[3];
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t n_entries;
    int32_t head_stack;       // query heads per workgroup of the schedule
    ksa_params p;
    int64_t aug_len;
    void *workspace;          // delta_i = dO_i . O_i per (batch, query head, row), fp32
    size_t workspace_bytes;
};
size_t ksa_prefill_bwd_workspace_size(const ksa_params &p, int64_t aug_len);
int ksa_launch_prefill_bwd(const KsaPrefillBwdLaunch &a, void *stream);

struct KsaDecodeLaunch {
    const void *q, *k_cache, *v_cache;
    const int32_t *pos;
    void *o;
    float *lse;
    int64_t cache_strides[3];
    float *workspace;
    int32_t n_splits;
    int32_t summary_capacity;
    int32_t kind;             // KSA_ROW_TEXT: pos is a text index; KSA_ROW_SUMMARY: pos is a summary ordinal
    ksa_params p;
};
int ksa_launch_decode(const KsaDecodeLaunch &a, void *stream);
// Device address (current device) of the library's static scratch array of KSA_DECODE_STATIC_SCRATCH_BYTES bytes.
int ksa_decode_static_scratch(float **ptr);

struct KsaCacheFillLaunch {
    const void *k, *v;
    void *k_cache, *v_cache;
    int64_t kv_strides[3], cache_strides[3];
    int64_t n_prefill;
    int32_t summary_capacity;
    ksa_params p;
};
int ksa_launch_cache_fill(const KsaCacheFillLaunch &a, void *stream);

struct KsaCacheAppendLaunch {
    const void *k_new, *v_new;
    const int32_t *pos;
    void *k_cache, *v_cache;
    int64_t cache_strides[3];
    int32_t kind;
    int32_t summary_capacity;
    ksa_params p;
};
int ksa_launch_cache_append(const KsaCacheAppendLaunch &a, void *stream);
int ksa_decode_default_splits(const ksa_params *p);

#endif
