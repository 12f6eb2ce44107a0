// Schedule records shared by the host scheduler and the prefill kernel (plain structs, no logic).
#ifndef KSA_SCHEDULE_H_
#define KSA_SCHEDULE_H_

#include <stdint.h>

// Heights of the tiles the schedule is cut into.  A workgroup of the prefill kernels owns KSA_Q_TILE (row, query
// head) pairs: a query tile of KSA_Q_TILE / S consecutive rows of one index space (compact text indices or compact
// summary ordinals) for S query heads that share a KV head (S = 1, 2 or 4, chosen per layout: the largest of them
// that divides the group size).  Stacking heads rather than rows keeps every wavefront of the workgroup busy on the
// short, chunk-aligned key runs of the mask (the sliding-chunk text, a summary row's own chunk), which a taller
// query tile visits with most of its rows masked.  A key tile is KSA_K_TILE rows.
#define KSA_Q_TILE 256
#define KSA_MAX_HEAD_STACK 4
#define KSA_K_TILE 64
#define KSA_MAX_SEGMENTS 2
#define KSA_NUM_XCD 8

// A run of consecutive key rows of one index space, walked in steps of KSA_K_TILE from `begin`.
// Every row of the query tile sees every key in [full_lo, full_hi) (an empty range if full_hi <= full_lo): a key
// tile that lies inside it needs no mask (FULL); for every other tile of the run the kernel clips each query
// row's visible range to [begin, end) (MASKED).
struct KsaSegment {
    int32_t space;   // KSA_SPACE_TEXT / KSA_SPACE_SUMMARY
    int32_t begin;
    int32_t end;
    int32_t full_lo;
    int32_t full_hi;
    int32_t pad;
};

// One query tile and the key runs that hold all of its visible keys.
struct KsaWorkItem {
    int32_t q_space;
    int32_t q_begin;
    int32_t q_count;   // <= the layout's query tile height
    int32_t n_seg;
    KsaSegment seg[KSA_MAX_SEGMENTS];
    int32_t n_tiles;   // key tiles over all segments (the item's cost)
    int32_t pipelined; // 1: every segment meets the conditions of the kernel's pipelined loop (see ksa_item_pipelined)
    int32_t pad[2];
};

// What workgroup blockIdx.x does: item < 0 means nothing.
struct KsaWgEntry {
    int32_t item;
    int32_t batch;
    int32_t q_head;    // first of the query heads the workgroup stacks
    int32_t pad;
};

#endif
