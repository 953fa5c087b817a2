// Constants and the device control block shared by the stages of the backward.
#pragma once
#include "emb_internal.h"

struct BwdCtrl {
    uint32_t abort;        // offsets are not a partition of [0, nnz): do nothing
    uint32_t num_runs;     // runs of equal keys, those of the sentinel included (distinct-row list only)
    uint32_t reserved0;
    uint32_t num_unique;   // U
    unsigned long long task_and_multi_count;  // low half: chunk tasks; high half: queued runs of several chunks
    uint32_t pad[58];
};
static_assert(sizeof(BwdCtrl) == 256, "control block is one 256-byte line");

constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_BLOCK = 512;
constexpr int SORT_WAVES = SORT_BLOCK / EMB_WAVE;
constexpr int SORT_ITEMS = 8;
constexpr int SORT_TILE = SORT_BLOCK * SORT_ITEMS;  // 4096 records per workgroup
constexpr int SORT_PAD = 320;                       // records of slack after the key / payload arrays

constexpr int UPD_BLOCK = 128;       // two wavefronts: measured better than four for the update kernels
constexpr int UPD_SPAN = 256;        // sorted records per wavefront in the update
constexpr int UPD_LOOK = 32;         // records of look-ahead after a span
constexpr int UPD_SHORT_MAX = 32;    // longest run the short-run kernel sums itself
constexpr int UPD_QSLOTS = UPD_SPAN / (UPD_SHORT_MAX + 1) + 1;  // runs longer than that which can start in one span
constexpr int LONG_CHUNK = 256;     // records of a queued run summed by one wavefront
constexpr int PREP_BLOCK = 1024;     // workgroup of the kernel that turns queued runs into tasks
constexpr int UPD_LDS_TABLES = 512; // table directories up to this size are staged in LDS

struct LongSeg {
    uint32_t lo, hi;       // records [lo, hi) of the sorted arrays
    uint32_t chunk_base;   // first chunk-sum slot (runs of several chunks)
    uint32_t n_chunks;
};
