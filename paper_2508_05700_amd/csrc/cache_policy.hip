// Which rows the HBM hot-row cache of a host-resident table holds (paper
// Section 3.3 for the hosted table; Section 6 names better caching strategies
// as open work and gives no policy, so this one is a stated choice):
// frequency-based admission with batched refresh.
//
//   observe   one u32 counter per table row counts the lookups of that row;
//   select    at a refresh the cache takes the num_hot rows with the largest
//             counters (a tie goes to the smaller row number), and the
//             counters are aged by a right shift.
//
// The selection is an exact top-k without a sort: four passes of 8-bit
// histograms, most significant digit first, find the counter value of the
// num_hot-th row in preference order (the threshold) and how many rows with
// exactly that value are taken; two more streaming passes then count and
// compact the selected rows in ascending row order, which is the order the
// cache index needs.  Everything is integer work: results are exact.
#include <mutex>

#include "emb_internal.h"
#include "u64mod.h"

namespace {

constexpr int CP_BLOCK = 256;
constexpr int SEL_RADIX = 256;
constexpr int SEL_PASSES = 4;
constexpr int SEL_PER_THREAD = 16;                         // consecutive rows per thread in count/write
constexpr int SEL_TILE = CP_BLOCK * SEL_PER_THREAD;        // rows per workgroup in count/write
constexpr int SCAN_BLOCK = 1024;

struct SelCtrl {
    uint64_t need;       // rows still to take among those whose high digits equal prefix
    uint32_t prefix;     // digits of the threshold fixed so far (most significant first)
    uint32_t pad;
};

// Workspace: SelCtrl | hist u64[4][256] | tile counts uint2[tiles] | gt_before u64[tiles] | eq_before u64[tiles]
struct SelLayout {
    size_t ctrl, hist, counts, gt_before, eq_before, total;
    int64_t tiles;
};

SelLayout sel_layout(int64_t num_rows)
{
    SelLayout L;
    L.tiles = (num_rows + SEL_TILE - 1) / SEL_TILE;
    size_t o = 0;
    L.ctrl = o;
    o += 256;
    L.hist = o;
    o += sizeof(uint64_t) * SEL_PASSES * SEL_RADIX;
    L.counts = o;
    o += ((size_t)L.tiles * sizeof(uint2) + 255) / 256 * 256;
    L.gt_before = o;
    o += ((size_t)L.tiles * sizeof(uint64_t) + 255) / 256 * 256;
    L.eq_before = o;
    o += ((size_t)L.tiles * sizeof(uint64_t) + 255) / 256 * 256;
    L.total = o;
    return L;
}

// Popular rows repeat: under a Zipf law the most popular row alone takes a tenth of all lookups, and
// atomics on one address are served one at a time by the L2.  A workgroup therefore first merges its
// OBS_TILE lookups in a small LDS hash table (row -> count, open addressing) and then adds each distinct
// row's count to its counter once.  A lookup that finds no slot within a few probes goes to its counter
// directly, so the result is the exact count either way.
constexpr int OBS_ITEMS = 8;                       // lookups per thread
constexpr int OBS_TILE = CP_BLOCK * OBS_ITEMS;     // lookups per workgroup
constexpr int OBS_SLOTS = 2 * OBS_TILE;            // load factor at most one half
constexpr int OBS_PROBES = 8;
constexpr unsigned long long OBS_EMPTY = ~0ull;    // not a row number: rows are below 2^63

template <bool HASHED>
__global__ __launch_bounds__(CP_BLOCK) void cache_observe_kernel(const int64_t *__restrict__ ids, int64_t nnz,
                                                                 uint64_t num_rows, uint64_t salt, uint64_t magic,
                                                                 uint32_t *freq, uint32_t *status)
{
    __shared__ unsigned long long keys[OBS_SLOTS];
    __shared__ uint32_t counts[OBS_SLOTS];
    for (int i = threadIdx.x; i < OBS_SLOTS; i += CP_BLOCK) {
        keys[i] = OBS_EMPTY;
        counts[i] = 0u;
    }
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * OBS_TILE;
#pragma unroll
    for (int k = 0; k < OBS_ITEMS; ++k) {
        const int64_t j = base + (int64_t)k * CP_BLOCK + threadIdx.x;
        if (j >= nnz) continue;
        uint64_t r = (uint64_t)ids[j];
        if (HASHED) r = emb_fast_mod(emb_splitmix64(r ^ salt), num_rows, magic);
        if (r >= num_rows) {  // negative row numbers are huge as unsigned
            emb_flag(status, EMB_STATUS_BAD_INDEX);
            continue;
        }
        uint32_t slot = (uint32_t)((r * UINT64_C(0x9E3779B97F4A7C15)) >> 32) & (OBS_SLOTS - 1);
        bool placed = false;
        for (int p = 0; p < OBS_PROBES && !placed; ++p) {
            const unsigned long long prev = atomicCAS(&keys[slot], OBS_EMPTY, (unsigned long long)r);
            if (prev == OBS_EMPTY || prev == (unsigned long long)r) {
                atomicAdd(&counts[slot], 1u);
                placed = true;
            } else {
                slot = (slot + 1) & (OBS_SLOTS - 1);
            }
        }
        if (!placed) atomicAdd(freq + r, 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < OBS_SLOTS; i += CP_BLOCK) {
        const uint32_t c = counts[i];
        if (c) atomicAdd(freq + keys[i], c);
    }
}

__global__ __launch_bounds__(CP_BLOCK) void sel_init_kernel(SelCtrl *ctrl, unsigned long long *hist, int64_t num_hot)
{
    for (int i = threadIdx.x; i < SEL_PASSES * SEL_RADIX; i += CP_BLOCK) hist[i] = 0ull;
    if (threadIdx.x == 0) {
        ctrl->need = (uint64_t)num_hot;
        ctrl->prefix = 0u;
        ctrl->pad = 0u;
    }
}

// Histogram of digit `pass` (0 = least significant byte) over the counters
// whose higher digits equal the prefix found so far.
__global__ __launch_bounds__(CP_BLOCK) void sel_hist_kernel(const uint32_t *__restrict__ freq, int64_t num_rows, int pass,
                                                            const SelCtrl *__restrict__ ctrl, unsigned long long *hist)
{
    __shared__ uint32_t lds[SEL_RADIX];
    lds[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t prefix = ctrl->prefix;
    const int high_shift = 8 * (pass + 1);   // 32 for the first pass: every counter matches
    const int low_shift = 8 * pass;
    const int64_t quads = (num_rows + 3) / 4;
    // grid-stride over groups of 4 counters; the trip count is uniform over a wavefront's lanes up to the
    // tail, and the ballots below are taken by every lane of the wavefront in each trip
    const int64_t stride = (int64_t)gridDim.x * CP_BLOCK;
    const int64_t trips = (quads + stride - 1) / stride;
    int64_t q = (int64_t)blockIdx.x * CP_BLOCK + threadIdx.x;
    for (int64_t it = 0; it < trips; ++it, q += stride) {
        uint32_t v[4] = {0u, 0u, 0u, 0u};
        int valid = 0;
        if (q < quads) {
            const int64_t r0 = q * 4;
            if (r0 + 4 <= num_rows) {
                const uint4 x = *reinterpret_cast<const uint4 *>(freq + r0);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                valid = 4;
            } else {
                valid = (int)(num_rows - r0);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (c < valid) v[c] = freq[r0 + c];
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool match = c < valid && (high_shift >= 32 || (v[c] >> high_shift) == prefix);
            const uint32_t digit = (v[c] >> low_shift) & (SEL_RADIX - 1);
            const unsigned long long active = __ballot(match);
            if (active == 0ull) continue;                                 // wavefront-uniform
            const int leader = __ffsll(active) - 1;
            const uint32_t d0 = __shfl(digit, leader, EMB_WAVE);
            const unsigned long long same = __ballot(match && digit == d0);
            if (same == active) {                                         // wavefront-uniform: one add for all lanes
                if ((int)(threadIdx.x & (EMB_WAVE - 1)) == leader) atomicAdd(&lds[d0], (uint32_t)__popcll(active));
            } else if (match) {
                atomicAdd(&lds[digit], 1u);
            }
        }
    }
    __syncthreads();
    const uint32_t n = lds[threadIdx.x];
    if (n) atomicAdd(hist + threadIdx.x, (unsigned long long)n);
}

// Fix the next digit of the threshold: the largest digit d such that the
// counters with a larger digit (and the prefix) number fewer than `need`.
__global__ __launch_bounds__(SEL_RADIX) void sel_pick_kernel(const unsigned long long *__restrict__ hist, SelCtrl *ctrl)
{
    __shared__ unsigned long long c[SEL_RADIX];
    c[threadIdx.x] = hist[threadIdx.x];
    __syncthreads();
    if (threadIdx.x != 0) return;
    const uint64_t need = ctrl->need;    // >= 1 and <= the number of matching counters
    uint64_t above = 0;
    int d = SEL_RADIX - 1;
    for (; d > 0; --d) {
        if (above + c[d] >= need) break;
        above += c[d];
    }
    ctrl->prefix = (ctrl->prefix << 8) | (uint32_t)d;
    ctrl->need = need - above;
}

__device__ __forceinline__ void sel_load16(const uint32_t *__restrict__ freq, int64_t r0, int64_t num_rows, uint32_t (&v)[SEL_PER_THREAD],
                                           int &valid)
{
    if (r0 + SEL_PER_THREAD <= num_rows) {
#pragma unroll
        for (int i = 0; i < SEL_PER_THREAD / 4; ++i) {
            const uint4 x = *reinterpret_cast<const uint4 *>(freq + r0 + 4 * i);
            v[4 * i] = x.x; v[4 * i + 1] = x.y; v[4 * i + 2] = x.z; v[4 * i + 3] = x.w;
        }
        valid = SEL_PER_THREAD;
    } else {
        valid = r0 < num_rows ? (int)(num_rows - r0) : 0;
#pragma unroll
        for (int i = 0; i < SEL_PER_THREAD; ++i) v[i] = i < valid ? freq[r0 + i] : 0u;
    }
}

// Inclusive scan over the workgroup of a value packed as (above-threshold count | at-threshold count << 16);
// neither field can exceed SEL_TILE = 4096.  Returns the exclusive prefix of the calling thread; total gets the sum.
__device__ __forceinline__ uint32_t sel_block_scan(uint32_t mine, uint32_t &total)
{
    __shared__ uint32_t wave_sum[CP_BLOCK / EMB_WAVE];
    const int lane = threadIdx.x & (EMB_WAVE - 1), wave = threadIdx.x / EMB_WAVE;
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < EMB_WAVE; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, EMB_WAVE);
        if (lane >= d) incl += up;
    }
    if (lane == EMB_WAVE - 1) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t before = 0u, all = 0u;
#pragma unroll
    for (int w = 0; w < CP_BLOCK / EMB_WAVE; ++w) {
        const uint32_t s = wave_sum[w];
        if (w < wave) before += s;
        all += s;
    }
    total = all;
    return before + incl - mine;
}

// Per tile of SEL_TILE rows: how many counters lie above the threshold, how many equal it.
__global__ __launch_bounds__(CP_BLOCK) void sel_count_kernel(const uint32_t *__restrict__ freq, int64_t num_rows,
                                                             const SelCtrl *__restrict__ ctrl, uint2 *counts)
{
    const uint32_t thr = ctrl->prefix;
    const int64_t r0 = (int64_t)blockIdx.x * SEL_TILE + (int64_t)threadIdx.x * SEL_PER_THREAD;
    uint32_t v[SEL_PER_THREAD];
    int valid;
    sel_load16(freq, r0, num_rows, v, valid);
    uint32_t mine = 0u;
#pragma unroll
    for (int i = 0; i < SEL_PER_THREAD; ++i)
        if (i < valid) mine += v[i] > thr ? 1u : (v[i] == thr ? 0x10000u : 0u);
    uint32_t total;
    (void)sel_block_scan(mine, total);
    if (threadIdx.x == 0) counts[blockIdx.x] = make_uint2(total & 0xFFFFu, total >> 16);
}

// Exclusive prefix sums of the tile counts, by one workgroup.
__global__ __launch_bounds__(SCAN_BLOCK) void sel_scan_kernel(const uint2 *__restrict__ counts, int64_t tiles,
                                                              unsigned long long *gt_before, unsigned long long *eq_before)
{
    __shared__ unsigned long long part_gt[SCAN_BLOCK], part_eq[SCAN_BLOCK];
    const int64_t per = (tiles + SCAN_BLOCK - 1) / SCAN_BLOCK;
    const int64_t lo = (int64_t)threadIdx.x * per, hi = lo + per < tiles ? lo + per : tiles;
    unsigned long long g = 0ull, e = 0ull;
    for (int64_t i = lo; i < hi; ++i) {
        const uint2 c = counts[i];
        g += c.x;
        e += c.y;
    }
    part_gt[threadIdx.x] = g;
    part_eq[threadIdx.x] = e;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 1024 partial sums
    for (int d = 1; d < SCAN_BLOCK; d <<= 1) {
        unsigned long long ag = 0ull, ae = 0ull;
        if ((int)threadIdx.x >= d) {
            ag = part_gt[threadIdx.x - d];
            ae = part_eq[threadIdx.x - d];
        }
        __syncthreads();
        part_gt[threadIdx.x] += ag;
        part_eq[threadIdx.x] += ae;
        __syncthreads();
    }
    g = part_gt[threadIdx.x] - g;   // exclusive
    e = part_eq[threadIdx.x] - e;
    for (int64_t i = lo; i < hi; ++i) {
        const uint2 c = counts[i];
        gt_before[i] = g;
        eq_before[i] = e;
        g += c.x;
        e += c.y;
    }
}

// Write the selected rows in ascending order and age the counters.  A row is
// selected if its counter is above the threshold, or equals it and fewer than
// `need` rows with that counter precede it.
__global__ __launch_bounds__(CP_BLOCK) void sel_write_kernel(uint32_t *freq, int64_t num_rows, const SelCtrl *__restrict__ ctrl,
                                                             const unsigned long long *__restrict__ gt_before,
                                                             const unsigned long long *__restrict__ eq_before,
                                                             int64_t num_hot, int decay_shift, int64_t *__restrict__ hot_out)
{
    const uint32_t thr = ctrl->prefix;
    const uint64_t take = ctrl->need;
    const int64_t r0 = (int64_t)blockIdx.x * SEL_TILE + (int64_t)threadIdx.x * SEL_PER_THREAD;
    uint32_t v[SEL_PER_THREAD];
    int valid;
    sel_load16(freq, r0, num_rows, v, valid);
    uint32_t mine = 0u;
#pragma unroll
    for (int i = 0; i < SEL_PER_THREAD; ++i)
        if (i < valid) mine += v[i] > thr ? 1u : (v[i] == thr ? 0x10000u : 0u);
    uint32_t total;
    const uint32_t excl = sel_block_scan(mine, total);
    uint64_t gt = gt_before[blockIdx.x] + (excl & 0xFFFFu);
    uint64_t eq = eq_before[blockIdx.x] + (excl >> 16);
#pragma unroll
    for (int i = 0; i < SEL_PER_THREAD; ++i) {
        if (i >= valid) continue;
        const bool above = v[i] > thr, tied = v[i] == thr;
        if (above || (tied && eq < take)) {
            const uint64_t pos = gt + (eq < take ? eq : take);
            if (pos < (uint64_t)num_hot) hot_out[pos] = r0 + i;   // always true; keeps a corrupted workspace from writing outside
        }
        gt += above ? 1u : 0u;
        eq += tied ? 1u : 0u;
    }
    if (decay_shift > 0) {
        if (valid == SEL_PER_THREAD) {
#pragma unroll
            for (int i = 0; i < SEL_PER_THREAD / 4; ++i)
                *reinterpret_cast<uint4 *>(freq + r0 + 4 * i) =
                    make_uint4(v[4 * i] >> decay_shift, v[4 * i + 1] >> decay_shift, v[4 * i + 2] >> decay_shift,
                               v[4 * i + 3] >> decay_shift);
        } else {
            for (int i = 0; i < valid; ++i) freq[r0 + i] = v[i] >> decay_shift;
        }
    }
}

// Aging alone (a refresh that keeps no rows).
__global__ __launch_bounds__(CP_BLOCK) void sel_age_kernel(uint32_t *freq, int64_t num_rows, int decay_shift)
{
    const int64_t r0 = (int64_t)blockIdx.x * SEL_TILE + (int64_t)threadIdx.x * SEL_PER_THREAD;
    for (int i = 0; i < SEL_PER_THREAD; ++i)
        if (r0 + i < num_rows) freq[r0 + i] >>= decay_shift;
}

__global__ __launch_bounds__(CP_BLOCK) void sel_info_kernel(const SelCtrl *__restrict__ ctrl, uint64_t *info)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        info[0] = ctrl->prefix;
        info[1] = ctrl->need;
    }
}

int observe_entry(int64_t num_rows, const int64_t *ids, int64_t nnz, uint32_t *freq_dev, uint32_t *status_dev, void *stream,
                  bool hashed, uint64_t salt)
{
    if (num_rows <= 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    if (nnz == 0) return EMB_OK;
    if (!ids || !freq_dev) return EMB_ERR_INVALID_ARG;
    const int64_t blocks = (nnz + OBS_TILE - 1) / OBS_TILE;
    if (blocks > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    const uint64_t magic = emb_mod_magic((uint64_t)num_rows);
    hipStream_t s = emb_stream(stream);
    if (hashed)
        hipLaunchKernelGGL(cache_observe_kernel<true>, dim3((unsigned)blocks), dim3(CP_BLOCK), 0, s, ids, nnz,
                           (uint64_t)num_rows, salt, magic, freq_dev, status_dev);
    else
        hipLaunchKernelGGL(cache_observe_kernel<false>, dim3((unsigned)blocks), dim3(CP_BLOCK), 0, s, ids, nnz,
                           (uint64_t)num_rows, salt, magic, freq_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

}  // namespace

extern "C" int emb_cache_observe(int64_t num_rows, const int64_t *rows_dev, int64_t nnz, uint32_t *freq_dev,
                                 uint32_t *status_dev, void *stream)
{
    return observe_entry(num_rows, rows_dev, nnz, freq_dev, status_dev, stream, false, 0);
}

extern "C" int emb_cache_observe_hashed(int64_t num_rows, uint64_t salt, const uint64_t *raw_dev, int64_t nnz,
                                        uint32_t *freq_dev, uint32_t *status_dev, void *stream)
{
    return observe_entry(num_rows, reinterpret_cast<const int64_t *>(raw_dev), nnz, freq_dev, status_dev, stream, true,
                         salt);
}

extern "C" int emb_cache_select_workspace_bytes(int64_t num_rows, size_t *bytes)
{
    if (num_rows <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = sel_layout(num_rows).total;
    return EMB_OK;
}

namespace {

// The launches of a selection over counters freq_dev, with the scratch memory at `ws` (laid out by
// sel_layout, at least that large, 256-byte aligned).  Nothing in `ws` has to be zero on entry:
// sel_init_kernel clears the control block and the histograms, every other word is written before
// it is read.
int select_run(uint32_t *freq_dev, int64_t num_rows, int64_t num_hot, int32_t decay_shift, const SelLayout &L, char *ws,
               int64_t *hot_rows_out_dev, uint64_t *info_out_dev, hipStream_t s)
{
    SelCtrl *ctrl = reinterpret_cast<SelCtrl *>(ws + L.ctrl);
    unsigned long long *hist = reinterpret_cast<unsigned long long *>(ws + L.hist);
    uint2 *counts = reinterpret_cast<uint2 *>(ws + L.counts);
    unsigned long long *gt_before = reinterpret_cast<unsigned long long *>(ws + L.gt_before);
    unsigned long long *eq_before = reinterpret_cast<unsigned long long *>(ws + L.eq_before);

    hipLaunchKernelGGL(sel_init_kernel, dim3(1), dim3(CP_BLOCK), 0, s, ctrl, hist, num_hot);
    EMB_RETURN_IF_LAUNCH_FAILED();
    if (num_hot > 0) {   // with nothing to take there is no threshold: the counters only age
        const int64_t quads = (num_rows + 3) / 4;
        int64_t hblocks = (quads + CP_BLOCK - 1) / CP_BLOCK;
        if (hblocks > 4096) hblocks = 4096;
        for (int pass = SEL_PASSES - 1; pass >= 0; --pass) {
            hipLaunchKernelGGL(sel_hist_kernel, dim3((unsigned)hblocks), dim3(CP_BLOCK), 0, s, freq_dev, num_rows, pass,
                               ctrl, hist + (size_t)pass * SEL_RADIX);
            EMB_RETURN_IF_LAUNCH_FAILED();
            hipLaunchKernelGGL(sel_pick_kernel, dim3(1), dim3(SEL_RADIX), 0, s, hist + (size_t)pass * SEL_RADIX, ctrl);
            EMB_RETURN_IF_LAUNCH_FAILED();
        }
        hipLaunchKernelGGL(sel_count_kernel, dim3((unsigned)L.tiles), dim3(CP_BLOCK), 0, s, freq_dev, num_rows, ctrl,
                           counts);
        EMB_RETURN_IF_LAUNCH_FAILED();
        hipLaunchKernelGGL(sel_scan_kernel, dim3(1), dim3(SCAN_BLOCK), 0, s, counts, L.tiles, gt_before, eq_before);
        EMB_RETURN_IF_LAUNCH_FAILED();
        hipLaunchKernelGGL(sel_write_kernel, dim3((unsigned)L.tiles), dim3(CP_BLOCK), 0, s, freq_dev, num_rows, ctrl,
                           gt_before, eq_before, num_hot, (int)decay_shift, hot_rows_out_dev);
        EMB_RETURN_IF_LAUNCH_FAILED();
    } else if (decay_shift > 0) {
        hipLaunchKernelGGL(sel_age_kernel, dim3((unsigned)L.tiles), dim3(CP_BLOCK), 0, s, freq_dev, num_rows,
                           (int)decay_shift);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    if (info_out_dev && num_hot > 0) {
        hipLaunchKernelGGL(sel_info_kernel, dim3(1), dim3(CP_BLOCK), 0, s, ctrl, info_out_dev);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    return EMB_OK;
}

int select_check(const uint32_t *freq_dev, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                 const int64_t *hot_rows_out_dev)
{
    if (num_rows <= 0 || num_hot < 0 || num_hot > num_rows || decay_shift < 0 || decay_shift > 31)
        return EMB_ERR_INVALID_ARG;
    if (!freq_dev || !emb_aligned(freq_dev, 16) || (num_hot > 0 && !hot_rows_out_dev)) return EMB_ERR_INVALID_ARG;
    return EMB_OK;
}

}  // namespace

extern "C" int emb_cache_select(uint32_t *freq_dev, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                                void *workspace_dev, size_t workspace_bytes, int64_t *hot_rows_out_dev,
                                uint64_t *info_out_dev, void *stream)
{
    const int rc = select_check(freq_dev, num_rows, num_hot, decay_shift, hot_rows_out_dev);
    if (rc != EMB_OK) return rc;
    const SelLayout L = sel_layout(num_rows);
    if (L.tiles > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    if (!workspace_dev || !emb_aligned(workspace_dev, 256) || workspace_bytes < L.total) return EMB_ERR_WORKSPACE;
    return select_run(freq_dev, num_rows, num_hot, decay_shift, L, reinterpret_cast<char *>(workspace_dev),
                      hot_rows_out_dev, info_out_dev, emb_stream(stream));
}

// ---------------------------------------------------------------------------
// the selection for callers that cannot allocate
// ---------------------------------------------------------------------------
// The scratch memory of emb_cache_select_static: one array per device, part of the
// loaded code object, held until the process ends.  In host code the name `scratch`
// is only a handle for hipGetSymbolAddress: the device address it stands for on a
// given device is looked up once per device (sel_static_address) and that address,
// never the name, is what the kernels are given.
constexpr size_t SEL_STATIC_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[SEL_STATIC_BYTES];

namespace {

constexpr int SEL_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[SEL_MAX_DEVICES];   // by device ordinal; null until that device's first call

// Device address of `scratch` on the current device; null if the runtime refuses.
char *sel_static_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SEL_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = reinterpret_cast<char *>(p);
    }
    return g_scratch_ptr[dev];
}

}  // namespace

static_assert(EMB_CACHE_SELECT_STATIC_MAX_ROWS / SEL_TILE + 1 <= (SEL_STATIC_BYTES - 256 - 8 * SEL_PASSES * SEL_RADIX - 3 * 256) / 24,
              "the static scratch array holds the selection's tile tables up to the stated maximum");

extern "C" int emb_cache_select_static(uint32_t *freq_dev, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                                       int64_t *hot_rows_out_dev, uint64_t *info_out_dev, void *stream)
{
    const int rc = select_check(freq_dev, num_rows, num_hot, decay_shift, hot_rows_out_dev);
    if (rc != EMB_OK) return rc;
    if (num_rows > EMB_CACHE_SELECT_STATIC_MAX_ROWS) return EMB_ERR_UNSUPPORTED;   // beyond the scratch array
    const SelLayout L = sel_layout(num_rows);
    if (L.total > SEL_STATIC_BYTES) return EMB_ERR_UNSUPPORTED;
    char *ws = sel_static_address();
    if (!ws) return EMB_ERR_HIP;
    return select_run(freq_dev, num_rows, num_hot, decay_shift, L, ws, hot_rows_out_dev, info_out_dev,
                      emb_stream(stream));
}
