// Segment reduce of the scattered gradients fused with the row-wise Adagrad
// update, working directly on the sorted (key, bag) records.
//
// Mapping.  A table row of `chunks` 16-byte chunks is covered by a group of LPR
// lanes holding CPL chunks each, with CPL as large as 4: a 256-byte row takes 4
// lanes, so a wavefront works on 16 rows at a time.  The work per row that is
// not per element (finding the run, addresses, the Adagrad scalars) is then
// paid once per 16 rows of a wavefront instruction instead of once per 4; with
// 64-wide wavefronts on 16-lane SIMDs that instruction count, not HBM, was the
// limit of a 16-lanes-per-row mapping.
//
// Short runs.  Each lane group takes UPD_EPG consecutive sorted records and
// owns every run of equal keys that starts in that range.  It stages the keys
// and bags of its range and of the UPD_EPG records after it in LDS, derives
// bit masks of run heads, and then handles its runs one after the other: the
// row, its accumulator and the first gradient rows are requested together,
// the remaining gradient rows EU at a time, the sum is taken in ascending
// record order and Adagrad is applied once.  All groups of a wavefront go
// through the same loop, so the code is convergent.  A run that is not over
// after the look-ahead is not touched; its first record is written to the
// group's queue slot (one slot per group: only the last run of a range can
// overflow), so there are no atomics and no ordering effects.
//
// Queued runs.  A second kernel finds the end of every queued run (galloping
// then bisecting in the sorted keys), cuts it into LONG_CHUNK-record chunks and
// makes one task per chunk.  A third kernel gives each task to one wavefront,
// whose lane groups take the chunk's records round-robin and are then combined
// by a fixed butterfly; runs of several chunks store their chunk sums, and the
// wavefront that completes a run's last chunk adds them in chunk order and
// applies Adagrad.  All sums are taken in a fixed order: results are
// bit-identical from run to run.
#pragma once
#include "bwd_common.h"
#include "gather.h"
#include "scan.h"

// ---------------------------------------------------------------------------
// table directory: row bases, weight and accumulator pointers of the T tables,
// staged in LDS when T is small enough
// ---------------------------------------------------------------------------
struct TableDir {
    const emb_table *tables;
    const int64_t *s_base;
    char *const *s_w;
    float *const *s_a;
    bool staged;
    __device__ __forceinline__ int64_t base(int t) const
    {
        int64_t v;
        if (staged) v = s_base[t]; else v = tables[t].row_base;
        return v;
    }
    __device__ __forceinline__ char *weights(int t) const
    {
        char *v;
        if (staged) v = s_w[t]; else v = reinterpret_cast<char *>(tables[t].weights);
        return v;
    }
    __device__ __forceinline__ float *accum(int t) const
    {
        float *v;
        if (staged) v = s_a[t]; else v = tables[t].accum;
        return v;
    }
};

#define EMB_STAGE_TABLE_DIR(dir, tables, T, BLOCK)                              \
    __shared__ int64_t dir##_base[UPD_LDS_TABLES];                              \
    __shared__ char *dir##_w[UPD_LDS_TABLES];                                   \
    __shared__ float *dir##_a[UPD_LDS_TABLES];                                  \
    TableDir dir{tables, dir##_base, dir##_w, dir##_a, (T) <= UPD_LDS_TABLES};  \
    if (dir.staged) {                                                           \
        for (int t_ = threadIdx.x; t_ < (T); t_ += (BLOCK)) {                   \
            dir##_base[t_] = tables[t_].row_base;                               \
            dir##_w[t_] = reinterpret_cast<char *>(tables[t_].weights);         \
            dir##_a[t_] = tables[t_].accum;                                     \
        }                                                                       \
    }

// The table of bag number `bag` is bag / B.  With magic = floor((2^32-1)/B) the
// high word of bag*magic is the quotient or one less; one compare fixes it.
struct BagDiv {
    uint32_t B, magic;
    __device__ __forceinline__ int table(uint32_t bag) const
    {
        uint32_t q = __umulhi(bag, magic);
        if (bag - q * B >= B) ++q;
        return (int)q;
    }
};

// ---------------------------------------------------------------------------
// lane-group reductions with DPP (a DPP row is 16 lanes, a quad 4)
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
constexpr int DPP_QUAD_XOR1 = 0xB1;     // quad_perm:[1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;     // quad_perm:[2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7-i inside each 8
constexpr int DPP_ROW_MIRROR = 0x140;   // lane i <-> 15-i inside each 16

// Sum over the LPR lanes of a group (LPR a power of two); every lane gets it.
template <int LPR>
__device__ __forceinline__ float group_sum(float v)
{
    if (LPR >= 2) v += __uint_as_float(dpp_u32<DPP_QUAD_XOR1>(__float_as_uint(v)));
    if (LPR >= 4) v += __uint_as_float(dpp_u32<DPP_QUAD_XOR2>(__float_as_uint(v)));
    if (LPR >= 8) v += __uint_as_float(dpp_u32<DPP_HALF_MIRROR>(__float_as_uint(v)));
    if (LPR >= 16) v += __uint_as_float(dpp_u32<DPP_ROW_MIRROR>(__float_as_uint(v)));
    if (LPR >= 32) v += __shfl_xor(v, 16, EMB_WAVE);
    if (LPR >= 64) v += __shfl_xor(v, 32, EMB_WAVE);
    return v;
}

template <int LPR>
__device__ __forceinline__ uint32_t group_or(uint32_t v)
{
    if (LPR >= 2) v |= dpp_u32<DPP_QUAD_XOR1>(v);
    if (LPR >= 4) v |= dpp_u32<DPP_QUAD_XOR2>(v);
    if (LPR >= 8) v |= dpp_u32<DPP_HALF_MIRROR>(v);
    if (LPR >= 16) v |= dpp_u32<DPP_ROW_MIRROR>(v);
    if (LPR >= 32) v |= (uint32_t)__shfl_xor((int)v, 16, EMB_WAVE);
    if (LPR >= 64) v |= (uint32_t)__shfl_xor((int)v, 32, EMB_WAVE);
    return v;
}

// ---------------------------------------------------------------------------
// per-lane gradient slice and the Adagrad row update
// ---------------------------------------------------------------------------
// The fp32 gradient values that line up with a lane's 16-byte chunk of the
// table row: 4 for fp32 rows, 8 for bf16 rows.
template <bool BF16>
struct GradAcc {
    static constexpr int F = BF16 ? 8 : 4;
    static constexpr int V = BF16 ? 2 : 1;  // float4 loads per chunk
    float a[F];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < F; ++i) a[i] = 0.f;
    }
    __device__ __forceinline__ void fma(float s, const float4 (&v)[V])
    {
#pragma unroll
        for (int x = 0; x < V; ++x) {
            a[4 * x + 0] += s * v[x].x;
            a[4 * x + 1] += s * v[x].y;
            a[4 * x + 2] += s * v[x].z;
            a[4 * x + 3] += s * v[x].w;
        }
    }
};

template <bool BF16>
__device__ __forceinline__ void load_grad(const float *p, float4 (&v)[BF16 ? 2 : 1])
{
    const float4 *q = reinterpret_cast<const float4 *>(p);
    v[0] = q[0];
    if (BF16) v[BF16 ? 1 : 0] = q[1];
}

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// S_new = S_old + mean_d G^2 ; W -= lr * G / (sqrt(S_new) + eps), for the row
// whose chunks `w` were loaded from `wrow`.  Called by all LPR lanes of a group.
// The scalar part uses the hardware square root and reciprocal (about 1 ulp
// each); the per-element part is one multiply and one subtract.
template <int LPR, int CPL, bool BF16>
__device__ __forceinline__ void adagrad_apply(const GradAcc<BF16> (&acc)[CPL], uint4 (&w)[CPL], float s_old,
                                              char *wrow, float *aptr, int l, int32_t chunks_per_row, float inv_D,
                                              float lr, float eps)
{
    constexpr int F = GradAcc<BF16>::F;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < F; ++i) sq += acc[c].a[i] * acc[c].a[i];  // lanes past the row hold zeros
    sq = group_sum<LPR>(sq);
    const float s_new = s_old + sq * inv_D;
    const float step = lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(s_new) + eps);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = l + c * LPR;
        if (chunk < chunks_per_row) {
            uint4 x = w[c];
            if (BF16) {
                uint32_t *wp = &x.x;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = __uint_as_float(wp[i] << 16) - step * acc[c].a[2 * i];
                    const float hi = __uint_as_float(wp[i] & 0xFFFF0000u) - step * acc[c].a[2 * i + 1];
                    wp[i] = bf16_rne(lo) | (bf16_rne(hi) << 16);
                }
            } else {
                x.x = __float_as_uint(__uint_as_float(x.x) - step * acc[c].a[0]);
                x.y = __float_as_uint(__uint_as_float(x.y) - step * acc[c].a[1]);
                x.z = __float_as_uint(__uint_as_float(x.z) - step * acc[c].a[2]);
                x.w = __float_as_uint(__uint_as_float(x.w) - step * acc[c].a[3]);
            }
            *reinterpret_cast<uint4 *>(wrow + (int64_t)chunk * 16) = x;
        }
    }
    if (l == 0) *aptr = s_new;
}

// NB consecutive records starting at an address aligned to their total size.
template <typename E, int NB>
__device__ __forceinline__ void load_records(const E *__restrict__ p, E (&out)[NB])
{
    constexpr int BYTES = NB * (int)sizeof(E);
    if constexpr (BYTES >= 16) {
        const uint4 *q = reinterpret_cast<const uint4 *>(p);
        uint4 tmp[BYTES / 16];
#pragma unroll
        for (int i = 0; i < BYTES / 16; ++i) tmp[i] = q[i];
        const E *t = reinterpret_cast<const E *>(tmp);
#pragma unroll
        for (int i = 0; i < NB; ++i) out[i] = t[i];
    } else {
#pragma unroll
        for (int i = 0; i < NB; ++i) out[i] = p[i];
    }
}

// ---------------------------------------------------------------------------
// short runs: one lane group per range of UPD_EPG sorted records
// ---------------------------------------------------------------------------
template <typename KeyT, int LPR, int CPL, int EU, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void update_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                           const KeyT *__restrict__ keys,
                                                           const uint32_t *__restrict__ pay, uint32_t n,
                                                           KeyT sentinel, const float *__restrict__ bag_scale,
                                                           const float *__restrict__ dout, int32_t chunks_per_row,
                                                           int32_t D, float inv_D, float lr, float eps, BagDiv bdiv,
                                                           const BwdCtrl *ctrl, uint32_t *__restrict__ queue,
                                                           uint32_t *__restrict__ wave_heads)
{
    if (ctrl->abort) return;
    constexpr int GROUPS = UPD_BLOCK / LPR;
    constexpr int WIN = 2 * UPD_EPG;                      // records staged per group
    constexpr int STAGERS = LPR < WIN ? LPR : WIN;        // lanes of a group that stage records
    constexpr int PER = WIN / STAGERS;                    // records staged per such lane
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    static_assert(WIN == 32, "head masks are 32 bits wide");
    EMB_STAGE_TABLE_DIR(dir, tables, T, UPD_BLOCK)
    __shared__ KeyT lk[GROUPS][WIN + 2];  // [0] = record before the range, [1 + e] = record e, [WIN + 1] = the one after
    __shared__ uint32_t lp[GROUPS][WIN];

    const int g = threadIdx.x / LPR;
    const int l = threadIdx.x % LPR;
    const uint64_t gid = (uint64_t)blockIdx.x * GROUPS + g;
    const uint64_t first = gid * UPD_EPG;
    const bool in = first < n;
    const uint32_t i0 = (uint32_t)first;

    // ---- stage this group's records (the arrays carry SORT_PAD records of slack)
    if (in && l < STAGERS) {
        KeyT k[PER];
        uint32_t b[PER];
        load_records<KeyT, PER>(keys + i0 + l * PER, k);
        load_records<uint32_t, PER>(pay + i0 + l * PER, b);
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const bool live = i0 + l * PER + e < n;
            lk[g][1 + l * PER + e] = live ? k[e] : sentinel;
            lp[g][l * PER + e] = live ? b[e] : 0u;
        }
        if (l == 0) {
            lk[g][0] = i0 > 0 ? keys[i0 - 1] : sentinel;
            lk[g][WIN + 1] = (n - i0 > (uint32_t)WIN) ? keys[i0 + WIN] : sentinel;
        }
    }
    __syncthreads();

    uint32_t heads = 0;
    if (in) {
        // ---- which records are valid (not the sentinel) and which start a run
        uint32_t valid = 0, head = 0;
        if (l < STAGERS) {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int idx = l * PER + e;
                const KeyT k = lk[g][1 + idx];
                const bool v = k != sentinel;
                valid |= (v ? 1u : 0u) << idx;
                head |= ((v && k != lk[g][idx]) ? 1u : 0u) << idx;   // record 0 of the whole array: lk[0] is the sentinel
            }
        }
        valid = group_or<LPR>(valid);
        head = group_or<LPR>(head);
        const uint32_t stop = head | ~valid;                 // a run ends before the next head or invalid record
        uint32_t todo = head & ((1u << UPD_EPG) - 1u);       // runs that start inside the range are ours
        uint32_t queued = 0xFFFFFFFFu;
        const int64_t row_bytes = (int64_t)chunks_per_row * 16;

        while (todo) {
            const int pos = __ffs((int)todo) - 1;
            todo &= todo - 1;
            ++heads;
            const uint32_t later = pos == 31 ? 0u : (stop >> (pos + 1)) << (pos + 1);
            const int end = later ? __ffs((int)later) - 1 : WIN;
            const KeyT key = lk[g][1 + pos];
            if (end == WIN && lk[g][WIN + 1] == key) {        // not over after the look-ahead: someone else's job
                queued = i0 + (uint32_t)pos;
                break;
            }
            // ---- the row, its accumulator and the first EU gradient rows, all requested together
            const int t = bdiv.table(lp[g][pos]);
            const int64_t r = (int64_t)key - dir.base(t);
            char *wrow = dir.weights(t) + r * row_bytes;
            float *aptr = dir.accum(t) + r;
            uint4 w[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int chunk = l + c * LPR;
                w[c] = make_uint4(0, 0, 0, 0);
                if (chunk < chunks_per_row) w[c] = load_chunk(wrow + (int64_t)chunk * 16);
            }
            const float s_old = *aptr;
            GradAcc<BF16> acc[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c].zero();
            for (int e0 = pos; e0 < end; e0 += EU) {
                float4 gr[EU][CPL][V];
                float sc[EU];
#pragma unroll
                for (int u = 0; u < EU; ++u) {
                    const int e = e0 + u;
                    sc[u] = 0.f;
#pragma unroll
                    for (int c = 0; c < CPL; ++c)
#pragma unroll
                        for (int x = 0; x < V; ++x) gr[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (e < end) {
                        const uint32_t bag = lp[g][e];
                        sc[u] = bag_scale[bag];
                        const float *grow = dout + (int64_t)bag * D;
#pragma unroll
                        for (int c = 0; c < CPL; ++c) {
                            const int chunk = l + c * LPR;
                            if (chunk < chunks_per_row) load_grad<BF16>(grow + (int64_t)chunk * F, gr[u][c]);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < EU; ++u)
#pragma unroll
                    for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], gr[u][c]);
            }
            adagrad_apply<LPR, CPL, BF16>(acc, w, s_old, wrow, aptr, l, chunks_per_row, inv_D, lr, eps);
        }
        if (l == 0) queue[gid] = queued;
    }

    // number of runs started = number of distinct rows; one store per wavefront
    uint32_t h = (l == 0) ? heads : 0u;
#pragma unroll
    for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) h += __shfl_xor(h, d, EMB_WAVE);
    if ((threadIdx.x & (EMB_WAVE - 1)) == 0)
        wave_heads[(uint64_t)blockIdx.x * (UPD_BLOCK / EMB_WAVE) + threadIdx.x / EMB_WAVE] = h;
}

// ---------------------------------------------------------------------------
// queued runs
// ---------------------------------------------------------------------------
// One thread per queue slot: find the run's end, cut it into chunks, create the
// tasks.  Also adds up the per-wavefront run counts of the short-run kernel.
template <typename KeyT>
__global__ __launch_bounds__(256) void long_prepare_kernel(const KeyT *__restrict__ keys, uint32_t n, BwdCtrl *ctrl,
                                                           const uint32_t *__restrict__ queue, uint32_t slots,
                                                           const uint32_t *__restrict__ wave_heads,
                                                           uint32_t n_wave_heads, LongSeg *__restrict__ segs,
                                                           uint32_t *__restrict__ seg_done,
                                                           uint2 *__restrict__ chunk_tasks, uint32_t chunk_cap,
                                                           uint32_t partial_cap)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[256 / EMB_WAVE];
    const uint32_t s = blockIdx.x * 256 + threadIdx.x;

    // distinct rows: sum of the run counts
    {
        uint32_t h = s < n_wave_heads ? wave_heads[s] : 0u, total;
        block_inclusive_scan<uint32_t, 256>(h, wave_sums, total);
        if (threadIdx.x == 0 && total) atomicAdd(&ctrl->num_unique, total);
    }

    uint32_t lo = 0xFFFFFFFFu;
    if (s < slots) lo = queue[s];
    uint32_t hi = 0, chunks = 0;
    if (lo != 0xFFFFFFFFu) {
        const KeyT key = keys[lo];
        // gallop: the run is at least UPD_EPG + 1 records long
        uint32_t step = UPD_EPG;
        uint32_t a = lo + 1, b = n;                 // the first record whose key differs lies in [a, b]
        for (;;) {
            const uint32_t probe = lo + step;
            if (probe >= n) break;
            if (keys[probe] == key) {
                a = probe + 1;
                if (step >= 0x40000000u) break;
                step <<= 1;
            } else {
                b = probe;
                break;
            }
        }
        while (a < b) {
            const uint32_t mid = a + ((b - a) >> 1);
            if (keys[mid] == key) a = mid + 1; else b = mid;
        }
        hi = a;
        chunks = (hi - lo + LONG_CHUNK - 1) / LONG_CHUNK;
    }
    // task slots: an exclusive scan inside the workgroup, one atomic per workgroup
    uint32_t total_chunks, total_part;
    const uint32_t inc_c = block_inclusive_scan<uint32_t, 256>(chunks, wave_sums, total_chunks);
    const uint32_t part = chunks > 1 ? chunks : 0u;   // chunk sums are stored only for runs of several chunks
    const uint32_t inc_p = block_inclusive_scan<uint32_t, 256>(part, wave_sums, total_part);
    __shared__ uint32_t s_base_c, s_base_p;
    if (threadIdx.x == 0) {
        s_base_c = total_chunks ? atomicAdd(&ctrl->chunk_count, total_chunks) : 0u;
        s_base_p = total_part ? atomicAdd(&ctrl->partial_count, total_part) : 0u;
    }
    __syncthreads();
    if (chunks) {
        const uint32_t cbase = s_base_c + inc_c - chunks;
        const uint32_t pbase = s_base_p + inc_p - part;
        LongSeg sg;
        sg.lo = lo;
        sg.hi = hi;
        sg.chunk_base = pbase;
        // the caps cannot be exceeded (see the workspace layout); the check only guards memory
        sg.n_chunks = (cbase + chunks <= chunk_cap && pbase + part <= partial_cap) ? chunks : 0u;
        segs[s] = sg;
        seg_done[s] = 0;
        for (uint32_t c = 0; c < sg.n_chunks; ++c) chunk_tasks[cbase + c] = make_uint2(s, c);
    }
}

// One wavefront per chunk task.
template <typename KeyT, int LPR, int CPL, int EU, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void long_reduce_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                const KeyT *__restrict__ keys,
                                                                const uint32_t *__restrict__ pay,
                                                                const float *__restrict__ bag_scale,
                                                                const float *__restrict__ dout,
                                                                int32_t chunks_per_row, int32_t D, float inv_D,
                                                                float lr, float eps, BagDiv bdiv, BwdCtrl *ctrl,
                                                                const LongSeg *__restrict__ segs,
                                                                uint32_t *__restrict__ seg_done,
                                                                const uint2 *__restrict__ chunk_tasks,
                                                                uint32_t chunk_cap, float *__restrict__ partials,
                                                                int64_t *num_unique_out)
{
    if (ctrl->abort) return;
    if (blockIdx.x == 0 && threadIdx.x == 0 && num_unique_out) *num_unique_out = (int64_t)ctrl->num_unique;
    EMB_STAGE_TABLE_DIR(dir, tables, T, UPD_BLOCK)
    __syncthreads();
    constexpr int GPW = EMB_WAVE / LPR;  // lane groups per wavefront
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int l = lane % LPR;
    const int g = lane / LPR;
    const int64_t row_floats = (int64_t)chunks_per_row * F;
    uint32_t tasks = ctrl->chunk_count;
    if (tasks > chunk_cap) tasks = chunk_cap;
    const uint32_t waves = gridDim.x * (UPD_BLOCK / EMB_WAVE);

    for (uint32_t task = blockIdx.x * (UPD_BLOCK / EMB_WAVE) + threadIdx.x / EMB_WAVE; task < tasks; task += waves) {
        const uint2 tk = chunk_tasks[task];
        const LongSeg sg = segs[tk.x];
        const uint32_t lo = sg.lo + tk.y * LONG_CHUNK;
        const uint32_t hi = (sg.hi - lo > (uint32_t)LONG_CHUNK) ? lo + LONG_CHUNK : sg.hi;

        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        for (uint32_t i0 = lo + g; i0 < hi; i0 += GPW * EU) {
            float4 v[EU][CPL][V];
            float sc[EU];
#pragma unroll
            for (int u = 0; u < EU; ++u) {
                const uint32_t i = i0 + u * GPW;
                sc[u] = 0.f;
#pragma unroll
                for (int c = 0; c < CPL; ++c)
#pragma unroll
                    for (int x = 0; x < V; ++x) v[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i < hi) {
                    const uint32_t bag = pay[i];
                    sc[u] = bag_scale[bag];
                    const float *grow = dout + (int64_t)bag * D;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int chunk = l + c * LPR;
                        if (chunk < chunks_per_row) load_grad<BF16>(grow + (int64_t)chunk * F, v[u][c]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < EU; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], v[u][c]);
        }
        // butterfly over the lane groups of the wavefront: every group ends with the chunk sum
#pragma unroll
        for (int d = LPR; d < EMB_WAVE; d <<= 1)
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int i = 0; i < F; ++i) acc[c].a[i] += __shfl_xor(acc[c].a[i], d, EMB_WAVE);

        bool finish = sg.n_chunks == 1;
        if (sg.n_chunks > 1) {
            // publish this chunk's sum, then find out whether it was the run's last outstanding one
            if (g == 0) {
                float *slot = partials + (int64_t)(sg.chunk_base + tk.y) * row_floats;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int chunk = l + c * LPR;
                    if (chunk < chunks_per_row) {
#pragma unroll
                        for (int i = 0; i < F; ++i)
                            __hip_atomic_store(slot + (int64_t)chunk * F + i, acc[c].a[i], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            __threadfence();
            uint32_t ticket = 0;
            if (lane == 0) ticket = atomicAdd(&seg_done[tk.x], 1u);
            ticket = (uint32_t)__shfl((int)ticket, 0, EMB_WAVE);
            finish = ticket == sg.n_chunks - 1;
            if (finish) {
                __threadfence();
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c].zero();
                for (uint32_t cc = 0; cc < sg.n_chunks; ++cc) {
                    const float *slot = partials + (int64_t)(sg.chunk_base + cc) * row_floats;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int chunk = l + c * LPR;
                        if (chunk < chunks_per_row) {
#pragma unroll
                            for (int i = 0; i < F; ++i)
                                acc[c].a[i] += __hip_atomic_load(slot + (int64_t)chunk * F + i, __ATOMIC_RELAXED,
                                                                 __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
        }
        if (finish && g == 0) {
            const int64_t key = (int64_t)keys[sg.lo];
            const int t = bdiv.table(pay[sg.lo]);
            const int64_t r = key - dir.base(t);
            char *wrow = dir.weights(t) + r * ((int64_t)chunks_per_row * 16);
            float *aptr = dir.accum(t) + r;
            uint4 w[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int chunk = l + c * LPR;
                w[c] = make_uint4(0, 0, 0, 0);
                if (chunk < chunks_per_row) w[c] = load_chunk(wrow + (int64_t)chunk * 16);
            }
            adagrad_apply<LPR, CPL, BF16>(acc, w, *aptr, wrow, aptr, l, chunks_per_row, inv_D, lr, eps);
        }
    }
}
