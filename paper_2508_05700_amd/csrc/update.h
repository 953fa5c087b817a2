// Segment reduce of the scattered gradients fused with the row-wise Adagrad
// update, working directly on the sorted (key, bag) records.
//
// A lane group (the LPR lanes that cover one table row) takes a fixed range of
// UPD_EPG consecutive sorted records and owns every run of equal keys whose
// first record lies in its range: it skips leading records that continue a run
// owned by an earlier range, and follows its last run past the end of the range.
// Runs are found on the fly by comparing neighbouring keys, so this stage needs
// no segment table.  Records are taken NB at a time: first the keys and bags of
// the batch, then - all issued together - the NB gradient-row chunks and, for
// records that start a run, the table-row chunk and accumulator; only then the
// batch is walked in order, adding gradients and applying Adagrad where a run
// ends.  Loads of one batch are independent of each other, so a group keeps up
// to 2*NB row reads in flight regardless of how short the runs are.
//
// A run that grows past LONG_SEGMENT records is abandoned (nothing was written)
// and queued; queued runs are cut into LONG_CHUNK-record chunks that whole
// workgroups sum, the workgroup that finishes last combining the chunk sums in
// chunk order.  All sums are taken in a fixed order: results are bit-identical
// from run to run.
#pragma once
#include "bwd_common.h"
#include "gather.h"

// ---------------------------------------------------------------------------
// table directory: row bases, weight and accumulator pointers of the T tables,
// staged in LDS when T is small enough
// ---------------------------------------------------------------------------
struct TableDir {
    const emb_table *tables;
    const int64_t *s_base;
    char *const *s_w;
    float *const *s_a;
    int32_t T;
    bool staged;
    __device__ __forceinline__ int64_t base(int t) const { return staged ? s_base[t] : tables[t].row_base; }
    __device__ __forceinline__ char *weights(int t) const
    {
        return staged ? s_w[t] : reinterpret_cast<char *>(tables[t].weights);
    }
    __device__ __forceinline__ float *accum(int t) const { return staged ? s_a[t] : tables[t].accum; }
    // the last table whose row_base is <= key
    __device__ __forceinline__ int find(int64_t key) const
    {
        int lo = 0, hi = T;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (base(mid) <= key) lo = mid; else hi = mid;
        }
        return lo;
    }
};

#define EMB_STAGE_TABLE_DIR(dir, tables, T, BLOCK)                                  \
    __shared__ int64_t dir##_base[UPD_LDS_TABLES];                                  \
    __shared__ char *dir##_w[UPD_LDS_TABLES];                                       \
    __shared__ float *dir##_a[UPD_LDS_TABLES];                                      \
    TableDir dir{tables, dir##_base, dir##_w, dir##_a, T, (T) <= UPD_LDS_TABLES};   \
    if (dir.staged) {                                                               \
        for (int t_ = threadIdx.x; t_ < (T); t_ += (BLOCK)) {                       \
            dir##_base[t_] = tables[t_].row_base;                                   \
            dir##_w[t_] = reinterpret_cast<char *>(tables[t_].weights);             \
            dir##_a[t_] = tables[t_].accum;                                         \
        }                                                                           \
        __syncthreads();                                                            \
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
template <int LPR, int CPL, bool BF16>
__device__ __forceinline__ void adagrad_apply(const GradAcc<BF16> (&acc)[CPL], uint4 (&w)[CPL], float s_old,
                                              char *wrow, float *aptr, int l, int32_t chunks_per_row, int32_t D,
                                              float lr, float eps)
{
    constexpr int F = GradAcc<BF16>::F;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < F; ++i) sq += acc[c].a[i] * acc[c].a[i];  // lanes past the row hold zeros
#pragma unroll
    for (int d = LPR >> 1; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, LPR);
    const float s_new = s_old + sq / (float)D;
    const float denom = sqrtf(s_new) + eps;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = l + c * LPR;
        if (chunk < chunks_per_row) {
            uint4 x = w[c];
            if (BF16) {
                uint32_t *wp = &x.x;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float lo = __uint_as_float(wp[i] << 16);
                    float hi = __uint_as_float(wp[i] & 0xFFFF0000u);
                    lo -= lr * acc[c].a[2 * i] / denom;
                    hi -= lr * acc[c].a[2 * i + 1] / denom;
                    wp[i] = bf16_rne(lo) | (bf16_rne(hi) << 16);
                }
            } else {
                x.x = __float_as_uint(__uint_as_float(x.x) - lr * acc[c].a[0] / denom);
                x.y = __float_as_uint(__uint_as_float(x.y) - lr * acc[c].a[1] / denom);
                x.z = __float_as_uint(__uint_as_float(x.z) - lr * acc[c].a[2] / denom);
                x.w = __float_as_uint(__uint_as_float(x.w) - lr * acc[c].a[3] / denom);
            }
            *reinterpret_cast<uint4 *>(wrow + (int64_t)chunk * 16) = x;
        }
    }
    if (l == 0) *aptr = s_new;
}

// NB consecutive records starting at a multiple of NB, as vector loads.
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
// main update: one lane group per range of UPD_EPG sorted records
// ---------------------------------------------------------------------------
template <typename KeyT, int LPR, int CPL, int NB, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void update_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                           const KeyT *__restrict__ keys,
                                                           const uint32_t *__restrict__ pay, uint32_t n,
                                                           KeyT sentinel, const float *__restrict__ bag_scale,
                                                           const float *__restrict__ dout, int32_t chunks_per_row,
                                                           int32_t D, float lr, float eps, BwdCtrl *ctrl,
                                                           uint32_t *__restrict__ long_list, uint32_t long_cap)
{
    static_assert(UPD_EPG % NB == 0, "a range is whole batches");
    if (ctrl->abort) return;
    EMB_STAGE_TABLE_DIR(dir, tables, T, UPD_BLOCK)
    constexpr int GROUPS = UPD_BLOCK / LPR;
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    const int l = threadIdx.x % LPR;
    const uint64_t first = ((uint64_t)blockIdx.x * GROUPS + threadIdx.x / LPR) * UPD_EPG;
    const int64_t row_bytes = (int64_t)chunks_per_row * 16;
    uint32_t heads = 0;

    if (first < n) {
        const uint32_t i0 = (uint32_t)first;
        const uint32_t i1 = (n - i0 > (uint32_t)UPD_EPG) ? i0 + UPD_EPG : n;
        bool active = false, done = false;
        uint32_t seg_lo = 0, count = 0;
        GradAcc<BF16> acc[CPL];
        uint4 wcur[CPL];
        float s_old = 0.f;
        char *wrow = nullptr;
        float *aptr = nullptr;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            acc[c].zero();
            wcur[c] = make_uint4(0, 0, 0, 0);
        }

        for (uint32_t p = i0; !done && (p < i1 || active); p += NB) {
            // ---- the batch's keys (with one neighbour on either side) and bags
            KeyT k[NB];
            uint32_t bag[NB];
            load_records<KeyT, NB>(keys + p, k);       // arrays carry SORT_PAD records of slack
            load_records<uint32_t, NB>(pay + p, bag);
            const KeyT kprev = p > 0 ? keys[p - 1] : sentinel;
            const KeyT knext = keys[p + NB];

            // ---- which records this group adds, which start a run, which end one
            uint32_t need = 0, head = 0, tail = 0;
            {
                bool a = active, dn = false;
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const uint32_t i = p + u;
                    const bool valid = i < n && k[u] != sentinel;
                    const KeyT before = u == 0 ? kprev : k[u - 1];
                    const KeyT after = u == NB - 1 ? knext : k[u + 1];
                    const bool is_head = valid && (i == 0 || k[u] != before);
                    const bool is_tail = valid && (i + 1 >= n || after != k[u]);
                    if (!valid) dn = true;                 // the sentinel records sort last
                    if (!dn && is_head) {
                        if (i >= i1) dn = true;            // a run that starts past the range is not ours
                        else a = true;
                    }
                    const bool nd = !dn && a;
                    need |= (nd ? 1u : 0u) << u;
                    head |= ((nd && is_head) ? 1u : 0u) << u;
                    tail |= ((nd && is_tail) ? 1u : 0u) << u;
                    if (nd && is_tail) a = false;
                }
                done = dn;
            }

            // ---- issue every load of the batch before using any of them
            float4 g[NB][CPL][V];
            float sc[NB];
            uint4 wv[NB][CPL];
            float sv[NB];
            int tt[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                sc[u] = 0.f;
                sv[u] = 0.f;
                tt[u] = 0;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    wv[u][c] = make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int x = 0; x < V; ++x) g[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
                if ((need >> u) & 1u) {
                    sc[u] = bag_scale[bag[u]];
                    const float *grow = dout + (int64_t)bag[u] * D;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int chunk = l + c * LPR;
                        if (chunk < chunks_per_row) load_grad<BF16>(grow + (int64_t)chunk * F, g[u][c]);
                    }
                }
                if ((head >> u) & 1u) {
                    const int64_t key = (int64_t)k[u];
                    const int t = dir.find(key);
                    tt[u] = t;
                    const int64_t r = key - dir.base(t);
                    sv[u] = dir.accum(t)[r];
                    const char *wr = dir.weights(t) + r * row_bytes;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int chunk = l + c * LPR;
                        if (chunk < chunks_per_row) wv[u][c] = load_chunk(wr + (int64_t)chunk * 16);
                    }
                }
            }

            // ---- walk the batch in order
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                if ((head >> u) & 1u) {
                    const int64_t key = (int64_t)k[u];
                    const int64_t r = key - dir.base(tt[u]);
                    wrow = dir.weights(tt[u]) + r * row_bytes;
                    aptr = dir.accum(tt[u]) + r;
                    s_old = sv[u];
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        wcur[c] = wv[u][c];
                        acc[c].zero();
                    }
                    seg_lo = p + u;
                    count = 0;
                    ++heads;
                }
                if ((need >> u) & 1u) {
#pragma unroll
                    for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], g[u][c]);
                    ++count;
                }
                if ((tail >> u) & 1u)
                    adagrad_apply<LPR, CPL, BF16>(acc, wcur, s_old, wrow, aptr, l, chunks_per_row, D, lr, eps);
            }
            // the run still open after the batch, if any
            active = false;
            if (need) {
                const int last = 31 - __clz(need);
                active = !((tail >> last) & 1u);
            }
            if (active && count > (uint32_t)LONG_SEGMENT) {
                if (l == 0) {
                    const uint32_t slot = atomicAdd(&ctrl->long_count, 1u);
                    if (slot < long_cap) long_list[slot] = seg_lo;  // cannot overflow: long_cap > n / LONG_SEGMENT
                }
                active = false;
                done = true;
            }
        }
    }

    // number of runs started = number of distinct rows; one atomic per wavefront
    uint32_t h = (l == 0) ? heads : 0u;
#pragma unroll
    for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) h += __shfl_xor(h, d, EMB_WAVE);
    if ((threadIdx.x & (EMB_WAVE - 1)) == 0 && h) atomicAdd(&ctrl->num_unique, h);
}

// ---------------------------------------------------------------------------
// long runs
// ---------------------------------------------------------------------------
// One thread per queued run: find its end, cut it into chunks, create the tasks.
template <typename KeyT>
__global__ __launch_bounds__(256) void long_prepare_kernel(const KeyT *__restrict__ keys, uint32_t n, BwdCtrl *ctrl,
                                                           const uint32_t *__restrict__ long_list, uint32_t long_cap,
                                                           LongSeg *__restrict__ segs, uint32_t *__restrict__ seg_done,
                                                           uint2 *__restrict__ chunk_tasks, uint32_t chunk_cap)
{
    if (ctrl->abort) return;
    uint32_t count = ctrl->long_count;
    if (count > long_cap) count = long_cap;
    const uint32_t s = blockIdx.x * 256 + threadIdx.x;
    if (s >= count) return;
    const uint32_t lo = long_list[s];
    const KeyT key = keys[lo];
    uint32_t a = lo + 1, b = n;  // first record after lo whose key differs lies in [a, b]
    while (a < b) {
        const uint32_t mid = a + ((b - a) >> 1);
        if (keys[mid] == key) a = mid + 1; else b = mid;
    }
    const uint32_t hi = a;
    const uint32_t chunks = (hi - lo + LONG_CHUNK - 1) / LONG_CHUNK;
    const uint32_t base = atomicAdd(&ctrl->chunk_count, chunks);
    LongSeg sg;
    sg.lo = lo;
    sg.hi = hi;
    sg.chunk_base = base;
    sg.n_chunks = (base + chunks <= chunk_cap) ? chunks : 0u;  // cannot overflow; guards memory anyway
    segs[s] = sg;
    seg_done[s] = 0;
    for (uint32_t c = 0; c < sg.n_chunks; ++c) chunk_tasks[base + c] = make_uint2(s, c);
}

// A workgroup sums one chunk: its LBLOCK/LPR lane groups take the chunk's
// records round-robin, then a fixed binary tree in LDS combines them.  The
// workgroup that completes a run's last outstanding chunk adds the chunk sums
// in chunk order and applies Adagrad.
template <typename KeyT, int LPR, int CPL, int UNROLL, bool BF16, int LBLOCK>
__global__ __launch_bounds__(LBLOCK) void long_reduce_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                             const KeyT *__restrict__ keys,
                                                             const uint32_t *__restrict__ pay,
                                                             const float *__restrict__ bag_scale,
                                                             const float *__restrict__ dout, int32_t chunks_per_row,
                                                             int32_t D, float lr, float eps, BwdCtrl *ctrl,
                                                             const LongSeg *__restrict__ segs,
                                                             uint32_t *__restrict__ seg_done,
                                                             const uint2 *__restrict__ chunk_tasks,
                                                             uint32_t chunk_cap, float *__restrict__ partials,
                                                             int64_t *num_unique_out)
{
    if (ctrl->abort) return;
    if (blockIdx.x == 0 && threadIdx.x == 0 && num_unique_out) *num_unique_out = (int64_t)ctrl->num_unique;
    EMB_STAGE_TABLE_DIR(dir, tables, T, LBLOCK)
    constexpr int GROUPS = LBLOCK / LPR;
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    __shared__ float part[LBLOCK * F];  // [GROUPS][LPR][F]
    __shared__ uint32_t s_ticket;
    const int l = threadIdx.x % LPR;
    const int g = threadIdx.x / LPR;
    const int64_t row_floats = (int64_t)chunks_per_row * F;
    uint32_t tasks = ctrl->chunk_count;
    if (tasks > chunk_cap) tasks = chunk_cap;

    for (uint32_t task = blockIdx.x; task < tasks; task += gridDim.x) {
        const uint2 tk = chunk_tasks[task];
        const LongSeg sg = segs[tk.x];
        const uint32_t lo = sg.lo + tk.y * LONG_CHUNK;
        const uint32_t hi = (sg.hi - lo > (uint32_t)LONG_CHUNK) ? lo + LONG_CHUNK : sg.hi;

        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        for (uint32_t i0 = lo + g; i0 < hi; i0 += GROUPS * UNROLL) {
            float4 v[UNROLL][CPL][V];
            float sc[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = i0 + u * GROUPS;
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
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], v[u][c]);
        }

        // tree over the lane groups, one chunk column at a time
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            float *mine = part + ((size_t)g * LPR + l) * F;
#pragma unroll
            for (int i = 0; i < F; ++i) mine[i] = acc[c].a[i];
            __syncthreads();
            for (int half = GROUPS >> 1; half >= 1; half >>= 1) {
                if (g < half) {
                    const float *other = part + ((size_t)(g + half) * LPR + l) * F;
#pragma unroll
                    for (int i = 0; i < F; ++i) mine[i] += other[i];
                }
                __syncthreads();
            }
            if (g == 0) {
#pragma unroll
                for (int i = 0; i < F; ++i) acc[c].a[i] = mine[i];
            }
            __syncthreads();
        }

        bool finish = sg.n_chunks == 1;
        if (sg.n_chunks > 1) {
            // publish this chunk's sum, then find out whether it was the last one
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
            __syncthreads();
            if (threadIdx.x == 0) s_ticket = atomicAdd(&seg_done[tk.x], 1u);
            __syncthreads();
            finish = s_ticket == sg.n_chunks - 1;
            if (finish && g == 0) {
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
            __syncthreads();  // s_ticket is reused by the next task
        }
        if (finish && g == 0) {
            const int64_t key = (int64_t)keys[sg.lo];
            const int t = dir.find(key);
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
            adagrad_apply<LPR, CPL, BF16>(acc, w, *aptr, wrow, aptr, l, chunks_per_row, D, lr, eps);
        }
    }
}
