// Segment reduce of the scattered gradients fused with the row-wise Adagrad
// update, working directly on the sorted (key, bag) records.
//
// Mapping.  A table row of `chunks` 16-byte chunks is covered by a group of LPR
// lanes holding CPL chunks each, normally CPL = 2: a 256-byte row takes 8 lanes,
// so a wavefront works on 8 rows at a time.  The work per row that is not per
// element (finding the run, addresses, the Adagrad scalars) is then paid once
// per 8 rows of a wavefront instruction; with 64-wide wavefronts on 16-lane
// SIMDs that instruction count, not HBM, was the limit of a 16-lanes-per-row
// mapping with per-lane-group control flow.  (4 lanes x 4 chunks halves the
// instruction count again but costs registers and occupancy; measured slower.)
//
// Short runs.  Each wavefront takes UPD_SPAN consecutive sorted records and
// owns every run of equal keys that starts in that span.  It stages the keys
// and bags of the span and of UPD_LOOK records after it in LDS, compacts the
// positions where the key changes into a list of runs, and deals the runs to
// its lane groups round-robin, so every group has the same number of runs to
// do.  For a run the row, its accumulator and the first gradient rows are
// requested together, the remaining gradient rows EU at a
// time; the sum is taken in ascending record order and Adagrad is applied
// once.  All groups go through the same loop, so the code is convergent.  A
// run longer than UPD_SHORT_MAX records, or not over after the look-ahead, is
// not touched; its first record goes to one of the wavefront's UPD_QSLOTS queue
// slots (no more such runs can start in one span).  Which slot is a matter of
// timing, but queued runs are independent of each other, so values are not.
//
// Queued runs.  The kernel that queues them also notes where runs start; a second
// kernel takes the end of every queued run from those notes (the next run start in
// its span, else the first run start of the spans after it), cuts it into
// LONG_CHUNK-record chunks and makes one task per chunk.  A third kernel gives each task to one wavefront,
// whose lane groups take the chunk's records round-robin and are then combined
// by a fixed butterfly; a run of one chunk is finished there, runs of several
// chunks store their chunk sums and a last small kernel, one wavefront per run,
// adds them in a fixed order and applies Adagrad.  (The kernel boundary is what makes the chunk sums
// visible: a device-wide fence inside a kernel writes back the whole L2 of the
// issuing XCD, dirty table rows included, and was far more expensive.)  All
// sums are taken in a fixed order: results are bit-identical from run to run.
#pragma once
#include "bwd_common.h"
#include "gather.h"
#include "scan.h"

// ---------------------------------------------------------------------------
// table directory: row bases, weight and accumulator pointers of the T tables,
// staged in LDS when T is small enough
// ---------------------------------------------------------------------------
// The staged copies are addressed as LDS (address space 3), the descriptors as device memory: a
// generic pointer that may be either would turn every access into a flat operation, whose wait also
// waits for the row stores of the run before.
typedef char *emb_char_ptr;
typedef float *emb_float_ptr;
#define EMB_LDS __attribute__((address_space(3)))
// ALWAYS_LDS: the caller knows at compile time that the directory is staged (T <= UPD_LDS_TABLES), so
// the accessors are plain LDS reads with no device-memory arm beside them (whose presence makes the
// compiler wait for every outstanding memory operation, the stores of the run before included, where
// the two arms join).
template <bool ALWAYS_LDS>
struct TableDirT {
    const emb_table *tables;
    const EMB_LDS int64_t *s_base;
    const EMB_LDS emb_char_ptr *s_w;
    const EMB_LDS emb_float_ptr *s_a;
    bool staged;
    __device__ __forceinline__ int64_t base(int t) const
    {
        int64_t v;
        if (ALWAYS_LDS || staged) v = s_base[t]; else v = tables[t].row_base;
        return v;
    }
    __device__ __forceinline__ char *weights(int t) const
    {
        char *v;
        if (ALWAYS_LDS || staged) v = s_w[t]; else v = reinterpret_cast<char *>(tables[t].weights);
        return v;
    }
    __device__ __forceinline__ float *accum(int t) const
    {
        float *v;
        if (ALWAYS_LDS || staged) v = s_a[t]; else v = tables[t].accum;
        return v;
    }
};
typedef TableDirT<false> TableDir;

#define EMB_STAGE_TABLE_DIR(dir, tables, T, BLOCK) EMB_STAGE_TABLE_DIR_T(dir, tables, T, BLOCK, false)
#define EMB_STAGE_TABLE_DIR_T(dir, tables, T, BLOCK, ALWAYS)                    \
    __shared__ int64_t dir##_base[UPD_LDS_TABLES];                              \
    __shared__ char *dir##_w[UPD_LDS_TABLES];                                   \
    __shared__ float *dir##_a[UPD_LDS_TABLES];                                  \
    TableDirT<ALWAYS> dir{tables, (const EMB_LDS int64_t *)dir##_base, (const EMB_LDS emb_char_ptr *)dir##_w,       \
                 (const EMB_LDS emb_float_ptr *)dir##_a, (T) <= UPD_LDS_TABLES};                            \
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
            store_chunk_nt(wrow + (int64_t)chunk * 16, x);
        }
    }
    if (l == 0) store_f32_nt(aptr, s_new);
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
// short runs: one wavefront per span of UPD_SPAN sorted records
// ---------------------------------------------------------------------------
template <typename KeyT, int LPR, int CPL, int EU, bool BF16, bool LDS_DIR>
__global__ __launch_bounds__(UPD_BLOCK) void update_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                           const KeyT *__restrict__ keys,
                                                           const uint32_t *__restrict__ pay, uint32_t n,
                                                           KeyT sentinel, const float *__restrict__ bag_scale,
                                                           const float *__restrict__ dout, int32_t chunks_per_row,
                                                           int32_t D, float inv_D, float lr, float eps, BagDiv bdiv,
                                                           const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    constexpr int WAVES = UPD_BLOCK / EMB_WAVE;
    constexpr int GPW = EMB_WAVE / LPR;            // lane groups per wavefront
    constexpr int WIN = UPD_SPAN + UPD_LOOK;       // records staged per wavefront
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    static_assert(UPD_SPAN == 4 * EMB_WAVE && UPD_LOOK == 32, "staging below assumes 4 records per lane + 32");
    EMB_STAGE_TABLE_DIR_T(dir, tables, T, UPD_BLOCK, LDS_DIR)
    // [0] = the record before the span, [1 + e] = record e of the window, [WIN + 1] = the record after it
    __shared__ KeyT lk[WAVES][WIN + 2];
    __shared__ uint32_t lp[WAVES][WIN];
    __shared__ uint16_t lh[WAVES][UPD_SPAN + 2];   // window positions of the run heads, ascending

    const int wave = threadIdx.x / EMB_WAVE;
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int g = lane / LPR;
    const int l = lane % LPR;
    // sorted records are table-major: one die works on one stretch of tables (emb_xcd_block)
    const uint64_t wid = (uint64_t)emb_xcd_block(blockIdx.x, gridDim.x) * WAVES + wave;
    const uint64_t first = wid * UPD_SPAN;
    const bool in = first < n;
    const uint32_t i0 = (uint32_t)first;

    // ---- stage the span and the look-ahead (the arrays carry SORT_PAD records of slack)
    if (in) {
        {
            KeyT k[4];
            uint32_t b[4];
            load_records<KeyT, 4>(keys + i0 + lane * 4, k);
            load_records<uint32_t, 4>(pay + i0 + lane * 4, b);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool live = i0 + lane * 4 + e < n;
                lk[wave][1 + lane * 4 + e] = live ? k[e] : sentinel;
                lp[wave][lane * 4 + e] = live ? b[e] : 0u;
            }
        }
        if (lane < UPD_LOOK / 4) {
            KeyT k[4];
            uint32_t b[4];
            const uint32_t at = i0 + UPD_SPAN + lane * 4;
            const bool any = at < n;       // a window that starts inside the array may end outside its slack
            if (any) {
                load_records<KeyT, 4>(keys + at, k);
                load_records<uint32_t, 4>(pay + at, b);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool live = any && at + e < n;
                lk[wave][1 + UPD_SPAN + lane * 4 + e] = live ? k[e] : sentinel;
                lp[wave][UPD_SPAN + lane * 4 + e] = live ? b[e] : 0u;
            }
        }
        if (lane == 0) {
            lk[wave][0] = i0 > 0 ? keys[i0 - 1] : sentinel;
            lk[wave][WIN + 1] = (n - i0 > (uint32_t)WIN) ? keys[i0 + WIN] : sentinel;
        }
    }
    __syncthreads();

    // ---- list the positions where the key changes (sentinel records form runs that nobody sums)
    uint32_t runs = 0;   // heads inside the span
    if (in) {
        uint32_t bits = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) bits |= (lk[wave][1 + lane * 4 + e] != lk[wave][lane * 4 + e] ? 1u : 0u) << e;
        const uint32_t c = __popc(bits);
        const uint32_t incl = wave_inclusive_scan<uint32_t>(c);
        runs = (uint32_t)__shfl((int)incl, EMB_WAVE - 1, EMB_WAVE);
        uint32_t at = incl - c;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if ((bits >> e) & 1u) lh[wave][at++] = (uint16_t)(lane * 4 + e);
        // the first head of the look-ahead ends the last run of the span
        uint32_t la = WIN;
        if (lane < UPD_LOOK / 4) {
#pragma unroll
            for (int e = 3; e >= 0; --e) {
                const int idx = UPD_SPAN + lane * 4 + e;
                if (lk[wave][1 + idx] != lk[wave][idx]) la = idx;
            }
        }
#pragma unroll
        for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)la, d, EMB_WAVE);
            la = o < la ? o : la;
        }
        if (lane == 0) lh[wave][runs] = (uint16_t)la;
    }
    __syncthreads();

    if (in) {
        const int64_t row_bytes = (int64_t)chunks_per_row * 16;
        // groups take the runs round-robin: every group gets the same number of runs, give or take one
        for (uint32_t k = g; k < runs; k += GPW) {
            const int pos = lh[wave][k];
            const int end = lh[wave][k + 1];
            const KeyT key = lk[wave][1 + pos];
            if (key == sentinel) continue;
            // longer than UPD_SHORT_MAX records (a run that is not over after the look-ahead is): not
            // this kernel's; long_detect_kernel has queued it for the chunked path
            if (end - pos > UPD_SHORT_MAX || (end == WIN && lk[wave][WIN + 1] == key)) continue;
            // ---- the row, its accumulator and the first EU gradient rows, all requested together
            const int t = bdiv.table(lp[wave][pos]);
            const int64_t r = (int64_t)key - dir.base(t);
            char *wrow = dir.weights(t) + r * row_bytes;
            float *aptr = dir.accum(t) + r;
            // gradient rows of records e0 .. e0 + EU - 1 of the run (zeros past its end)
            auto load_batch = [&](int e0, float4 (&gr)[EU][CPL][V], float (&sc)[EU]) {
#pragma unroll
                for (int u = 0; u < EU; ++u) {
                    const int e = e0 + u;
                    sc[u] = 0.f;
#pragma unroll
                    for (int c = 0; c < CPL; ++c)
#pragma unroll
                        for (int x = 0; x < V; ++x) gr[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (e < end) {
                        const uint32_t bag = lp[wave][e];
                        sc[u] = bag_scale[bag];
                        const float *grow = dout + (int64_t)bag * D;
#pragma unroll
                        for (int c = 0; c < CPL; ++c) {
                            const int chunk = l + c * LPR;
                            if (chunk < chunks_per_row) load_grad<BF16>(grow + (int64_t)chunk * F, gr[u][c]);
                        }
                    }
                }
            };
            GradAcc<BF16> acc[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c].zero();
            // The first gradient rows are requested before the table row and its accumulator: loads come
            // back in the order they were asked for, so the sum can start while the row is still on its way.
            float4 gr[EU][CPL][V];
            float sc[EU];
            load_batch(pos, gr, sc);
            uint4 w[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int chunk = l + c * LPR;
                w[c] = make_uint4(0, 0, 0, 0);
                if (chunk < chunks_per_row) w[c] = load_chunk_nt(wrow + (int64_t)chunk * 16);
            }
            const float s_old = load_f32_nt(aptr);
#pragma unroll
            for (int u = 0; u < EU; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], gr[u][c]);
            for (int e0 = pos + EU; e0 < end; e0 += EU) {
                load_batch(e0, gr, sc);
#pragma unroll
                for (int u = 0; u < EU; ++u)
#pragma unroll
                    for (int c = 0; c < CPL; ++c) acc[c].fma(sc[u], gr[u][c]);
            }
            adagrad_apply<LPR, CPL, BF16>(acc, w, s_old, wrow, aptr, l, chunks_per_row, inv_D, lr, eps);
        }
    }
}

// ---------------------------------------------------------------------------
// queued runs
// ---------------------------------------------------------------------------
// Runs longer than UPD_SHORT_MAX records are not summed by update_kernel but cut into
// chunks for whole wavefronts.  This kernel finds them: one wavefront per span of
// UPD_SPAN sorted records (the spans of update_kernel), four records per lane.
// Record i starts such a run iff it starts a run and record i + UPD_SHORT_MAX has the
// same key (keys are sorted).  Two such starts are more than UPD_SHORT_MAX records
// apart, so a span has at most UPD_QSLOTS of them: they go to the span's queue slots
// in ascending order, unused slots are marked.  The kernel only reads the keys, so
// it and the kernels it feeds can run beside update_kernel on another stream.
// It also counts the runs (= distinct rows) of the span, and records where runs
// start, which is where the run before them ends: for every queued run the next
// run start inside the span (queue_end, NO_RECORD if there is none), and the
// span's first run start (span_head), so that the end of a run that leaves its span
// is found by looking at the spans after it and not by searching the keys.
constexpr uint32_t NO_RECORD = 0xFFFFFFFFu;

template <typename KeyT>
__global__ __launch_bounds__(256) void long_detect_kernel(const KeyT *__restrict__ keys, uint32_t n, KeyT sentinel,
                                                          const BwdCtrl *ctrl, uint32_t *__restrict__ queue,
                                                          uint32_t *__restrict__ queue_end,
                                                          uint32_t *__restrict__ span_head,
                                                          uint32_t *__restrict__ wave_heads, uint32_t slots)
{
    if (ctrl->abort) return;
    static_assert(UPD_SPAN == 4 * EMB_WAVE, "four records per lane");
    static_assert(UPD_SHORT_MAX % 4 == 0 && UPD_SHORT_MAX + 4 <= SORT_PAD, "far records are read four at a time");
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const uint32_t wid = blockIdx.x * (256 / EMB_WAVE) + threadIdx.x / EMB_WAVE;
    if (wid >= slots) return;                       // whole wavefronts leave together
    const uint32_t i = wid * UPD_SPAN + lane * 4;   // < n + UPD_SPAN: inside the slack of the array
    KeyT k[4], far[4];
    KeyT prev = sentinel;
    if (i < n) {
        load_records<KeyT, 4>(keys + i, k);
        load_records<KeyT, 4>(keys + i + UPD_SHORT_MAX, far);
        if (i > 0) prev = keys[i - 1];
    }
    uint32_t heads = 0, start = NO_RECORD;
    uint32_t change = 0;   // bit e: record i + e starts a run (of a row, or of the marker of invalid rows)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (i + e < n) {
            const bool first = i + e == 0 || k[e] != prev;
            const bool head = first && k[e] != sentinel;
            change |= (first ? 1u : 0u) << e;
            heads += head ? 1u : 0u;
            if (head && i + e + UPD_SHORT_MAX < n && far[e] == k[e]) start = i + e;   // at most one per lane
            prev = k[e];
        }
    }
    // the run starts of the span as four masks over the lanes (position in the span = 4 * lane + e)
    uint64_t cm[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) cm[e] = __ballot(((change >> e) & 1u) != 0);
    const uint64_t above = (lane == EMB_WAVE - 1) ? 0ull : (~0ull << (lane + 1));   // the lanes after mine
    uint32_t next = NO_RECORD;   // first run start after my queued run, inside the span
    uint32_t head0 = NO_RECORD;  // first run start of the span
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (cm[e]) head0 = min(head0, (uint32_t)(__ffsll((unsigned long long)cm[e]) - 1) * 4 + e);
        if (start != NO_RECORD) {
            const uint64_t later = cm[e] & ((uint32_t)e > start - i ? (above | (1ull << lane)) : above);
            if (later) next = min(next, (uint32_t)(__ffsll((unsigned long long)later) - 1) * 4 + e);
        }
    }
    const uint64_t m = __ballot(start != NO_RECORD);
    const uint32_t rank = (uint32_t)__popcll(m & ((lane == 0) ? 0ull : (~0ull >> (64 - lane))));
    const uint32_t count = (uint32_t)__popcll(m);
    uint32_t *q = queue + (size_t)wid * UPD_QSLOTS;
    if (start != NO_RECORD && rank < (uint32_t)UPD_QSLOTS) {
        q[rank] = start;
        queue_end[(size_t)wid * UPD_QSLOTS + rank] = next == NO_RECORD ? NO_RECORD : wid * UPD_SPAN + next;
    }
    if (lane < UPD_QSLOTS && (uint32_t)lane >= count) q[lane] = NO_RECORD;
#pragma unroll
    for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) heads += __shfl_xor(heads, d, EMB_WAVE);
    if (lane == 0) {
        wave_heads[wid] = heads;
        span_head[wid] = head0 == NO_RECORD ? NO_RECORD : wid * UPD_SPAN + head0;
    }
}

// One thread per queue slot: the run's end, its chunks, the tasks.  Also adds up the
// per-span run counts.  A run ends where the next run starts: inside its own span
// (queue_end), else at the first run start of the spans after it, which the
// wavefront looks up together, 64 spans per round trip.
__global__ __launch_bounds__(PREP_BLOCK) void long_prepare_kernel(uint32_t n, BwdCtrl *ctrl,
                                                           const uint32_t *__restrict__ queue,
                                                           const uint32_t *__restrict__ queue_end, uint32_t slots,
                                                           const uint32_t *__restrict__ span_head,
                                                           const uint32_t *__restrict__ wave_heads,
                                                           uint32_t n_spans, LongSeg *__restrict__ segs,
                                                           uint32_t *__restrict__ multi_list,
                                                           uint2 *__restrict__ chunk_tasks, uint32_t chunk_cap)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[PREP_BLOCK / EMB_WAVE];
    const uint32_t s = blockIdx.x * PREP_BLOCK + threadIdx.x;
    const int lane = threadIdx.x & (EMB_WAVE - 1);

    // distinct rows: sum of the run counts
    {
        uint32_t h = s < n_spans ? wave_heads[s] : 0u, total;
        block_inclusive_scan<uint32_t, PREP_BLOCK>(h, wave_sums, total);
        if (threadIdx.x == 0 && total) atomicAdd(&ctrl->num_unique, total);
    }

    uint32_t lo = NO_RECORD, hi = 0, chunks = 0;
    if (s < slots) {   // both asked for together; queue_end of an unused slot is never looked at
        lo = queue[s];
        hi = queue_end[s];
    }
    // runs that leave their span: one at a time, the whole wavefront looks at the following spans
    uint64_t open = __ballot(lo != NO_RECORD && hi == NO_RECORD);
    while (open) {   // uniform
        const int l = __ffsll((unsigned long long)open) - 1;
        open &= open - 1;
        uint32_t w = (uint32_t)__shfl((int)lo, l, EMB_WAVE) / UPD_SPAN + 1;
        uint32_t found = n;                                 // no later run start: the run ends with the records
        while (w < n_spans) {   // uniform
            const uint32_t v = w + lane < n_spans ? span_head[w + lane] : NO_RECORD;
            const uint64_t hit = __ballot(v != NO_RECORD);
            if (hit) {
                found = (uint32_t)__shfl((int)v, __ffsll((unsigned long long)hit) - 1, EMB_WAVE);
                break;
            }
            w += EMB_WAVE;
        }
        if (lane == l) hi = found;
    }
    if (lo != NO_RECORD) chunks = (hi - lo + LONG_CHUNK - 1) / LONG_CHUNK;
    // task slots: exclusive scans inside the workgroup, then ONE atomic per workgroup on a packed
    // counter (tasks in the low half, runs of several chunks in the high half): same-address
    // device atomics are slow, and there are hundreds of workgroups
    uint32_t total_chunks, total_multi;
    const uint32_t inc_c = block_inclusive_scan<uint32_t, PREP_BLOCK>(chunks, wave_sums, total_chunks);
    const uint32_t multi = chunks > 1 ? 1u : 0u;
    const uint32_t inc_m = block_inclusive_scan<uint32_t, PREP_BLOCK>(multi, wave_sums, total_multi);
    __shared__ unsigned long long s_base;
    if (threadIdx.x == 0) {
        s_base = 0;
        if (total_chunks)
            s_base = atomicAdd(&ctrl->task_and_multi_count,
                               (unsigned long long)total_chunks | ((unsigned long long)total_multi << 32));
    }
    __syncthreads();
    if (chunks) {
        const uint32_t cbase = (uint32_t)s_base + inc_c - chunks;
        const uint32_t mbase = (uint32_t)(s_base >> 32) + inc_m - multi;
        LongSeg sg;
        sg.lo = lo;
        sg.hi = hi;
        sg.chunk_base = cbase;   // the chunk sums of a run use the slots of its tasks
        // the cap cannot be exceeded (see the workspace layout); the check only guards memory
        sg.n_chunks = (cbase + chunks <= chunk_cap) ? chunks : 0u;
        segs[s] = sg;
        for (uint32_t c = 0; c < sg.n_chunks; ++c) chunk_tasks[cbase + c] = make_uint2(s, c);
        if (sg.n_chunks > 1 && mbase < slots) multi_list[mbase] = s;
    }
}

// The row update of a queued run, by the LPR lanes that hold its summed gradient.
template <typename KeyT, int LPR, int CPL, bool BF16>
__device__ __forceinline__ void finish_run(const GradAcc<BF16> (&acc)[CPL], const TableDir &dir, const BagDiv &bdiv,
                                           const KeyT *__restrict__ keys, const uint32_t *__restrict__ pay,
                                           uint32_t lo, int l, int32_t chunks_per_row, float inv_D, float lr,
                                           float eps)
{
    const int64_t key = (int64_t)keys[lo];
    const int t = bdiv.table(pay[lo]);
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

// One wavefront per chunk task.
template <typename KeyT, int LPR, int CPL, int EU, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void long_reduce_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                const KeyT *__restrict__ keys,
                                                                const uint32_t *__restrict__ pay,
                                                                const float *__restrict__ bag_scale,
                                                                const float *__restrict__ dout,
                                                                int32_t chunks_per_row, int32_t D, float inv_D,
                                                                float lr, float eps, BagDiv bdiv,
                                                                const BwdCtrl *ctrl,
                                                                const LongSeg *__restrict__ segs,
                                                                const uint2 *__restrict__ chunk_tasks,
                                                                uint32_t chunk_cap, float *__restrict__ partials)
{
    if (ctrl->abort) return;
    EMB_STAGE_TABLE_DIR(dir, tables, T, UPD_BLOCK)
    __syncthreads();
    constexpr int GPW = EMB_WAVE / LPR;  // lane groups per wavefront
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int l = lane % LPR;
    const int g = lane / LPR;
    const int64_t row_floats = (int64_t)chunks_per_row * F;
    uint32_t tasks = (uint32_t)ctrl->task_and_multi_count;
    if (tasks > chunk_cap) tasks = chunk_cap;
    // Tasks were created roughly in record order, so neighbours mostly share a table: every die
    // (the grid is a multiple of EMB_XCDS) takes one contiguous eighth of them, strided over by
    // its wavefronts, and reads mostly one stretch of the output gradient.
    const uint32_t per_die = (tasks + EMB_XCDS - 1) / EMB_XCDS;
    const uint32_t die = blockIdx.x % EMB_XCDS;
    const uint32_t die_end = (die + 1) * per_die < tasks ? (die + 1) * per_die : tasks;
    const uint32_t waves = (gridDim.x / EMB_XCDS) * (UPD_BLOCK / EMB_WAVE);

    for (uint32_t task = die * per_die + (blockIdx.x / EMB_XCDS) * (UPD_BLOCK / EMB_WAVE) + threadIdx.x / EMB_WAVE;
         task < die_end; task += waves) {
        const uint2 tk = chunk_tasks[task];
        const LongSeg sg = segs[tk.x];
        const uint32_t lo = sg.lo + tk.y * LONG_CHUNK;
        const uint32_t hi = (sg.hi - lo > (uint32_t)LONG_CHUNK) ? lo + LONG_CHUNK : sg.hi;

        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        // a group's records are lo + g, lo + g + GPW, ...: their bags are requested PF at a time,
        // then the gradient rows EU at a time, so a chunk costs few dependent memory round trips
        constexpr int PF = (LONG_CHUNK / GPW) < 16 ? (LONG_CHUNK / GPW) : 16;
        static_assert(PF % EU == 0, "prefetch depth must be whole sub-batches");
        for (uint32_t i0 = lo + g; i0 < hi; i0 += GPW * PF) {
            uint32_t bags[PF];
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const uint32_t i = i0 + u * GPW;
                bags[u] = i < hi ? pay[i] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u0 = 0; u0 < PF; u0 += EU) {
                if (bags[u0] == 0xFFFFFFFFu) continue;   // past the end of the chunk
                float4 v[EU][CPL][V];
                float sc[EU];
#pragma unroll
                for (int u = 0; u < EU; ++u) {
                    const uint32_t bag = bags[u0 + u];
                    sc[u] = 0.f;
#pragma unroll
                    for (int c = 0; c < CPL; ++c)
#pragma unroll
                        for (int x = 0; x < V; ++x) v[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (bag != 0xFFFFFFFFu) {
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
        }
        // butterfly over the lane groups of the wavefront: every group ends with the chunk sum
#pragma unroll
        for (int d = LPR; d < EMB_WAVE; d <<= 1)
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int i = 0; i < F; ++i) acc[c].a[i] += __shfl_xor(acc[c].a[i], d, EMB_WAVE);

        if (g == 0) {
            if (sg.n_chunks == 1) {
                finish_run<KeyT, LPR, CPL, BF16>(acc, dir, bdiv, keys, pay, sg.lo, l, chunks_per_row, inv_D, lr, eps);
            } else {
                float *slot = partials + (int64_t)(sg.chunk_base + tk.y) * row_floats;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int chunk = l + c * LPR;
                    if (chunk < chunks_per_row) {
                        float4 *o = reinterpret_cast<float4 *>(slot + (int64_t)chunk * F);
#pragma unroll
                        for (int x = 0; x < V; ++x)
                            o[x] = make_float4(acc[c].a[4 * x], acc[c].a[4 * x + 1], acc[c].a[4 * x + 2],
                                               acc[c].a[4 * x + 3]);
                    }
                }
            }
        }
    }
}

// Runs of several chunks: one wavefront per run.  Its lane groups take the chunk
// sums round-robin in chunk order and are combined by the same fixed butterfly,
// then Adagrad is applied.  Also publishes the number of distinct rows.
template <typename KeyT, int LPR, int CPL, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void long_combine_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                 const KeyT *__restrict__ keys,
                                                                 const uint32_t *__restrict__ pay,
                                                                 int32_t chunks_per_row, float inv_D, float lr,
                                                                 float eps, BagDiv bdiv, const BwdCtrl *ctrl,
                                                                 const LongSeg *__restrict__ segs,
                                                                 const uint32_t *__restrict__ multi_list,
                                                                 uint32_t multi_cap,
                                                                 const float *__restrict__ partials,
                                                                 int64_t *num_unique_out)
{
    if (ctrl->abort) return;
    if (blockIdx.x == 0 && threadIdx.x == 0 && num_unique_out) *num_unique_out = (int64_t)ctrl->num_unique;
    EMB_STAGE_TABLE_DIR(dir, tables, T, UPD_BLOCK)
    __syncthreads();
    constexpr int GPW = EMB_WAVE / LPR;
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = GradAcc<BF16>::V;
    constexpr int CU = 2;  // chunk sums a group requests together
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int l = lane % LPR;
    const int g = lane / LPR;
    const int64_t row_floats = (int64_t)chunks_per_row * F;
    uint32_t count = (uint32_t)(ctrl->task_and_multi_count >> 32);
    if (count > multi_cap) count = multi_cap;
    const uint32_t waves = gridDim.x * (UPD_BLOCK / EMB_WAVE);
    for (uint32_t m = blockIdx.x * (UPD_BLOCK / EMB_WAVE) + threadIdx.x / EMB_WAVE; m < count; m += waves) {
        const LongSeg sg = segs[multi_list[m]];
        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        for (uint32_t c0 = g; c0 < sg.n_chunks; c0 += GPW * CU) {
            float4 v[CU][CPL][V];
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const uint32_t cc = c0 + u * GPW;
#pragma unroll
                for (int c = 0; c < CPL; ++c)
#pragma unroll
                    for (int x = 0; x < V; ++x) v[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (cc < sg.n_chunks) {
                    const float *slot = partials + (int64_t)(sg.chunk_base + cc) * row_floats;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int chunk = l + c * LPR;
                        if (chunk < chunks_per_row) load_grad<BF16>(slot + (int64_t)chunk * F, v[u][c]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < CU; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c].fma(1.0f, v[u][c]);
        }
#pragma unroll
        for (int d = LPR; d < EMB_WAVE; d <<= 1)
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int i = 0; i < F; ++i) acc[c].a[i] += __shfl_xor(acc[c].a[i], d, EMB_WAVE);
        if (g == 0)
            finish_run<KeyT, LPR, CPL, BF16>(acc, dir, bdiv, keys, pay, sg.lo, l, chunks_per_row, inv_D, lr, eps);
    }
}
