// Device-side pieces shared by the vector-ALU and the MFMA decode kernels:
// 128-bit load/store helpers and the in-kernel ancestor resolution that turns
// the raw parent table into the list of distinct response rows to read.
#pragma once
#include "segkv_common.h"
#include "segkv_launch.h"

namespace segkv {

// Threads that take part in the response-list construction: one per response
// step of a chunk.  Work-groups may be larger; the extra threads only join the
// barriers.
constexpr int kListThreads = kMaxStepsPerChunk;

__device__ __forceinline__ u32x4_t load16(const _Float16* p)
{
    return *reinterpret_cast<const u32x4_t*>(p);
}
// K/V rows are read exactly once per launch: non-temporal, so they stream past
// the caches instead of evicting what is reused (Q, parent table, partials).
__device__ __forceinline__ u32x4_t load16_stream(const _Float16* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
}
__device__ __forceinline__ void store16(_Float16* p, u32x4_t v)
{
    *reinterpret_cast<u32x4_t*>(p) = v;
}
__device__ __forceinline__ half2_t as_half2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }

// ---------------------------------------------------------------------------
// Ancestor resolution for the response steps [s0, s1) of request b
// (Section 3.3, index select).  With P_s the packed parent map of step s, the
// slot map of step s is A_s = P_{s+1} o P_{s+2} o ... o P_{T-1} (A_{T-1} = id),
// i.e. a suffix composition: computed as an ordered tree reduction for the
// steps after the chunk and a block-wide suffix scan inside it.
// Leaves in LDS: ent[0..total) = (local step << 16) | (slot << 8) | beam mask
// for every distinct row referenced, ordered by step.  All threads must call.
// ---------------------------------------------------------------------------
struct ResponseListSmem {
    uint32_t map[2][kListThreads];
    int cnt[2][kListThreads];
    uint32_t ent[kListThreads * 8];
    int total;
};

__device__ __forceinline__ uint32_t load_parent_map(const int32_t* parent, int N, int W, int b, int s)
{
    const int32_t* row = parent + (size_t)s * N + (size_t)b * W;
    uint32_t f = kIdentityMap;
    for (int x = 0; x < W; ++x) {
        // entries are trusted to lie in [0, W); clamping keeps a bad table inside
        // the request's own rows instead of reading past the buffers
        const uint32_t v = (uint32_t)min(max(row[x], 0), W - 1);
        f = (f & ~(15u << (4 * x))) | (v << (4 * x));
    }
    return f;
}

// Every thread of the work-group must call this (it contains barriers); only
// threads 0..kListThreads-1 do the work.  Requires blockDim.x >= kListThreads
// and s1 - s0 <= kListThreads.
__device__ void build_response_list(ResponseListSmem& sm, const int32_t* parent, int32_t* anc_out,
                                    int B, int W, int T, int b, int s0, int s1)
{
    const int t = threadIdx.x;
    const bool active = t < kListThreads;
    const int n = s1 - s0;
    const int N = B * W;
    if (W == 1) {
        if (t < n) {
            sm.ent[t] = ((uint32_t)t << 16) | 1u;
            if (anc_out) anc_out[(size_t)(s0 + t) * N + b] = 0;
        }
        if (t == 0) sm.total = n;
        __syncthreads();
        return;
    }

    // (1) carry = A_{s1-1} = P_{s1} o ... o P_{T-1}
    uint32_t carry = kIdentityMap;
    const int later = T - s1;
    if (later > 0) {
        if (active) {
            const int per = (later + kListThreads - 1) / kListThreads;
            const int lo = s1 + t * per;
            const int hi = min(lo + per, T);
            uint32_t c = kIdentityMap;
            for (int s = lo; s < hi; ++s) c = map_compose(c, load_parent_map(parent, N, W, b, s));
            sm.map[0][t] = c;
        }
        for (int stride = 1; stride < kListThreads; stride <<= 1) {
            __syncthreads();
            if (active && (t & (2 * stride - 1)) == 0)
                sm.map[0][t] = map_compose(sm.map[0][t], sm.map[0][t + stride]);
        }
        __syncthreads();
        carry = sm.map[0][0];
        __syncthreads();
    }

    // (2) inclusive suffix scan of y_t = P_{s0+t+1} (t < n-1), y_{n-1} = carry
    uint32_t y = kIdentityMap;
    if (t < n - 1) y = load_parent_map(parent, N, W, b, s0 + t + 1);
    else if (t == n - 1) y = carry;
    int cur = 0;
    if (active) sm.map[0][t] = y;
    __syncthreads();
    for (int off = 1; off < kListThreads; off <<= 1) {
        if (active) {
            uint32_t x = sm.map[cur][t];
            if (t + off < kListThreads) x = map_compose(x, sm.map[cur][t + off]);
            sm.map[cur ^ 1][t] = x;
        }
        cur ^= 1;
        __syncthreads();
    }
    const uint32_t A = active ? sm.map[cur][t] : kIdentityMap;   // slot map of step s0+t

    // (3) distinct slots referenced at this step, and their exclusive prefix sum
    uint32_t present = 0;
    if (t < n)
        for (int j = 0; j < W; ++j) present |= 1u << map_get(A, j);
    const int mine = __popc(present);
    int ccur = 0;
    if (active) sm.cnt[0][t] = mine;
    __syncthreads();
    for (int off = 1; off < kListThreads; off <<= 1) {
        if (active) {
            int x = sm.cnt[ccur][t];
            if (t >= off) x += sm.cnt[ccur][t - off];
            sm.cnt[ccur ^ 1][t] = x;
        }
        ccur ^= 1;
        __syncthreads();
    }
    int pos = active ? sm.cnt[ccur][t] - mine : 0;
    if (t == kListThreads - 1) sm.total = sm.cnt[ccur][t];

    // (4) entries, and the resolved table if asked for
    if (t < n) {
        for (int u = 0; u < W; ++u) {
            if (present & (1u << u)) {
                uint32_t mask = 0;
                for (int j = 0; j < W; ++j)
                    if (map_get(A, j) == (uint32_t)u) mask |= 1u << j;
                sm.ent[pos++] = ((uint32_t)t << 16) | ((uint32_t)u << 8) | mask;
            }
        }
        if (anc_out)
            for (int j = 0; j < W; ++j)
                anc_out[(size_t)(s0 + t) * N + (size_t)b * W + j] = (int32_t)map_get(A, j);
    }
    __syncthreads();
}

}  // namespace segkv
