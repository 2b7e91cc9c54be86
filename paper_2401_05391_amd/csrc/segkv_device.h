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

// Work-groups are handed to the 8 XCDs round-robin (group i runs on XCD i % 8).
// Remap the hardware index so that each XCD works through one contiguous run of
// logical work items: neighbours in memory (the KV heads of one request, the
// chunks of one unit) then share an XCD and its L2, and every XCD sweeps whole
// rows instead of one fixed 256-byte column of them.
constexpr int kNumXcd = 8;
__device__ __forceinline__ int xcd_contiguous_index(int id, int n)
{
    const int xcd = id % kNumXcd;
    const int k = id / kNumXcd;
    const int per = n / kNumXcd;
    const int rem = n % kNumXcd;
    return xcd * per + min(xcd, rem) + k;
}

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
    uint32_t map[kListThreads];        // ordered tree reduction (steps after the chunk)
    uint32_t wave_map[kListThreads / 64];
    int wave_cnt[kListThreads / 64];
    uint32_t ent[kMaxListEntries];
    int total;
};

// One step's parent slots of request b, as loaded (not yet packed), so that a
// kernel can issue these loads early and consume them after other requests
// have been put in flight.
struct ParentRow {
    int32_t v[8];
};

__device__ __forceinline__ ParentRow load_parent_row(const int32_t* parent, int N, int W, int b, int s)
{
    const int32_t* row = parent + (size_t)s * N + (size_t)b * W;
    ParentRow r;
#pragma unroll
    for (int x = 0; x < 8; ++x) r.v[x] = (x < W) ? row[x] : x;
    return r;
}

__device__ __forceinline__ uint32_t pack_parent_row(const ParentRow& r, int W)
{
    uint32_t f = 0;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        // entries are trusted to lie in [0, W); clamping keeps a bad table inside
        // the request's own rows instead of reading past the buffers
        const uint32_t v = (x < W) ? (uint32_t)min(max(r.v[x], 0), W - 1) : (uint32_t)x;
        f |= v << (4 * x);
    }
    return f;
}

__device__ __forceinline__ uint32_t load_parent_map(const int32_t* parent, int N, int W, int b, int s)
{
    return pack_parent_row(load_parent_row(parent, N, W, b, s), W);
}

// The list thread t of a chunk [s0, s1) owns step s0+t and contributes the
// parent map of the following step; this issues its loads (nothing for threads
// without one: identity is substituted when packing).
__device__ __forceinline__ bool list_thread_has_row(int W, int s0, int s1)
{
    return W > 1 && (int)threadIdx.x < (s1 - s0) - 1;
}

// Every thread of the work-group must call this (it contains barriers); only
// threads 0..kListThreads-1 do the work.  Requires blockDim.x >= kListThreads,
// blockDim.x a multiple of 64, and s1 - s0 <= kListThreads.
// The scans run inside each wave with lane shuffles and are stitched across
// the kListThreads/64 waves through LDS, so a call costs three barriers (plus
// the tree reduction when steps follow the chunk).
// `own_map` is this thread's packed parent map of step s0+t+1 when
// list_thread_has_row() holds (ignored otherwise).
__device__ void build_response_list(ResponseListSmem& sm, const int32_t* parent, int32_t* anc_out,
                                    int B, int W, int T, int b, int s0, int s1, uint32_t own_map)
{
    constexpr int kListWaves = kListThreads / 64;
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int w = t >> 6;
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
            sm.map[t] = c;
        }
        for (int stride = 1; stride < kListThreads; stride <<= 1) {
            __syncthreads();
            if (active && (t & (2 * stride - 1)) == 0)
                sm.map[t] = map_compose(sm.map[t], sm.map[t + stride]);
        }
        __syncthreads();
        carry = sm.map[0];
    }

    // (2) inclusive suffix scan of y_t = P_{s0+t+1} (t < n-1), y_{n-1} = carry
    uint32_t x = kIdentityMap;
    if (t < n - 1) x = own_map;
    else if (t == n - 1) x = carry;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_down(x, off);
        if (lane + off < 64) x = map_compose(x, o);
    }
    if (active && lane == 0) sm.wave_map[w] = x;      // composition of the whole wave
    __syncthreads();
    if (active)
        for (int ww = w + 1; ww < kListWaves; ++ww) x = map_compose(x, sm.wave_map[ww]);
    const uint32_t A = x;                              // slot map of step s0+t

    // (3) distinct slots referenced at this step, and their exclusive prefix sum
    uint32_t present = 0;
    if (t < n)
        for (int j = 0; j < W; ++j) present |= 1u << map_get(A, j);
    const int mine = __popc(present);
    int c = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(c, off);
        if (lane >= off) c += o;
    }
    if (active && lane == 63) sm.wave_cnt[w] = c;
    __syncthreads();
    int pos = c - mine;
    if (active)
        for (int ww = 0; ww < w; ++ww) pos += sm.wave_cnt[ww];
    if (t == 0) {
        int tot = 0;
        for (int ww = 0; ww < kListWaves; ++ww) tot += sm.wave_cnt[ww];
        sm.total = tot;
    }

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

// ---------------------------------------------------------------------------
// The same list built by ONE wave, with no work-group barrier: the other waves
// of the group keep streaming prompt tiles meanwhile and take what is finished of
// the list (`top`, then `ready`) when they reach a response tile.
//
// Beam maps are kept one BYTE per beam here (byte j = slot of beam j), so that a
// composition is two v_perm_b32 byte permutes.  The chunk's steps are walked in
// windows of 256 (4 per lane) from the last window to the first -- the slot map
// of a step is a suffix composition, so it flows backwards -- and each window's
// entries are placed below the previous window's, from the end of the buffer
// down: after every window ent[top .. CAP) is a finished part of the list, ordered
// by step, and the whole list once the first window is done.
// ---------------------------------------------------------------------------
constexpr int kListStepsPerLane = 4;
constexpr int kListWindow = 64 * kListStepsPerLane;

struct BeamMap {
    uint32_t lo, hi;   // slots of beams 0..3 and 4..7, one byte each
};
constexpr uint32_t kIdBytesLo = 0x03020100u;
constexpr uint32_t kIdBytesHi = 0x07060504u;

// (f o g)[j] = f[g[j]]: the bytes of g select among the eight bytes of f
__device__ __forceinline__ BeamMap bm_compose(BeamMap f, BeamMap g)
{
    return BeamMap{__builtin_amdgcn_perm(f.hi, f.lo, g.lo), __builtin_amdgcn_perm(f.hi, f.lo, g.hi)};
}
__device__ __forceinline__ uint32_t bm_get(BeamMap f, int j)
{
    return ((j < 4 ? f.lo : f.hi) >> (8 * (j & 3))) & 0xffu;
}
__device__ __forceinline__ BeamMap bm_shfl_down(BeamMap f, int off)
{
    return BeamMap{(uint32_t)__shfl_down((int)f.lo, off), (uint32_t)__shfl_down((int)f.hi, off)};
}
__device__ __forceinline__ BeamMap bm_broadcast(BeamMap f, int src)
{
    return BeamMap{(uint32_t)__shfl((int)f.lo, src), (uint32_t)__shfl((int)f.hi, src)};
}
// entries are trusted to lie in [0, W); clamping keeps a bad table inside the
// request's own rows instead of reading past the buffers
__device__ __forceinline__ BeamMap bm_pack(const ParentRow& r, int W)
{
    uint32_t w[2] = {kIdBytesLo, kIdBytesHi};
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        if (x < W) {
            const uint32_t v = (uint32_t)min(max(r.v[x], 0), W - 1);
            w[x >> 2] = (w[x >> 2] & ~(0xffu << (8 * (x & 3)))) | (v << (8 * (x & 3)));
        }
    }
    return BeamMap{w[0], w[1]};
}

// Inclusive suffix composition over the lanes of a wave: lane i ends up with
// x_i o x_{i+1} o ... o x_63.
__device__ __forceinline__ BeamMap wave_suffix_compose(BeamMap x, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const BeamMap o = bm_shfl_down(x, off);
        const BeamMap c = bm_compose(x, o);
        if (lane + off < 64) x = c;
    }
    return x;
}

struct ListRows {
    ParentRow r[kListStepsPerLane];
};

// Requests the parent rows lane `lane` needs for the window that starts at step
// `a`: row a+t+1 for its steps t = 4 lane .. 4 lane + 3.  Rows past the table are
// pointed at the last valid row and ignored later, so that no load is
// conditional.  Requires W > 1 (parent non-null) and T >= 1.
__device__ __forceinline__ void load_list_rows(ListRows& rows, const int32_t* parent, int N, int W,
                                               int T, int b, int a, int lane)
{
#pragma unroll
    for (int k = 0; k < kListStepsPerLane; ++k) {
        const int s = min(a + kListStepsPerLane * lane + k + 1, T - 1);
        rows.r[k] = load_parent_row(parent, N, W, b, s);
    }
}

// First step of the last window of the chunk [s0, s1): the rows a kernel should
// request early (load_list_rows) and hand to build_response_list_wave.
__device__ __forceinline__ int list_last_window_start(int s0, int s1)
{
    return s0 + ((s1 - s0 - 1) / kListWindow) * kListWindow;
}

template <int CAP>
struct WaveListSmem {
    uint32_t ent[CAP];   // (local step << 16) | (slot << 8) | beam mask
    int top;             // ent[top .. CAP) is written; only ever decreases.  The
                         // kernel sets it to CAP before the builder starts.
    int ready;           // set (release) once top is final: the list is ent[top .. CAP)
};

// Called by all 64 lanes of exactly one wave.  Requires (s1 - s0) * W <= CAP and
// s1 - s0 < 65536.  `first_rows`: load_list_rows() of the window that starts at
// list_last_window_start(s0, s1) (ignored when W == 1).
template <int CAP>
__device__ void build_response_list_wave(WaveListSmem<CAP>& sm, const int32_t* parent,
                                         int32_t* anc_out, int B, int W, int T, int b, int s0,
                                         int s1, const ListRows& first_rows, int lane)
{
    constexpr int SPL = kListStepsPerLane;
    const int n_all = s1 - s0;
    const int N = B * W;
    if (W == 1) {
        for (int t = lane; t < n_all; t += 64) {
            sm.ent[CAP - n_all + t] = ((uint32_t)t << 16) | 1u;
            if (anc_out) anc_out[(size_t)(s0 + t) * N + b] = 0;
        }
        __hip_atomic_store(&sm.top, CAP - n_all, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_store(&sm.ready, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        return;
    }

    // slot map of the step that follows the chunk, A_{s1} = P_{s1+1} o ... o P_{T-1}
    // (only needed when the chunk does not end at T)
    BeamMap a_next = {kIdBytesLo, kIdBytesHi};
    if (s1 < T) {
        const int later = T - 1 - s1;
        const int per = (later + 63) / 64;
        const int lo = s1 + 1 + lane * per;
        const int hi = min(lo + per, T);
        BeamMap c = {kIdBytesLo, kIdBytesHi};
        for (int s = lo; s < hi; ++s) c = bm_compose(c, bm_pack(load_parent_row(parent, N, W, b, s), W));
        a_next = bm_broadcast(wave_suffix_compose(c, lane), 0);
    }

    int top = CAP;
    ListRows rows = first_rows;
    for (int a = list_last_window_start(s0, s1); a >= s0; a -= kListWindow) {
        const int bnd = min(a + kListWindow, s1);          // window [a, bnd)
        const int n = bnd - a;
        ListRows next_rows;
        if (a > s0) load_list_rows(next_rows, parent, N, W, T, b, a - kListWindow, lane);

        // y_t = P_{a+t+1} for t < n-1; y_{n-1} = P_bnd o A_bnd (identity when bnd == T);
        // A_{a+t} = y_t o y_{t+1} o ... o y_{n-1}
        BeamMap suf[SPL];
#pragma unroll
        for (int k = SPL - 1; k >= 0; --k) {
            const int t = SPL * lane + k;
            BeamMap y = {kIdBytesLo, kIdBytesHi};
            if (t < n && a + t + 1 < T) {
                y = bm_pack(rows.r[k], W);
                if (t == n - 1) y = bm_compose(y, a_next);
            }
            suf[k] = (k == SPL - 1) ? y : bm_compose(y, suf[k + 1]);
        }
        const BeamMap incl = wave_suffix_compose(suf[0], lane);
        BeamMap after = bm_shfl_down(incl, 1);             // composition of all later lanes
        if (lane == 63) after = BeamMap{kIdBytesLo, kIdBytesHi};
        a_next = bm_broadcast(incl, 0);                    // A_a, for the window below

        // per step: byte u of (mlo, mhi) = mask of the beams that sit on slot u
        BeamMap A[SPL];
        uint32_t mlo[SPL], mhi[SPL];
        int mine = 0;
#pragma unroll
        for (int k = 0; k < SPL; ++k) {
            A[k] = (k == 0) ? incl : bm_compose(suf[k], after);
            mlo[k] = 0;
            mhi[k] = 0;
            if (SPL * lane + k < n) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (j < W) {
                        const uint32_t slot = bm_get(A[k], j);
                        const uint32_t bit = (1u << j) << (8 * (slot & 3));
                        mlo[k] |= slot < 4 ? bit : 0u;
                        mhi[k] |= slot < 4 ? 0u : bit;
                    }
                }
            }
            // number of non-zero bytes
            const uint32_t nzl = (mlo[k] | ((mlo[k] & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u;
            const uint32_t nzh = (mhi[k] | ((mhi[k] & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u;
            mine += __popc(nzl) + __popc(nzh);
        }
        int c = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(c, off);
            if (lane >= off) c += o;
        }
        top -= __shfl(c, 63);                              // this window's rows go below the later ones
        int pos = top + c - mine;

#pragma unroll
        for (int k = 0; k < SPL; ++k) {
            const int t = SPL * lane + k;
            if (t < n) {
                const uint32_t step = (uint32_t)(a - s0 + t) << 16;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t mask = ((u < 4 ? mlo[k] : mhi[k]) >> (8 * (u & 3))) & 0xffu;
                    if (mask) sm.ent[pos++] = step | ((uint32_t)u << 8) | mask;
                }
                if (anc_out) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j < W)
                            anc_out[(size_t)(a + t) * N + (size_t)b * W + j] = (int32_t)bm_get(A[k], j);
                }
            }
        }
        // the window's rows are usable from here on, while the older windows are built
        __hip_atomic_store(&sm.top, top, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        rows = next_rows;
    }
    __hip_atomic_store(&sm.ready, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Index of the first entry of a lineage list (sorted by step) whose step is >=
// `step`, found by all 64 lanes of a wave together: every round samples the
// remaining range at 64 points, so 16 K entries take three dependent loads.
__device__ __forceinline__ int lineage_lower_bound(const uint32_t* ent, int n, int step, int lane)
{
    const uint32_t key = (uint32_t)step << 16;
    int lo = 0, hi = n;                                   // the answer lies in [lo, hi]
    while (hi > lo) {
        const int stride = (hi - lo + 63) / 64;
        const int idx = lo + lane * stride;
        const bool ge = (idx < hi) ? (ent[idx] >= key) : true;
        const unsigned long long votes = __ballot(ge);
        const int f = votes ? __ffsll((long long)votes) - 1 : 64;   // first sample >= key
        if (f == 0) return lo;
        if (stride == 1) return lo + f;
        hi = min(hi, lo + f * stride);
        lo = lo + (f - 1) * stride + 1;
    }
    return lo;
}

// The response list of the chunk [s0, s1) taken from the request's lineage list
// (`hdr`: its header, entries behind it) instead of being derived from the
// parent table: the entries of those steps are copied to the top of sm.ent with
// their steps made chunk-local.  Called by all 64 lanes of exactly one wave.
// Slots and steps are clamped into the chunk so that a list that was not kept up
// to date cannot send a load outside the request's rows.
template <int CAP>
__device__ void load_response_list_wave(WaveListSmem<CAP>& sm, const uint32_t* hdr, int capacity,
                                        int W, int T, int s0, int s1, int lane)
{
    const uint32_t* const ent = hdr + kLineageHeaderWords;
    const int n = min((int)hdr[0], capacity);
    const bool whole = (int)hdr[1] == T;                  // the list ends with step T-1
    const int i0 = (s0 > 0) ? lineage_lower_bound(ent, n, s0, lane) : 0;
    const int i1 = (s1 < T || !whole) ? lineage_lower_bound(ent, n, s1, lane) : n;
    const int cnt = min(max(i1 - i0, 0), CAP);
    const int top = CAP - cnt;
    for (int i = lane; i < cnt; i += 64) {
        const uint32_t e = ent[i0 + i];
        const uint32_t step = (uint32_t)min(max((int)(e >> 16) - s0, 0), s1 - s0 - 1);
        const uint32_t slot = min((e >> 8) & 0xffu, (uint32_t)(W - 1));
        sm.ent[top + i] = (step << 16) | (slot << 8) | (e & 0xffu);
    }
    __hip_atomic_store(&sm.top, top, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_store(&sm.ready, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Any other wave: waits until ent[want .. CAP) is written or the list is final,
// whichever comes first.  Returns the published top and sets `final`.
// The builder wave never waits for anything (it neither takes a barrier nor
// reads what other waves produce before it publishes), so the wait ends after
// one window's worth of composition at most.  The poll is bounded all the same:
// should a later change break that invariant, the wave leaves after
// kListWaitPolls polls with an EMPTY list (wrong attention output, which the
// parity tests catch) instead of occupying the GPU for good.
constexpr int kListWaitPolls = 1 << 22;   // x ~0.1 us per poll: far beyond any list build
template <int CAP>
__device__ __forceinline__ int wait_response_list(WaveListSmem<CAP>& sm, int want, bool& final)
{
    for (int poll = 0; poll < kListWaitPolls; ++poll) {
        const int rdy = __builtin_amdgcn_readfirstlane(
            __hip_atomic_load(&sm.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
        const int top = __builtin_amdgcn_readfirstlane(
            __hip_atomic_load(&sm.top, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
        if (rdy || top <= want) {
            final = rdy != 0;
            return top;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    final = true;
    return CAP;
}

}  // namespace segkv
