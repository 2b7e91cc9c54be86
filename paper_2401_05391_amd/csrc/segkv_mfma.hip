// libsegkv device code: fused decode-step attention over a segment KV cache
// (arxiv 2401.05391, Section 3.3) for gfx950, matrix-core (MFMA) path.
//
// Used when several queries share every K/V row of a unit (request b, KV head
// g): the W beams and, under grouped-query attention, the G query heads of the
// group.  Up to 32 such queries form the N dimension of 32x32x16 fp16 MFMAs, a
// tile of 32 keys forms M:
//     S^T[key][query]  = K[key][:]   . Q^T[:][query]       (contraction over D)
//     O^T[d][query]   += V^T[d][key] . P^T[key][query]     (contraction over keys)
// so that each K/V row is read from HBM once and reused by all queries.
//
// Each wave streams its own key tiles, with no work-group barrier in the loop:
//   global (coalesced 128-bit, non-temporal) -> registers -> wave-private LDS
//   tile (rows padded by 16 bytes against bank conflicts) -> MFMA operands.
// While a tile is being multiplied the next one is already in flight in
// registers.  Softmax statistics are fp32; P is rounded to fp16 for the PV
// product; the running maximum is only moved when a tile exceeds it by 2^8 so
// that the accumulator rescale is rare.  Waves are merged through LDS at the end.
#include "segkv_common.h"
#include "segkv_launch.h"
#include "segkv_device.h"
#include "segkv_mfma_tile.h"

#include <cstdlib>

// Optional phase timestamps for kernel tuning (compiled in only with
// -DSEGKV_TIMING; slot k of work-group g, wave w lands in p.timing).
#ifdef SEGKV_TIMING
#define SEGKV_STAMP(k)                                                                   \
    do {                                                                                 \
        if (p.timing && (threadIdx.x & 63) == 0)                                         \
            p.timing[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (k)] = wall_clock64(); \
    } while (0)
#define SEGKV_STAMP_FIRST(k)                                                             \
    do {                                                                                 \
        if (p.timing && (threadIdx.x & 63) == 0 &&                                       \
            p.timing[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (k)] == 0)     \
            p.timing[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (k)] = wall_clock64(); \
    } while (0)
#define SEGKV_PHASE_DECL unsigned long long ph_t = __builtin_readcyclecounter(), ph_acc[4] = {0, 0, 0, 0}
#define SEGKV_PHASE_BEGIN ph_t = __builtin_readcyclecounter()
#define SEGKV_PHASE(k)                                       \
    do {                                                     \
        const unsigned long long now_ = __builtin_readcyclecounter(); \
        ph_acc[k] += now_ - ph_t;                            \
        ph_t = now_;                                         \
    } while (0)
#define SEGKV_PHASE_DUMP                                                                   \
    do {                                                                                   \
        if (p.timing && (threadIdx.x & 63) == 0)                                           \
            for (int k_ = 0; k_ < 4; ++k_)                                                 \
                p.timing[(((size_t)1 << 16) * 16 * 8) + ((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 4 + k_] = ph_acc[k_]; \
    } while (0)
#else
#define SEGKV_STAMP(k) do { } while (0)
#define SEGKV_STAMP_FIRST(k) do { } while (0)
#define SEGKV_PHASE_DECL do { } while (0)
#define SEGKV_PHASE_BEGIN do { } while (0)
#define SEGKV_PHASE(k) do { } while (0)
#define SEGKV_PHASE_DUMP do { } while (0)
#endif

namespace segkv {

template <int D, int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64) void sdpa_decode_mfma_kernel(SdpaParams p)
{
    using Geo = MfmaGeometry<D>;
    constexpr int CPR = Geo::CPR, RPI = Geo::RPI, NLD = Geo::NLD, NKS = Geo::NKS, NDB = Geo::NDB;
    constexpr int ROWB = Geo::ROWB, VROWB = Geo::VROWB, TILEB = Geo::TILEB, MROW = Geo::MROW;
    constexpr int REGIONB = Geo::REGIONB;
    constexpr int NT = NW * 64;
    static_assert(NT >= kListThreads, "the response list needs one thread per step");

    __shared__ __align__(16) unsigned char s_region[NW * REGIONB];
    __shared__ __align__(16) unsigned char s_q[kQueryTile * ROWB];   // Q^T operand, shared by the waves
    __shared__ ResponseListSmem s_list;
    __shared__ float s_ml[NW][kQueryTile][2];
    __shared__ int s_next_tile;                        // next unclaimed tile of the stream

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: tile indices stay uniform
    SEGKV_STAMP(0);
    const int n = lane & 31;        // query slot (MFMA column) / key row (MFMA A row) / d within block
    const int h = lane >> 5;        // lane half: which 8 of the 16 contraction slots
    const int srow = lane / CPR;    // staging: row within a load instruction
    const int schunk = lane % CPR;  // staging: 16-byte chunk of the row

    // ---- which work item ----
    // Hardware order (group i runs on XCD i % 8): with the KV head as the fastest
    // index each XCD streams one 256-byte column class of every request.  Measured
    // 2% faster on MI355X than giving each XCD a contiguous run of requests.
    int id = (int)blockIdx.x;
    const int qb = id % p.n_qblocks; id /= p.n_qblocks;
    const int g = id % p.Hkv;        id /= p.Hkv;
    const int chunk = id % p.n_chunks;
    const int b = id / p.n_chunks;
    const int N = p.B * p.W;

    int k0 = 0, k1 = 0, s0 = 0, s1 = 0;
    if (p.merged) {
        k1 = p.Lp;
        s1 = p.T;
    } else if (chunk < p.n_rchunks) {
        s0 = chunk * p.rchunk;
        s1 = min(s0 + p.rchunk, p.T);
    } else {
        k0 = (chunk - p.n_rchunks) * p.pchunk;
        k1 = min(k0 + p.pchunk, p.Lp);
    }
    const bool direct_out = (p.n_chunks == 1);

    unsigned char* const region = s_region + wave * REGIONB;
    unsigned char* const k_tile = region;
    unsigned char* const v_tile = region + TILEB;      // K tile first, then the V tile

    // ---- queries of this block: staged once into LDS in the same padded row
    // layout as the key tiles; every wave reads its QK^T B operand from there ----
    const int lq = qb * kQueryTile + n;
    const bool q_valid = lq < p.nq;
    const int lqc = q_valid ? lq : (p.nq - 1);
    const int qbeam = lqc / p.G;
    const int hq = g * p.G + (lqc % p.G);
    const float slope2 = p.slopes ? p.slopes[hq] * kLog2e : 0.0f;
    const int qpos = p.Lp + p.T - 1;
    // Requests that later steps depend on go out first, in this order: the Q
    // chunks this thread stages, its row of the parent table, then (below) the
    // wave's first key tile.  They are consumed in the same order, so each wait
    // leaves the younger requests in flight.
    constexpr int QCH = (kQueryTile * CPR + NT - 1) / NT;
    u32x4_t qw[QCH];
#pragma unroll
    for (int c = 0; c < QCH; ++c) {
        const int i = tid + c * NT;
        const int qn = i / CPR;
        const int ch = i % CPR;
        const int lqn = qb * kQueryTile + qn;
        qw[c] = u32x4_t{0u, 0u, 0u, 0u};               // unused query slots multiply as zeros
        if (i < kQueryTile * CPR && lqn < p.nq) {
            const size_t row = (size_t)(b * p.W + lqn / p.G) * p.Hq + g * p.G + (lqn % p.G);
            qw[c] = load16(p.q + row * D + ch * 8);
        }
    }
    // One wave (the last) resolves the response list on its own while the others
    // stream prompt tiles; its parent rows are requested here, with the Q chunks.
    const bool has_resp = s1 > s0;                              // uniform over the work-group
    const bool is_builder = has_resp && wave == NW - 1;         // uniform over the wave
    ListRows lrows;
    if (is_builder && p.W > 1) load_list_rows(lrows, p.parent, N, p.W, p.T, b, s0, lane);

    // ---- fused append: the block that owns step T-1 copies the unit's new rows.
    // One (K, V) vector pair per thread; only the loads are issued here, the
    // stores follow once the Q tile has arrived, so nothing waits on them. ----
    const bool have_new = (p.k_new != nullptr);
    constexpr int kVecPerRow = D / 8;
    static_assert(8 * kVecPerRow <= NT, "one append vector pair per thread (beam <= 8)");
    const bool appends = have_new && qb == 0 && s1 == p.T && s0 < s1 && tid < p.W * kVecPerRow;
    u32x4_t app_k = {0u, 0u, 0u, 0u}, app_v = {0u, 0u, 0u, 0u};
    size_t app_dst = 0;
    if (appends) {
        const int u = tid / kVecPerRow;
        const int col = tid % kVecPerRow;
        const size_t src = ((size_t)(b * p.W + u) * p.Hkv + g) * D + col * 8;
        app_dst = (((size_t)(p.T - 1) * N + b * p.W + u) * p.Hkv + g) * D + col * 8;
        app_k = load16(p.k_new + src);
        app_v = load16(p.v_new + src);
    }

    SEGKV_PHASE_DECL;
    // ---- running state: reference max and partial sum per lane, O^T accumulators ----
    float m_ref = kEmptyMax;
    float l_part = 0.0f;            // sum of p over this lane's 16 keys of every tile
    float16_t o_acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.0f;

    struct Staged {
        u32x4_t k[NLD];
        u32x4_t v[NLD];
    };

    // registers -> the wave's LDS tiles
    auto stage_to_lds = [&](const Staged& st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int row = RPI * i + srow;
            *reinterpret_cast<u32x4_t*>(k_tile + row * ROWB + (schunk << 4)) = st.k[i];
            *reinterpret_cast<u32x4_t*>(v_tile + row * VROWB + (schunk << 4)) = st.v[i];
        }
    };

    // One tile of 32 keys.  `mode` (uniform) selects how S^T becomes base-2 logits:
    // 0 full prompt tile without positional bias, 1 prompt tile with masking of
    // the tail and ALiBi, 2 response tile (per-row beam masks and positions).
    auto compute_tile = [&](int mode, int base, int total) __attribute__((always_inline)) {
        // S^T = K . Q^T
        float16_t s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
        for (int t = 0; t < NKS; ++t) {
            const int off = n * ROWB + ((2 * t + h) << 4);
            const half8_t a = *reinterpret_cast<const half8_t*>(k_tile + off);
            const half8_t bq = *reinterpret_cast<const half8_t*>(s_q + off);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bq, s, 0, 0, 0);
        }
        SEGKV_PHASE(1);
        // logits, tile maximum for this lane's query
        float m_tile = -INFINITY;
        if (mode == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[r] *= p.scale2;
                m_tile = fmaxf(m_tile, s[r]);
            }
        } else if (mode == 1) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kpos = base + 8 * (r >> 2) + 4 * h + (r & 3);
                const float z = s[r] * p.scale2 + slope2 * (float)(kpos - qpos);
                s[r] = kpos < k1 ? z : -INFINITY;
                m_tile = fmaxf(m_tile, s[r]);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int e = base + 8 * (r >> 2) + 4 * h + (r & 3);
                const uint32_t ent = s_list.ent[min(e, total - 1)];
                const int kpos = p.Lp + s0 + (int)(ent >> 16);
                const float z = s[r] * p.scale2 + slope2 * (float)(kpos - qpos);
                const bool vis = (e < total) && ((ent >> qbeam) & 1u);
                s[r] = vis ? z : -INFINITY;
                m_tile = fmaxf(m_tile, s[r]);
            }
        }
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
        // move the reference maximum only when a tile exceeds it by the slack
        if (__any(m_tile > m_ref + kRescaleSlack)) {
            const float m_new = fmaxf(m_ref, m_tile);
            const float corr = fast_exp2(m_ref - m_new);
            m_ref = m_new;
            l_part *= corr;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= corr;
        }
        // P = 2^(z - m_ref), fp16 for the PV product
        half8_t pb[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float pr = fast_exp2(s[r] - m_ref);
            l_part += pr;
            pb[r >> 3][r & 7] = (_Float16)pr;
        }
        SEGKV_PHASE(2);
        // O^T += V^T . P^T.  The A operand wants, per lane, 8 keys of one head-dim
        // column; the V tile is row-major [key][d].  ds_read_b64_tr_b16 does the
        // transpose on the way out of LDS: a 16-lane group reads 4 rows x 16
        // columns (lane i supplies row i/4, columns 4*(i%4)..+3) and lane i
        // receives column i of all 4 rows.  Two such reads give the 8 keys
        // 16u + 8r + 4h + {0..3}, r = 0, 1, matching the keys of P's registers.
        {
            const int grp = lane >> 4;                 // 16-lane group: d half (grp&1), key half h
            const int li = lane & 15;
            const int tr_base = (4 * h + (li >> 2)) * VROWB + ((16 * (grp & 1) + 4 * (li & 3)) << 1);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int off = tr_base + (16 * u) * VROWB + db * 64;
                    const half4_t lo = lds_read_tr16(v_tile + off);
                    const half4_t hi = lds_read_tr16(v_tile + off + 8 * VROWB);
                    const half8_t a = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[u], o_acc[db], 0, 0, 0);
                }
                // keep the operand reads of later blocks from piling up in registers
                if (NDB > 4) __builtin_amdgcn_sched_barrier(0);
            }
        }
        SEGKV_PHASE(3);
    };

    // ---- one tile stream per work-group: prompt tiles first (Section 3.3: loop
    // over the prompt keys), then the response tiles (index select fused: rows
    // chosen by the beam lineage).  Waves claim tiles from a shared counter, so a
    // wave whose loads come back sooner takes more of them.  Each wave keeps one
    // tile in flight in registers while it computes the previous one.  A fetch is
    // never skipped: past the end of the stream it is pointed at one row that is
    // already cached, so that the code is free of conditional loads and every
    // wait covers exactly the tile it needs. ----
    const int n_ptiles = (k1 > k0) ? (k1 - k0 + kKeyTile - 1) / kKeyTile : 0;
    const _Float16* const dummy = p.q + (size_t)b * p.W * p.Hq * D + schunk * 8;
    // Prompt tiles are addressed as (scalar tile base) + (32-bit lane offset):
    // the lane offsets are the same for every full tile, so no per-load 64-bit
    // address has to be kept in registers.
    const uint32_t row_stride = (uint32_t)p.Hkv * D;   // elements between consecutive keys
    auto fetch_prompt = [&](Staged& st, int ti) __attribute__((always_inline)) {
        const int base = k0 + ti * kKeyTile;
        const int lim = min(kKeyTile - 1, k1 - 1 - base);          // last valid row of the tile
        const size_t tile_off = (((size_t)b * p.Lp + base) * p.Hkv + g) * D;
        const _Float16* const kb = p.prompt_k + tile_off;
        const _Float16* const vb = p.prompt_v + tile_off;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const uint32_t off = (uint32_t)min(RPI * i + srow, lim) * row_stride + schunk * 8;
            st.k[i] = load16_stream(kb + off);
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const uint32_t off = (uint32_t)min(RPI * i + srow, lim) * row_stride + schunk * 8;
            st.v[i] = load16_stream(vb + off);
        }
    };
    auto fetch_dummy = [&](Staged& st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) st.k[i] = load16(dummy);
#pragma unroll
        for (int i = 0; i < NLD; ++i) st.v[i] = load16(dummy);
    };

    // The response list comes from the builder wave; a wave asks for it when it
    // first claims a tile past the prompt tiles (by then it is long finished).
    int total = 0;
    int n_tiles = n_ptiles;
    bool list_known = !has_resp;
    auto need_list = [&]() {
        if (!list_known) {
            total = wait_response_list(s_list);
            n_tiles = n_ptiles + (total + kKeyTile - 1) / kKeyTile;
            list_known = true;
        }
    };
    auto claim_tile = [&]() {
        int v = 0;
        if (lane == 0) v = atomicAdd(&s_next_tile, 1);
        return __builtin_amdgcn_readfirstlane(v);
    };

    auto fetch_response = [&](Staged& st, int ti) __attribute__((always_inline)) {
        const int base = ti * kKeyTile;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = min(base + RPI * i + srow, total - 1);
            const uint32_t ent = s_list.ent[e];
            const int s = s0 + (int)(ent >> 16);
            const int slot = (int)((ent >> 8) & 0xffu);
            // one load per operand through a selected pointer (two loads under
            // divergent branches would have to wait for each other)
            const bool is_new = have_new && s == p.T - 1;
            const size_t off_new = ((size_t)(b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
            const size_t off_old = (((size_t)s * N + b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
            const _Float16* const kp = is_new ? p.k_new + off_new : p.resp_k + off_old;
            const _Float16* const vp = is_new ? p.v_new + off_new : p.resp_v + off_old;
            st.k[i] = load16_stream(kp);
            st.v[i] = load16_stream(vp);
        }
    };
    auto fetch = [&](Staged& st, int ti) __attribute__((always_inline)) {
        if (ti < n_ptiles)      fetch_prompt(st, ti);
        else if (ti < n_tiles)  fetch_response(st, ti - n_ptiles);
        else                    fetch_dummy(st);
    };
    auto process = [&](int ti) __attribute__((always_inline)) {
        if (ti < n_ptiles) {
            const int base = k0 + ti * kKeyTile;
            const bool plain = (p.slopes == nullptr) && (base + kKeyTile <= k1);
            compute_tile(plain ? 0 : 1, base, 0);
        } else {
            compute_tile(2, (ti - n_ptiles) * kKeyTile, total);
        }
    };

    // DEPTH tiles are in flight per wave, each in its own named register set.
    Staged st_a, st_b;
    const int n_static = has_resp ? NW - 1 : NW;       // waves with static first tiles
    int ta = wave;                                     // static first tiles (not for the builder)
    int tb = wave + n_static;
    if (tid == 0) {
        s_next_tile = DEPTH * n_static;
        s_list.ready = 0;
    }
    // the first tiles need nothing but addresses when they are prompt tiles
    const bool early_a = !is_builder && ta < n_ptiles;
    const bool early_b = DEPTH > 1 && !is_builder && tb < n_ptiles;
    if (early_a) fetch_prompt(st_a, ta);
    if (early_b) fetch_prompt(st_b, tb);
    // Q tile to LDS: requested before the tiles above, so waiting for it leaves
    // them in flight
#pragma unroll
    for (int c = 0; c < QCH; ++c) {
        const int i = tid + c * NT;
        if (i < kQueryTile * CPR)
            *reinterpret_cast<u32x4_t*>(s_q + (i / CPR) * ROWB + ((i % CPR) << 4)) = qw[c];
    }
    if (appends) {
        store16(p.resp_k + app_dst, app_k);
        store16(p.resp_v + app_dst, app_v);
    }
    __syncthreads();                                   // Q tile, tile counter, list flag visible
    SEGKV_STAMP(1);
    if (is_builder) {
        build_response_list_wave(s_list, p.parent, (g == 0 && qb == 0) ? p.anc_out : nullptr, p.B,
                                 p.W, p.T, b, s0, s1, lrows, lane);
        need_list();
        SEGKV_STAMP(2);
        ta = claim_tile();
        if (DEPTH > 1) tb = claim_tile();
    }
    if (!early_a) {
        if (ta >= n_ptiles) need_list();
        fetch(st_a, ta);
    }
    if (DEPTH > 1 && !early_b) {
        if (tb >= n_ptiles) need_list();
        fetch(st_b, tb);
    }
    SEGKV_PHASE_BEGIN;
    // One turn: the set's tile has landed -> LDS, the set is refilled with the
    // next claimed tile, the tile in LDS is multiplied.
    auto turn = [&](Staged& st, int& ti) __attribute__((always_inline)) {
        stage_to_lds(st);
        SEGKV_STAMP_FIRST(3);
        const int nxt = claim_tile();
        if (nxt >= n_ptiles) need_list();
        fetch(st, nxt);
        SEGKV_PHASE(0);
        process(ti);
        ti = nxt;
    };
    // claims only grow, so the first set that runs dry ends the stream
    if (DEPTH == 1) {
        while (ta < n_tiles) turn(st_a, ta);
    } else {
        while (true) {
            if (ta >= n_tiles) break;
            turn(st_a, ta);
            if (tb >= n_tiles) break;
            turn(st_b, tb);
        }
    }
    SEGKV_PHASE_DUMP;

    SEGKV_STAMP(4);
    // ---- merge the waves through LDS (each wave reuses its own tile region) ----
    l_part += __shfl_xor(l_part, 32);
    float* const mrg = reinterpret_cast<float*>(region);
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4_t v4 = {o_acc[db][4 * i + 0], o_acc[db][4 * i + 1], o_acc[db][4 * i + 2],
                           o_acc[db][4 * i + 3]};
            *reinterpret_cast<float4_t*>(mrg + n * MROW + 32 * db + 8 * i + 4 * h) = v4;
        }
    if (h == 0) {
        s_ml[wave][n][0] = m_ref;
        s_ml[wave][n][1] = l_part;
    }
    __syncthreads();
    SEGKV_STAMP(5);

    const int NQ = N * p.Hq;
    const int nq_here = min(kQueryTile, p.nq - qb * kQueryTile);
    for (int idx = tid; idx < nq_here * (D / 4); idx += NT) {
        const int qn = idx / (D / 4);
        const int d4 = (idx % (D / 4)) * 4;
        float mm = s_ml[0][qn][0];
#pragma unroll
        for (int w = 1; w < NW; ++w) mm = fmaxf(mm, s_ml[w][qn][0]);
        float ll = 0.0f;
        float4_t aa = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = fast_exp2(s_ml[w][qn][0] - mm);
            ll += s_ml[w][qn][1] * f;
            const float4_t a = *reinterpret_cast<const float4_t*>(
                reinterpret_cast<const float*>(s_region + w * REGIONB) + qn * MROW + d4);
            aa += a * f;
        }
        const int lqn = qb * kQueryTile + qn;
        const int j = lqn / p.G;
        const int hqn = g * p.G + (lqn % p.G);
        const size_t row = (size_t)(b * p.W + j) * p.Hq + hqn;
        if (direct_out) {
            const float inv = 1.0f / ll;
            half4_t o;
            o.x = (_Float16)(aa.x * inv);
            o.y = (_Float16)(aa.y * inv);
            o.z = (_Float16)(aa.z * inv);
            o.w = (_Float16)(aa.w * inv);
            *reinterpret_cast<half4_t*>(p.out + row * D + d4) = o;
        } else {
            *reinterpret_cast<float4_t*>(p.ws_acc + ((size_t)chunk * NQ + row) * D + d4) = aa;
            if (d4 == 0) {
                p.ws_ml[((size_t)chunk * NQ + row) * 2 + 0] = mm;
                p.ws_ml[((size_t)chunk * NQ + row) * 2 + 1] = ll;
            }
        }
    }
    SEGKV_STAMP(6);
}

// ---------------------------------------------------------------------------
// Host-side launcher
// ---------------------------------------------------------------------------
template <int D, int NW, int DEPTH>
static void launch_variant(const SdpaParams& p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((sdpa_decode_mfma_kernel<D, NW, DEPTH>), dim3(grid), dim3(NW * 64), 0, st, p);
}

hipError_t launch_sdpa_decode_mfma(const SdpaParams& p, int D, unsigned grid, hipStream_t st)
{
    const char* v = std::getenv("SEGKV_MFMA_VARIANT");   // A/B measurements: "<waves><depth>"
    const int var = v ? std::atoi(v) : 0;
    switch (D) {
        case 64:  launch_variant<64, kMfmaWaves64, 1>(p, grid, st); break;
        case 128:
            if (var == 42)      launch_variant<128, 4, 2>(p, grid, st);
            else if (var == 41) launch_variant<128, 4, 1>(p, grid, st);
            else if (var == 82) launch_variant<128, 8, 2>(p, grid, st);
            else                launch_variant<128, kMfmaWaves128, 1>(p, grid, st);
            break;
        case 256: launch_variant<256, kMfmaWaves256, 1>(p, grid, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace segkv
