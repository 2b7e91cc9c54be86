// libsegkv device code: fused decode-step attention over a segment KV cache
// (arxiv 2401.05391, Section 3.3) for gfx950, matrix-core (MFMA) path.
//
// The queries that share every K/V row of a unit (request b, KV head g) -- the W
// beams and, under grouped-query attention, the G query heads of the group; a
// single query in greedy decode -- are the N dimension of the MFMAs, a tile of
// keys is M:
//     S^T[key][query]  = K[key][:]   . Q^T[:][query]       (contraction over D)
//     O^T[d][query]   += V^T[d][key] . P^T[key][query]     (contraction over keys)
// so that each K/V row is read from HBM once and reused by all queries.
// Two shapes: QT = 32 query slots on 32x32x16 MFMAs (beams x grouped heads), and
// QT = 16 slots on 16x16x32 / 16x16x16 MFMAs (beam search without grouping: few
// queries, half the accumulator registers, head dimension up to 256).
//
// Each wave streams its own key tiles (dealt round-robin), with no work-group
// barrier in the loop:
//   global (coalesced 128-bit, non-temporal) -> registers -> wave-private LDS
//   tile (rows padded by 16 bytes against bank conflicts) -> MFMA operands.
// While a tile is being multiplied the next one is already in flight in
// registers.  The last wave first resolves the beam lineage into the list of
// response rows, newest steps first, publishing it window by window; the
// others take the response tiles from the newest end as they become available,
// and deal the first rounds of tiles among themselves while the builder is
// busy.  Softmax statistics are fp32; P is rounded to fp16 for the PV product;
// the running maximum is only moved when a tile exceeds it by 2^8 so that the
// accumulator rescale is rare.  Waves are merged through LDS at the end.
#include "segkv_common.h"
#include "segkv_launch.h"
#include "segkv_device.h"
#include "segkv_mfma_tile.h"

namespace segkv {

// Tile geometry of the decode kernel for head dimension D and QT query slots.
// A wave's tile is 16 KB of K plus V rows: 32 keys, or 16 keys at D = 256.
template <int D, int QT>
struct DecodeGeometry {
    static constexpr int KT = (D == 256) ? 16 : 32;   // keys per tile
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;              // rows per staging load instruction
    static constexpr int NLD = KT / RPI;              // staging loads per operand per tile
    // Row pitch 2D+16 bytes = 16 mod 256: the 16 (or 32) consecutive rows that read
    // the same 16-byte column as MFMA operands fall into different bank groups.
    static constexpr int ROWB = D * 2 + 16;
    static constexpr int TILEB = KT * ROWB;           // bytes of a K (or V) tile
    static constexpr int MROW = D + 4;                // floats per query row in the merge layout
    static constexpr int MERGEB = QT * MROW * 4;
    static constexpr int REGIONB = (2 * TILEB > MERGEB) ? 2 * TILEB : MERGEB;   // per wave
    static_assert(QT == 32 || QT == 16, "query slots per work-group");
    static_assert(QT == 16 || KT == 32, "the 32-slot shape multiplies 32-key tiles");
};

// PAIR: every 2D-byte row holds TWO adjacent KV heads of D/2 elements each (a
// D/2 = 64 multi-head model seen as rows of 128): one work-group serves both
// heads, so that K/V rows are fetched in 256-byte instead of 128-byte pieces
// (measured +10-20% of HBM bandwidth).  Q, K, V and the output have the same
// memory layout either way; the products are block-diagonal (each head contracts
// over its own half of the row) and every head keeps its own softmax state.
template <int D, int NW, int QT, bool SHARED, bool PAIR = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void sdpa_decode_mfma_kernel(SdpaParams p)
{
    using Geo = DecodeGeometry<D, QT>;
    constexpr int KT = Geo::KT, CPR = Geo::CPR, RPI = Geo::RPI, NLD = Geo::NLD;
    constexpr int ROWB = Geo::ROWB, VROWB = Geo::ROWB, TILEB = Geo::TILEB, MROW = Geo::MROW;
    constexpr int REGIONB = Geo::REGIONB;
    constexpr int NT = NW * 64;
    constexpr bool WIDE = (QT == 32);
    // accumulator registers per lane: O^T is D x QT fp32 over 64 lanes
    constexpr int NOB = WIDE ? D / 32 : D / 16;        // blocks of the PV product
    constexpr int OBR = WIDE ? 16 : 4;                 // registers per block
    constexpr int NSR = WIDE ? 16 : (KT / 16) * 4;     // S^T registers per lane, tile and head
    constexpr int NH = PAIR ? 2 : 1;                   // heads per row
    constexpr int DH = D / NH;                         // elements per head
    static_assert(!PAIR || (!WIDE && D == 128), "head pairs: 16-slot shape, 64-element heads");

    __shared__ __align__(16) unsigned char s_region[NW * REGIONB];
    __shared__ __align__(16) unsigned char s_q[QT * ROWB];   // Q^T operand, shared by the waves
    constexpr int LISTCAP = mfma_list_capacity(D, QT, NW, PAIR ? 2 : 1);
    static_assert(LISTCAP >= 64, "no room for a response list");
    __shared__ WaveListSmem<LISTCAP> s_list;
    __shared__ float s_ml[NW][NH][QT][2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: tile indices stay uniform
    // MFMA lane roles.  32-slot shape: lane = n + 32 h (n: query column / key row /
    // d within a block, h: which 8 of the 16 contraction slots).  16-slot shape:
    // lane = n + 16 h (h = 0..3: which quarter of the contraction slots).
    const int n = WIDE ? (lane & 31) : (lane & 15);
    const int h = WIDE ? (lane >> 5) : (lane >> 4);
    const int srow = lane / CPR;    // staging: row within a load instruction
    const int schunk = lane % CPR;  // staging: 16-byte chunk of the row

    // ---- which work item ----
    // Hardware order (group i runs on XCD i % 8): with the KV head as the fastest
    // index each XCD streams one 256-byte column class of every request.  Measured
    // 2% faster on MI355X than giving each XCD a contiguous run of requests.
    // The query blocks of one unit read the same K/V rows: they get work-group
    // indices 8 apart, i.e. the same XCD at about the same time, so that the
    // re-reads are served by that XCD's L2 (and K/V loads are then ordinary, not
    // non-temporal, loads).
    int id = (int)blockIdx.x;
    int qb = 0;
    if (SHARED) {
        const int nqb = p.n_qblocks;
        const int n_units = (int)gridDim.x / nqb;
        const int full = (n_units / 8) * 8 * nqb;
        if (id < full) {
            const int r = id % (8 * nqb);
            qb = r / 8;
            id = (id / (8 * nqb)) * 8 + (r % 8);
        } else {
            const int r = id - full;
            qb = r % nqb;
            id = (n_units / 8) * 8 + r / nqb;
        }
    }
    // Which KV head: consecutive indices are consecutive heads, and within every
    // aligned run of eight (one per XCD) the planner may permute them so that the
    // heads whose K/V columns are served more slowly run on the faster XCDs
    // (identity when it has no reason to).
    const int g0 = id % p.Hkv;       id /= p.Hkv;
    const int g = (g0 & ~7) | (int)((p.head_perm8 >> (4 * (g0 & 7))) & 7u);
    const int chunk = id % p.n_chunks;
    const int b = id / p.n_chunks;
    const int N = p.B * p.W;

    // valid prompt rows of this request (a padded batch passes per-request lengths)
    const int Lp = p.prompt_lens ? min(max(p.prompt_lens[b], 0), p.Lp) : p.Lp;
    int k0 = 0, k1 = 0, s0 = 0, s1 = 0;
    if (p.merged) {
        k1 = Lp;
        s1 = p.T;
    } else if (chunk < p.n_rchunks) {
        s0 = chunk * p.rchunk;
        s1 = min(s0 + p.rchunk, p.T);
    } else {
        k0 = min((chunk - p.n_rchunks) * p.pchunk, Lp);
        k1 = min(k0 + p.pchunk, Lp);
        if (p.resp_in_last && chunk == p.n_chunks - 1) s1 = p.T;
    }
    const bool direct_out = (p.n_chunks == 1);

    unsigned char* const region = s_region + wave * REGIONB;
    unsigned char* const k_tile = region;
    unsigned char* const v_tile = region + TILEB;      // K tile first, then the V tile

    // ---- queries of this block: staged once into LDS in the same padded row
    // layout as the key tiles; every wave reads its QK^T B operand from there ----
    const int lq = qb * QT + n;
    const bool q_valid = lq < p.nq;
    const int lqc = q_valid ? lq : (p.nq - 1);
    const int qbeam = lqc / p.G;
    const int hq = g * p.G + (lqc % p.G);
    float slope2[NH];
#pragma unroll
    for (int hd = 0; hd < NH; ++hd) slope2[hd] = p.slopes ? p.slopes[NH * hq + hd] * kLog2e : 0.0f;
    const int qpos = Lp + p.T - 1;
    // Requests that later steps depend on go out first, in this order: the Q
    // chunks this thread stages, its row of the parent table, then (below) the
    // wave's first key tile.  They are consumed in the same order, so each wait
    // leaves the younger requests in flight.
    constexpr int QCH = (QT * CPR + NT - 1) / NT;
    u32x4_t qw[QCH];
#pragma unroll
    for (int c = 0; c < QCH; ++c) {
        const int i = tid + c * NT;
        const int qn = i / CPR;
        const int ch = i % CPR;
        const int lqn = qb * QT + qn;
        qw[c] = u32x4_t{0u, 0u, 0u, 0u};               // unused query slots multiply as zeros
        if (i < QT * CPR && lqn < p.nq) {
            const size_t row = (size_t)(b * p.W + lqn / p.G) * p.Hq + g * p.G + (lqn % p.G);
            qw[c] = load16(p.q + row * D + ch * 8);
        }
    }
    // One wave (the last) resolves the response list on its own while the others
    // stream prompt tiles; its parent rows are requested here, with the Q chunks.
    const bool has_resp = s1 > s0;                              // uniform over the work-group
    const bool is_builder = has_resp && wave == NW - 1;         // uniform over the wave
    ListRows lrows;
    const bool from_lineage = p.lineage != nullptr && p.W > 1;  // the list is kept across steps
    if (is_builder && p.W > 1 && !from_lineage)
        load_list_rows(lrows, p.parent, N, p.W, p.T, b, list_last_window_start(s0, s1), lane);

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

    const uint32_t* const ent = s_list.ent;
    // ---- running state: reference max and partial sum per lane, O^T accumulators ----
    float m_ref[NH], l_part[NH];    // l_part: sum of p over this lane's keys of every tile
#pragma unroll
    for (int hd = 0; hd < NH; ++hd) {
        m_ref[hd] = kEmptyMax;
        l_part[hd] = 0.0f;
    }
    typedef float acc_t __attribute__((ext_vector_type(OBR)));
    acc_t o_acc[NOB];
#pragma unroll
    for (int ob = 0; ob < NOB; ++ob)
#pragma unroll
        for (int r = 0; r < OBR; ++r) o_acc[ob][r] = 0.0f;

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

    // One tile of KT keys.  `mode` (uniform) selects how S^T becomes base-2 logits:
    // 0 full prompt tile without positional bias, 1 prompt tile with masking of
    // the tail and ALiBi, 2 response tile (per-row beam masks and positions).
    // Register r of S^T holds, for this lane's query, the key at tile row
    //   32-slot shape: 8 (r / 4) + 4 h + (r % 4)
    //   16-slot shape: 16 (r / 4) + 4 h + (r % 4)
    auto key_row = [&](int r) { return (WIDE ? 8 : 16) * (r >> 2) + 4 * h + (r & 3); };
    auto compute_tile = [&](int mode, int base, int lo) __attribute__((always_inline)) {
        // the tile was written to LDS by this wave's own lanes in staging layout
        wave_lds_exchange_point();
        // S^T = K . Q^T
        float s[NH][NSR];
        if constexpr (WIDE) {
            float16_t acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < D / 16; ++t) {
                const int off = n * ROWB + ((2 * t + h) << 4);
                const half8_t a = *reinterpret_cast<const half8_t*>(k_tile + off);
                const half8_t bq = *reinterpret_cast<const half8_t*>(s_q + off);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bq, acc, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) s[0][r] = acc[r];
        } else {
            // 16 keys x 16 queries per MFMA, 32 head-dim elements per step; a head
            // contracts over its own DH / 32 steps of the row
#pragma unroll
            for (int kb = 0; kb < KT / 16; ++kb) {
#pragma unroll
                for (int hd = 0; hd < NH; ++hd) {
                    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int t = hd * (DH / 32); t < (hd + 1) * (DH / 32); ++t) {
                        const int col = (4 * t + h) << 4;
                        const half8_t a =
                            *reinterpret_cast<const half8_t*>(k_tile + (16 * kb + n) * ROWB + col);
                        const half8_t bq = *reinterpret_cast<const half8_t*>(s_q + n * ROWB + col);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq, acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) s[hd][4 * kb + r] = acc[r];
                }
            }
        }
        // logits, tile maximum for this lane's query; P = 2^(z - m_ref), fp16 for the
        // PV product -- per head of the row
        _Float16 ph[NH][NSR];
#pragma unroll
        for (int hd = 0; hd < NH; ++hd) {
            float m_tile = -INFINITY;
            if (mode == 0) {
#pragma unroll
                for (int r = 0; r < NSR; ++r) {
                    s[hd][r] *= p.scale2;
                    m_tile = fmaxf(m_tile, s[hd][r]);
                }
            } else if (mode == 1) {
#pragma unroll
                for (int r = 0; r < NSR; ++r) {
                    const int kpos = base + key_row(r);
                    const float z = s[hd][r] * p.scale2 + slope2[hd] * (float)(kpos - qpos);
                    s[hd][r] = kpos < k1 ? z : -INFINITY;
                    m_tile = fmaxf(m_tile, s[hd][r]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < NSR; ++r) {
                    const int e = base + key_row(r);
                    const uint32_t en = ent[max(e, lo)];
                    const int kpos = Lp + s0 + (int)(en >> 16);
                    const float z = s[hd][r] * p.scale2 + slope2[hd] * (float)(kpos - qpos);
                    const bool vis = (e >= lo) && ((en >> qbeam) & 1u);
                    s[hd][r] = vis ? z : -INFINITY;
                    m_tile = fmaxf(m_tile, s[hd][r]);
                }
            }
            // Move the reference maximum only when a tile exceeds it by the slack.  The
            // lanes that share a query hold different keys, but the vote is wave-wide, so
            // their maxima need to be exchanged only when the reference does move.
            if (__any(m_tile > m_ref[hd] + kRescaleSlack)) {
                if constexpr (!WIDE) m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16));
                m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
                const float m_new = fmaxf(m_ref[hd], m_tile);
                const float corr = fast_exp2(m_ref[hd] - m_new);
                m_ref[hd] = m_new;
                l_part[hd] *= corr;
#pragma unroll
                for (int ob = hd * (NOB / NH); ob < (hd + 1) * (NOB / NH); ++ob)
#pragma unroll
                    for (int r = 0; r < OBR; ++r) o_acc[ob][r] *= corr;
            }
#pragma unroll
            for (int r = 0; r < NSR; ++r) {
                const float pr = fast_exp2(s[hd][r] - m_ref[hd]);
                l_part[hd] += pr;
                ph[hd][r] = (_Float16)pr;
            }
        }
        // O^T += V^T . P^T.  The A operand wants, per lane, several keys of one
        // head-dim column; the V tile is row-major [key][d].  ds_read_b64_tr_b16
        // does the transpose on the way out of LDS: a 16-lane group reads 4 rows x
        // 16 columns (lane i supplies row i/4, columns 4*(i%4)..+3) and lane i
        // receives column i of all 4 rows.
        const int li = lane & 15;
        if constexpr (WIDE) {
            // two reads give the 8 keys 16u + 8r + 4h + {0..3}, r = 0, 1, the keys
            // of S^T registers 8u .. 8u+7
            const int grp = lane >> 4;                 // 16-lane group: d half (grp&1), key half h
            const int tr_base = (4 * h + (li >> 2)) * VROWB + ((16 * (grp & 1) + 4 * (li & 3)) << 1);
#pragma unroll
            for (int ob = 0; ob < NOB; ++ob) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int off = tr_base + (16 * u) * VROWB + ob * 64;
                    const half4_t lo = lds_read_tr16(v_tile + off);
                    const half4_t hi = lds_read_tr16(v_tile + off + 8 * VROWB);
                    const half8_t a = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    const half8_t pb = {ph[0][8 * u + 0], ph[0][8 * u + 1], ph[0][8 * u + 2],
                                        ph[0][8 * u + 3], ph[0][8 * u + 4], ph[0][8 * u + 5],
                                        ph[0][8 * u + 6], ph[0][8 * u + 7]};
                    o_acc[ob] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb, o_acc[ob], 0, 0, 0);
                }
                // keep the operand reads of later blocks from piling up in registers
                if (NOB > 4) __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // 16 head-dim columns x 16 queries per MFMA, contraction over the 16 keys
            // of block kb: one read gives keys 16 kb + 4 h + {0..3}, the keys of S^T
            // registers 4 kb .. 4 kb + 3
            const int tr_base = (4 * h + (li >> 2)) * VROWB + ((4 * (li & 3)) << 1);
#pragma unroll
            for (int kb = 0; kb < KT / 16; ++kb) {
#pragma unroll
                for (int ob = 0; ob < NOB; ++ob) {
                    constexpr int kBlocksPerHead = NOB / NH;       // output blocks of one head
                    const int hd = ob / kBlocksPerHead;
                    const half4_t pb = {ph[hd][4 * kb + 0], ph[hd][4 * kb + 1], ph[hd][4 * kb + 2],
                                        ph[hd][4 * kb + 3]};
                    const half4_t a = lds_read_tr16(v_tile + tr_base + (16 * kb) * VROWB + ob * 32);
                    o_acc[ob] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, pb, o_acc[ob], 0, 0, 0);
                }
            }
        }
    };

    // ---- one tile stream per work-group: prompt tiles first (Section 3.3: loop
    // over the prompt keys), then the response tiles (index select fused: rows
    // chosen by the beam lineage), dealt to the waves round-robin.  Each wave keeps one
    // tile in flight in registers while it computes the previous one.  A fetch is
    // never skipped: past the end of the stream it is pointed at one row that is
    // already cached, so that the code is free of conditional loads and every
    // wait covers exactly the tile it needs. ----
    const int n_ptiles = (k1 > k0) ? (k1 - k0 + KT - 1) / KT : 0;
    const _Float16* const dummy = p.q + (size_t)b * p.W * p.Hq * D + schunk * 8;
    // Prompt tiles are addressed as (scalar tile base) + (32-bit lane offset):
    // the lane offsets are the same for every full tile, so no per-load 64-bit
    // address has to be kept in registers.
    const uint32_t row_stride = p.prompt_row_stride;   // elements between consecutive keys
    auto fetch_prompt = [&](Staged& st, int ti) __attribute__((always_inline)) {
        const int base = k0 + ti * KT;
        const int lim = min(KT - 1, k1 - 1 - base);          // last valid row of the tile
        const size_t tile_off = (size_t)b * p.prompt_req_stride + (size_t)base * row_stride + g * D;
        const _Float16* const kb = p.prompt_k + tile_off;
        const _Float16* const vb = p.prompt_v + tile_off;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const uint32_t off = (uint32_t)min(RPI * i + srow, lim) * row_stride + schunk * 8;
            st.k[i] = SHARED ? load16(kb + off) : load16_stream(kb + off);
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const uint32_t off = (uint32_t)min(RPI * i + srow, lim) * row_stride + schunk * 8;
            st.v[i] = SHARED ? load16(vb + off) : load16_stream(vb + off);
        }
    };
    auto fetch_dummy = [&](Staged& st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) st.k[i] = load16(dummy);
#pragma unroll
        for (int i = 0; i < NLD; ++i) st.v[i] = load16(dummy);
    };

    // The response list comes from the builder wave, which fills s_list.ent from
    // the top down, newest window of steps first, and publishes how far it has
    // got after each window.  Response tile j is ent[LISTCAP - KT (j+1) .. LISTCAP
    // - KT j): the waves take the tiles of the newest steps while the builder is
    // still composing the older ones.  Until the list is final the number of
    // tiles is unknown (n_tiles is an upper bound); a wave asks for tile j just
    // before it requests that tile's rows.
    int lo = LISTCAP;                                  // ent[lo .. LISTCAP) is known to be written
    int n_tiles = has_resp ? (1 << 30) : n_ptiles;
    bool list_final = !has_resp;
    auto need_tile = [&](int j) {
        if (!list_final) {
            lo = wait_response_list(s_list, LISTCAP - KT * (j + 1), list_final);
            if (list_final) n_tiles = n_ptiles + (LISTCAP - lo + KT - 1) / KT;
        }
    };
    auto fetch_response = [&](Staged& st, int j) __attribute__((always_inline)) {
        const int base = LISTCAP - KT * (j + 1);
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = max(base + RPI * i + srow, lo);
            const uint32_t en = ent[e];
            const int s = s0 + (int)(en >> 16);
            const int slot = (int)((en >> 8) & 0xffu);
            // one load per operand through a selected pointer (two loads under
            // divergent branches would have to wait for each other)
            const bool is_new = have_new && s == p.T - 1;
            const size_t off_new = ((size_t)(b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
            const size_t off_old = (((size_t)s * N + b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
            const _Float16* const kp = is_new ? p.k_new + off_new : p.resp_k + off_old;
            const _Float16* const vp = is_new ? p.v_new + off_new : p.resp_v + off_old;
            st.k[i] = SHARED ? load16(kp) : load16_stream(kp);
            st.v[i] = SHARED ? load16(vp) : load16_stream(vp);
        }
    };
    auto fetch = [&](Staged& st, int ti) __attribute__((always_inline)) {
        if (ti < n_ptiles)      fetch_prompt(st, ti);
        else if (ti < n_tiles)  fetch_response(st, ti - n_ptiles);
        else                    fetch_dummy(st);
    };
    auto process = [&](int ti) __attribute__((always_inline)) {
        if (ti < n_ptiles) {
            const int base = k0 + ti * KT;
            const bool plain = (p.slopes == nullptr) && (base + KT <= k1);
            compute_tile(plain ? 0 : 1, base, 0);
        } else {
            compute_tile(2, LISTCAP - KT * (ti - n_ptiles + 1), lo);
        }
    };

    // Tiles are dealt in a fixed order, round-robin over the waves.  (Claiming
    // them from a shared counter measured within 1% of this, and a fixed deal
    // keeps the result bit-identical from run to run.)
    Staged st;
    // While the builder wave composes the list the other NW-1 waves deal the
    // tiles among themselves; it joins the deal after `skip` rounds (a window of
    // the list costs it about two rounds; measured best among 0 .. 2 per window).
    const int n_win = (s1 - s0 + kListWindow - 1) / kListWindow;
    const int skip = (has_resp && p.W > 1) ? (from_lineage ? 1 : 2 * n_win - 1) : 0;
    const int t_join = skip * (NW - 1);
    int ti = wave < NW - 1 ? wave : t_join + NW - 1;
    if (tid == 0) {
        s_list.ready = 0;
        s_list.top = LISTCAP;
    }
    // the first tile needs nothing but addresses when it is a prompt tile
    const bool early = !is_builder && ti < n_ptiles;
    if (early) fetch_prompt(st, ti);
    // Q tile to LDS: requested before the tile above, so waiting for it leaves
    // the tile in flight
#pragma unroll
    for (int c = 0; c < QCH; ++c) {
        const int i = tid + c * NT;
        if (i < QT * CPR)
            *reinterpret_cast<u32x4_t*>(s_q + (i / CPR) * ROWB + ((i % CPR) << 4)) = qw[c];
    }
    if (appends) {
        store16(p.resp_k + app_dst, app_k);
        store16(p.resp_v + app_dst, app_v);
    }
    __syncthreads();                                   // Q tile and list flag visible
    if (is_builder && from_lineage) {
        load_response_list_wave(s_list, p.lineage + (size_t)b * p.lineage_stride,
                                p.lineage_stride - kLineageHeaderWords, p.W, p.T, s0, s1, lane);
        need_tile(0);
    } else if (is_builder) {
        build_response_list_wave(s_list, p.parent, (g == 0 && qb == 0) ? p.anc_out : nullptr, p.B,
                                 p.W, p.T, b, s0, s1, lrows, lane);
        need_tile(0);                                  // final: this wave has just built it
    }
    if (!early) {
        if (ti >= n_ptiles) need_tile(ti - n_ptiles);
        fetch(st, ti);
    }
    // One turn: the tile has landed -> LDS, the registers are refilled with the
    // wave's next tile, the tile in LDS is multiplied.  (Two tiles in flight per
    // wave measured slower: the CU's outstanding-load limit, not the wave's, binds.)
    while (ti < n_tiles) {
        stage_to_lds(st);
        const int nxt = ti + (ti < t_join ? NW - 1 : NW);
        if (nxt >= n_ptiles) need_tile(nxt - n_ptiles);
        fetch(st, nxt);
        process(ti);
        ti = nxt;
    }

    // ---- merge the waves through LDS (each wave reuses its own tile region) ----
#pragma unroll
    for (int hd = 0; hd < NH; ++hd) {
        l_part[hd] += __shfl_xor(l_part[hd], 32);
        if constexpr (!WIDE) l_part[hd] += __shfl_xor(l_part[hd], 16);
    }
    float* const mrg = reinterpret_cast<float*>(region);
    // register j of block ob is O^T[d][n] with d = (WIDE ? 32 ob + 8 (j/4) + 4 h : 16 ob + 4 h) + j%4
#pragma unroll
    for (int ob = 0; ob < NOB; ++ob)
#pragma unroll
        for (int i = 0; i < OBR / 4; ++i) {
            float4_t v4 = {o_acc[ob][4 * i + 0], o_acc[ob][4 * i + 1], o_acc[ob][4 * i + 2],
                           o_acc[ob][4 * i + 3]};
            const int d0 = WIDE ? 32 * ob + 8 * i + 4 * h : 16 * ob + 4 * h;
            *reinterpret_cast<float4_t*>(mrg + n * MROW + d0) = v4;
        }
    if (h == 0) {
#pragma unroll
        for (int hd = 0; hd < NH; ++hd) {
            s_ml[wave][hd][n][0] = m_ref[hd];
            s_ml[wave][hd][n][1] = l_part[hd];
        }
    }
    __syncthreads();

    const int NQ = N * p.Hq;
    const int nq_here = min(QT, p.nq - qb * QT);
    for (int idx = tid; idx < nq_here * (D / 4); idx += NT) {
        const int qn = idx / (D / 4);
        const int d4 = (idx % (D / 4)) * 4;
        const int hd = d4 / DH;                         // which head of the row these columns belong to
        float mm = s_ml[0][hd][qn][0];
#pragma unroll
        for (int w = 1; w < NW; ++w) mm = fmaxf(mm, s_ml[w][hd][qn][0]);
        float ll = 0.0f;
        float4_t aa = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = fast_exp2(s_ml[w][hd][qn][0] - mm);
            ll += s_ml[w][hd][qn][1] * f;
            const float4_t a = *reinterpret_cast<const float4_t*>(
                reinterpret_cast<const float*>(s_region + w * REGIONB) + qn * MROW + d4);
            aa += a * f;
        }
        const int lqn = qb * QT + qn;
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
            if (d4 % DH == 0) {                         // one (m, l) pair per query and head
                p.ws_ml[(((size_t)chunk * NQ + row) * NH + hd) * 2 + 0] = mm;
                p.ws_ml[(((size_t)chunk * NQ + row) * NH + hd) * 2 + 1] = ll;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host-side launcher
// ---------------------------------------------------------------------------
template <int D, int NW, int QT>
static hipError_t launch_variant(const SdpaParams& p, unsigned grid, hipStream_t st)
{
    if constexpr (D == 128 && QT == 16) {
        if (p.head_pairs)       // planner: never with several query blocks
            return SEGKV_LAUNCH((sdpa_decode_mfma_kernel<D, NW, QT, false, true>), dim3(grid),
                                dim3(NW * 64), st, p);
    }
    // several query blocks per unit: the variant whose blocks share K/V rows through L2
    if (p.n_qblocks > 1)
        return SEGKV_LAUNCH((sdpa_decode_mfma_kernel<D, NW, QT, true>), dim3(grid), dim3(NW * 64), st, p);
    return SEGKV_LAUNCH((sdpa_decode_mfma_kernel<D, NW, QT, false>), dim3(grid), dim3(NW * 64), st, p);
}

hipError_t launch_sdpa_decode_mfma(const SdpaParams& p, int D, int QT, int NW, unsigned grid,
                                   hipStream_t st)
{
    if ((QT != 16 && QT != 32) || (NW != 8 && NW != 4)) return hipErrorInvalidValue;
    if (NW == 4 && (QT != 16 || D > 128)) return hipErrorInvalidValue;
    switch (D) {
        case 64:
            if (QT == 32) return launch_variant<64, 8, 32>(p, grid, st);
            if (NW == 8)  return launch_variant<64, 8, 16>(p, grid, st);
            return launch_variant<64, 4, 16>(p, grid, st);
        case 128:
            if (QT == 32) return launch_variant<128, 8, 32>(p, grid, st);
            if (NW == 8)  return launch_variant<128, 8, 16>(p, grid, st);
            return launch_variant<128, 4, 16>(p, grid, st);
        case 256:
            if (QT == 32) return hipErrorInvalidValue;   // accumulators would not fit: planner uses 16
            return launch_variant<256, 8, 16>(p, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace segkv
