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

namespace segkv {

constexpr int kKeyTile = 32;          // keys per MFMA tile (M)
constexpr int kQueryTile = 32;        // query slots per work-group (N)
constexpr float kRescaleSlack = 8.0f; // log2 units a tile may exceed the reference max

template <int D>
struct MfmaGeometry {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;              // rows per staging load instruction
    static constexpr int NLD = kKeyTile / RPI;        // staging loads per operand per tile
    static constexpr int NKS = D / 16;                // k-steps of the QK^T product
    static constexpr int NDB = D / 32;                // 32-wide head-dim blocks of the PV product
    // Bytes per row of an LDS tile: 16 bytes of padding make the row pitch
    // 16 mod 64, so that 16 consecutive rows read at the same column (QK^T
    // operand) and rows 4 apart read 64 bytes wide (PV operand) fall into
    // different banks, while every address stays "lane base + constant".
    static constexpr int ROWB = D * 2 + 16;
    static constexpr int TILEB = kKeyTile * ROWB;     // bytes per operand tile
    static constexpr int MROW = D + 4;                // floats per query row in the merge layout
    static constexpr int MERGEB = kQueryTile * MROW * 4;
    static constexpr int REGIONB = (2 * TILEB > MERGEB) ? 2 * TILEB : MERGEB;  // per wave
};

template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void sdpa_decode_mfma_kernel(SdpaParams p)
{
    using Geo = MfmaGeometry<D>;
    constexpr int CPR = Geo::CPR, RPI = Geo::RPI, NLD = Geo::NLD, NKS = Geo::NKS, NDB = Geo::NDB;
    constexpr int ROWB = Geo::ROWB, TILEB = Geo::TILEB, MROW = Geo::MROW, REGIONB = Geo::REGIONB;
    constexpr int NT = NW * 64;
    static_assert(NT >= kListThreads, "the response list needs one thread per step");

    __shared__ __align__(16) unsigned char s_region[NW * REGIONB];
    __shared__ ResponseListSmem s_list;
    __shared__ float s_ml[NW][kQueryTile][2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = lane & 31;        // query slot (MFMA column) / key row (MFMA A row) / d within block
    const int h = lane >> 5;        // lane half: which 8 of the 16 contraction slots
    const int srow = lane / CPR;    // staging: row within a load instruction
    const int schunk = lane % CPR;  // staging: 16-byte chunk of the row

    // ---- which work item ----
    int id = blockIdx.x;
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
    unsigned char* const v_tile = region + TILEB;

    // ---- this lane's query: B operand of the QK^T product, kept in registers ----
    const int lq = qb * kQueryTile + n;
    const bool q_valid = lq < p.nq;
    const int lqc = q_valid ? lq : (p.nq - 1);
    const int qbeam = lqc / p.G;
    const int hq = g * p.G + (lqc % p.G);
    const size_t qidx = (size_t)(b * p.W + qbeam) * p.Hq + hq;
    const float slope2 = p.slopes ? p.slopes[hq] * kLog2e : 0.0f;
    const int qpos = p.Lp + p.T - 1;
    half8_t qreg[NKS];
#pragma unroll
    for (int t = 0; t < NKS; ++t) {
        u32x4_t w = load16(p.q + qidx * D + 16 * t + 8 * h);
        if (!q_valid) w = u32x4_t{0u, 0u, 0u, 0u};
        qreg[t] = __builtin_bit_cast(half8_t, w);
    }

    // ---- fused append: the block that owns step T-1 copies the unit's new rows ----
    const bool have_new = (p.k_new != nullptr);
    if (have_new && qb == 0 && s1 == p.T && s0 < s1) {
        constexpr int kVecPerRow = D / 8;
        const int total = p.W * kVecPerRow * 2;
        for (int i = tid; i < total; i += NT) {
            const int which = i / (p.W * kVecPerRow);
            const int rem = i % (p.W * kVecPerRow);
            const int u = rem / kVecPerRow;
            const int col = rem % kVecPerRow;
            const size_t src = ((size_t)(b * p.W + u) * p.Hkv + g) * D + col * 8;
            const size_t dst = (((size_t)(p.T - 1) * N + b * p.W + u) * p.Hkv + g) * D + col * 8;
            if (which == 0) store16(p.resp_k + dst, load16(p.k_new + src));
            else            store16(p.resp_v + dst, load16(p.v_new + src));
        }
    }

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
    auto stage_to_lds = [&](const Staged& st) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int row = RPI * i + srow;
            const int off = row * ROWB + (schunk << 4);
            *reinterpret_cast<u32x4_t*>(k_tile + off) = st.k[i];
            *reinterpret_cast<u32x4_t*>(v_tile + off) = st.v[i];
        }
    };

    // One tile of 32 keys: z_of(r, key) gives the masked base-2 logit for S^T register r.
    auto compute_tile = [&](auto&& logit_of) {
        // S^T = K . Q^T
        float16_t s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
        for (int t = 0; t < NKS; ++t) {
            const int off = n * ROWB + ((2 * t + h) << 4);
            const half8_t a = *reinterpret_cast<const half8_t*>(k_tile + off);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[t], s, 0, 0, 0);
        }
        // logits, tile maximum for this lane's query
        float m_tile = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r >> 2) + 4 * h + (r & 3);
            s[r] = logit_of(s[r], key);
            m_tile = fmaxf(m_tile, s[r]);
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
        // O^T += V^T . P^T
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int d = 32 * db + n;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                half8_t a;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = 16 * u + 8 * (e >> 2) + 4 * h + (e & 3);
                    const int off = key * ROWB + (d << 1);
                    a[e] = *reinterpret_cast<const _Float16*>(v_tile + off);
                }
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[u], o_acc[db], 0, 0, 0);
            }
            // keep the gathers of later blocks from being hoisted above this one:
            // their 16-bit loads would all be live at once
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prompt segment (Section 3.3: loop over the prompt keys) ----
    if (k1 > k0) {
        const int n_tiles = (k1 - k0 + kKeyTile - 1) / kKeyTile;
        auto fetch = [&](Staged& st, int ti) {
            const int base = k0 + ti * kKeyTile;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int row = min(base + RPI * i + srow, k1 - 1);
                const size_t off = (((size_t)b * p.Lp + row) * p.Hkv + g) * D + schunk * 8;
                st.k[i] = load16_stream(p.prompt_k + off);
                st.v[i] = load16_stream(p.prompt_v + off);
            }
        };
        Staged st;
        int ti = wave;
        if (ti < n_tiles) fetch(st, ti);
        for (; ti < n_tiles; ti += NW) {
            stage_to_lds(st);
            if (ti + NW < n_tiles) fetch(st, ti + NW);
            const int base = k0 + ti * kKeyTile;
            compute_tile([&](float dot, int key) {
                const int kpos = base + key;
                const float z = dot * p.scale2 + slope2 * (float)(kpos - qpos);
                return kpos < k1 ? z : -INFINITY;
            });
        }
    }

    // ---- response segment (index select fused: rows chosen by the beam lineage) ----
    if (s1 > s0) {
        build_response_list(s_list, p.parent, (g == 0 && qb == 0) ? p.anc_out : nullptr, p.B, p.W,
                            p.T, b, s0, s1);
        const int total = s_list.total;
        const int n_tiles = (total + kKeyTile - 1) / kKeyTile;
        auto fetch = [&](Staged& st, int ti) {
            const int base = ti * kKeyTile;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int e = min(base + RPI * i + srow, total - 1);
                const uint32_t ent = s_list.ent[e];
                const int s = s0 + (int)(ent >> 16);
                const int slot = (int)((ent >> 8) & 0xffu);
                const _Float16* kp;
                const _Float16* vp;
                if (have_new && s == p.T - 1) {
                    const size_t off = ((size_t)(b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
                    kp = p.k_new + off;
                    vp = p.v_new + off;
                } else {
                    const size_t off = (((size_t)s * N + b * p.W + slot) * p.Hkv + g) * D + schunk * 8;
                    kp = p.resp_k + off;
                    vp = p.resp_v + off;
                }
                st.k[i] = load16_stream(kp);
                st.v[i] = load16_stream(vp);
            }
        };
        Staged st;
        int ti = wave;
        if (ti < n_tiles) fetch(st, ti);
        for (; ti < n_tiles; ti += NW) {
            stage_to_lds(st);
            if (ti + NW < n_tiles) fetch(st, ti + NW);
            const int base = ti * kKeyTile;
            compute_tile([&](float dot, int key) {
                const int e = base + key;
                const uint32_t ent = s_list.ent[min(e, total - 1)];
                const int kpos = p.Lp + s0 + (int)(ent >> 16);
                const float z = dot * p.scale2 + slope2 * (float)(kpos - qpos);
                const bool vis = (e < total) && ((ent >> qbeam) & 1u);
                return vis ? z : -INFINITY;
            });
        }
    }

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
}

// ---------------------------------------------------------------------------
// Host-side launcher
// ---------------------------------------------------------------------------
hipError_t launch_sdpa_decode_mfma(const SdpaParams& p, int D, unsigned grid, hipStream_t st)
{
    switch (D) {
        case 64:
            hipLaunchKernelGGL((sdpa_decode_mfma_kernel<64, kMfmaWaves64>), dim3(grid),
                               dim3(kMfmaWaves64 * 64), 0, st, p);
            break;
        case 128:
            hipLaunchKernelGGL((sdpa_decode_mfma_kernel<128, kMfmaWaves128>), dim3(grid),
                               dim3(kMfmaWaves128 * 64), 0, st, p);
            break;
        case 256:
            hipLaunchKernelGGL((sdpa_decode_mfma_kernel<256, kMfmaWaves256>), dim3(grid),
                               dim3(kMfmaWaves256 * 64), 0, st, p);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace segkv
