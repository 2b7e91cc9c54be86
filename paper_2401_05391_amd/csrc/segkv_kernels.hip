// libsegkv device code: fused decode-step attention over a segment KV cache
// (arxiv 2401.05391, Section 3.3) for gfx950, vector-ALU path.
//
// Work decomposition
//   unit   = (request b, KV head g): the W*G queries (W beams x G grouped query
//            heads) that share every prompt K/V row of that head.
//   qblock = QB of those queries handled together by one work-group.
//   chunk  = a slice of the unit's keys: either a range of prompt positions or
//            a range of response steps.  With one chunk the work-group writes
//            the fp16 context itself; with more it writes an (m, l, acc)
//            partial per query and sdpa_merge_kernel combines them.
//   Inside a work-group the 4 waves take key tiles round-robin.  A wave reads
//   R = 64/LPR rows per 128-bit load (LPR lanes of 16 bytes cover one row
//   slice), keeps one online-softmax state per lane group, and the states are
//   merged across lane groups (shuffles) and waves (LDS) at the end.
//
// Response rows are visited through a compacted list of the distinct
// (step, slot) rows that some beam of the request descends from, each with the
// mask of beams that see it, so a row shared by several beams is read once.
#include "segkv_common.h"
#include "segkv_launch.h"
#include "segkv_device.h"

namespace segkv {

constexpr int kThreads = 256;          // work-group size of the vector-ALU kernel
constexpr int kWaves = kThreads / 64;
static_assert(kThreads >= kListThreads, "the response list needs one thread per step");

// Software pipeline over the tiles ti = first, first+kWaves, ... < n_tiles of one
// wave: the loads of the next tile are issued before the current one is
// consumed.  Two named buffers alternate (no register copies), and the steady
// state has no conditional fetch, so the wait before a consume only covers the
// tile it needs and leaves the newer loads in flight.
template <class Tile, class Fetch, class Consume>
__device__ __forceinline__ void stream_tiles_impl(Fetch& fetch, Consume& consume, int first,
                                                  int n_tiles)
{
    if (first >= n_tiles) return;
    int rem = (n_tiles - first + kWaves - 1) / kWaves;   // tiles of this wave not yet consumed
    int ti = first;
    Tile a, b;
    fetch(a, ti);
    while (rem >= 3) {
        fetch(b, ti + kWaves);
        consume(a);
        fetch(a, ti + 2 * kWaves);
        consume(b);
        ti += 2 * kWaves;
        rem -= 2;
    }
    if (rem == 2) {
        fetch(b, ti + kWaves);
        consume(a);
        consume(b);
    } else {
        consume(a);
    }
}

// ---------------------------------------------------------------------------
// Main kernel
// ---------------------------------------------------------------------------
// Lane geometry for head dimension D and HP KV heads per wave.  A wave-wide
// 128-bit load covers NG = 64/LPR row slices of LPR*16 bytes; HP of them are
// the same key row in HP adjacent KV heads (contiguous in memory, since the
// head index is the next-to-innermost dimension of every K/V tensor), the
// remaining factor R = NG/HP are consecutive key rows.
template <int D, int HP>
struct Geometry {
    static constexpr int LPR = (D >= 128) ? 16 : D / 8;   // lanes per row slice
    static constexpr int NV = D / (8 * LPR);              // 16-byte vectors per lane per row
    static constexpr int NG = 64 / LPR;                   // lane groups per wave
    static constexpr int R = NG / HP;                     // key rows per wave-wide load
    static constexpr int U = (NV == 1) ? 4 : 2;           // loads in flight per operand
    static constexpr int EPL = NV * 8;                    // head-dim elements per lane
    static_assert(NG % HP == 0 && R >= 1, "HP must divide the lane groups of a wave");
};

template <int D, int QB, int HP>
struct MergeSmem {
    float ml[kWaves][HP][QB][2];
    float acc[kWaves][HP][QB][D];
};

template <int D, int QB, int HP>
union KernelSmem {
    ResponseListSmem list;
    MergeSmem<D, QB, HP> merge;
};

template <int D, int QB, int HP>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(QB == 1 ? 3 : 2)))
void sdpa_decode_alu_kernel(SdpaParams p)
{
    using Geo = Geometry<D, HP>;
    constexpr int LPR = Geo::LPR, NV = Geo::NV, R = Geo::R, U = Geo::U, EPL = Geo::EPL;
    constexpr int TILE = R * U;

    __shared__ KernelSmem<D, QB, HP> smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: tile bases stay uniform
    const int c = lane % LPR;            // 16-byte column of the row slice
    const int grp = lane / LPR;          // lane group
    const int hl = grp % HP;             // KV head within the block of HP heads
    const int rl = grp / HP;             // key row within a wave-wide load

    // ---- which work item ----
    int id = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const int qb = id % p.n_qblocks;     id /= p.n_qblocks;
    const int gb = id % (p.Hkv / HP);    id /= (p.Hkv / HP);
    const int chunk = id % p.n_chunks;
    const int b = id / p.n_chunks;
    const int N = p.B * p.W;
    const int g = gb * HP + hl;          // this lane's KV head

    // merged: one work-group walks the whole prompt and the whole response;
    // otherwise a chunk is a slice of response steps or of prompt positions.
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

    // ---- queries of this block (Section 3.3: Q is loaded into registers first) ----
    half2_t qv[QB][NV * 4];
    float slope2[QB];
    int qbeam[QB];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        // queries past the end of the unit repeat the last one and are not stored
        const int lq = min(qb * QB + qi, p.nq - 1);
        const int j = lq / p.G;
        const int hq = g * p.G + (lq % p.G);
        qbeam[qi] = j;
        const size_t qoff = ((size_t)(b * p.W + j) * p.Hq + hq) * D;
        slope2[qi] = p.slopes ? p.slopes[hq] * kLog2e : 0.0f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const u32x4_t w = load16(p.q + qoff + v * (LPR * 8) + c * 8);
            qv[qi][v * 4 + 0] = as_half2(w.x);
            qv[qi][v * 4 + 1] = as_half2(w.y);
            qv[qi][v * 4 + 2] = as_half2(w.z);
            qv[qi][v * 4 + 3] = as_half2(w.w);
        }
    }
    const int qpos = Lp + p.T - 1;

    // ---- fused append: the block that owns step T-1 copies its heads' new rows ----
    const bool have_new = (p.k_new != nullptr);
    if (have_new && qb == 0 && s1 == p.T && s0 < s1) {
        constexpr int kVecPerRow = HP * D / 8;          // HP adjacent heads are contiguous
        const int total = p.W * kVecPerRow * 2;
        for (int i = tid; i < total; i += kThreads) {
            const int which = i / (p.W * kVecPerRow);
            const int rem = i % (p.W * kVecPerRow);
            const int u = rem / kVecPerRow;
            const int col = rem % kVecPerRow;
            const size_t src = ((size_t)(b * p.W + u) * p.Hkv + gb * HP) * D + col * 8;
            const size_t dst =
                (((size_t)(p.T - 1) * N + b * p.W + u) * p.Hkv + gb * HP) * D + col * 8;
            if (which == 0) store16(p.resp_k + dst, load16(p.k_new + src));
            else            store16(p.resp_v + dst, load16(p.v_new + src));
        }
    }

    // ---- online softmax state, one per lane group ----
    float m[QB], l[QB], acc[QB][EPL];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        m[qi] = kEmptyMax;
        l[qi] = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[qi][e] = 0.0f;
    }

    struct Tile {
        u32x4_t k[U][NV];
        u32x4_t v[U][NV];
        uint32_t meta[U];    // (key position << 8) | mask of beams that see the row (0 = invalid)
    };

    auto consume = [&](const Tile& t) {
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            float z[U];
            float m_new = m[qi];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float d = 0.0f;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    d = __builtin_amdgcn_fdot2(qv[qi][v * 4 + 0], as_half2(t.k[u][v].x), d, false);
                    d = __builtin_amdgcn_fdot2(qv[qi][v * 4 + 1], as_half2(t.k[u][v].y), d, false);
                    d = __builtin_amdgcn_fdot2(qv[qi][v * 4 + 2], as_half2(t.k[u][v].z), d, false);
                    d = __builtin_amdgcn_fdot2(qv[qi][v * 4 + 3], as_half2(t.k[u][v].w), d, false);
                }
                d = group_allreduce_sum<LPR>(d);
                const float zz = d * p.scale2 + slope2[qi] * (float)((int)(t.meta[u] >> 8) - qpos);
                const bool vis = (t.meta[u] >> qbeam[qi]) & 1u;
                z[u] = vis ? zz : -INFINITY;
                m_new = fmaxf(m_new, z[u]);
            }
            const float corr = fast_exp2(m[qi] - m_new);
            m[qi] = m_new;
            float pu[U];
            float psum = 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pu[u] = fast_exp2(z[u] - m_new);
                psum += pu[u];
            }
            l[qi] = l[qi] * corr + psum;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[qi][e] *= corr;
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const uint32_t w[4] = {t.v[u][v].x, t.v[u][v].y, t.v[u][v].z, t.v[u][v].w};
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const half2_t hv = as_half2(w[h]);
                        acc[qi][v * 8 + 2 * h + 0] = fmaf(pu[u], (float)hv.x, acc[qi][v * 8 + 2 * h + 0]);
                        acc[qi][v * 8 + 2 * h + 1] = fmaf(pu[u], (float)hv.y, acc[qi][v * 8 + 2 * h + 1]);
                    }
                }
            }
        }
    };

    // ---- prompt segment (Section 3.3: loop over the prompt keys, FlashAttention style) ----
    if (k1 > k0) {
        const int n_tiles = (k1 - k0 + TILE - 1) / TILE;
        // (scalar tile base) + (32-bit lane offset): no 64-bit address per load
        const uint32_t row_stride = p.prompt_row_stride;
        const uint32_t lane_off = (uint32_t)hl * D + c * 8;
        auto fetch = [&](Tile& t, int ti) {
            const int base = k0 + ti * TILE;
            const int lim = min(TILE - 1, k1 - 1 - base);          // last valid row of the tile
            const size_t tile_off =
                (size_t)b * p.prompt_req_stride + (size_t)base * row_stride + gb * HP * D;
            const _Float16* const kb = p.prompt_k + tile_off;
            const _Float16* const vb = p.prompt_v + tile_off;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = u * R + rl;
                const uint32_t off = (uint32_t)min(row, lim) * row_stride + lane_off;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    t.k[u][v] = load16_stream(kb + off + v * (LPR * 8));
                    t.v[u][v] = load16_stream(vb + off + v * (LPR * 8));
                }
                t.meta[u] = ((uint32_t)(base + min(row, lim)) << 8) | (row <= lim ? 0xffu : 0u);
            }
        };
        stream_tiles_impl<Tile>(fetch, consume, wave, n_tiles);
    }

    // ---- response segment (index select fused: rows chosen by the beam lineage) ----
    if (s1 > s0) {
        const uint32_t own_map = list_thread_has_row(p.W, s0, s1)
                                     ? load_parent_map(p.parent, N, p.W, b, s0 + tid + 1)
                                     : kIdentityMap;
        build_response_list(smem.list, p.parent, (gb == 0 && qb == 0) ? p.anc_out : nullptr,
                            p.B, p.W, p.T, b, s0, s1, own_map);
        const int total = smem.list.total;
        const int n_tiles = (total + TILE - 1) / TILE;
        auto fetch = [&](Tile& t, int ti) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = ti * TILE + u * R + rl;
                const bool ok = e < total;
                const uint32_t ent = smem.list.ent[ok ? e : (total - 1)];
                const int s = s0 + (int)(ent >> 16);
                const int slot = (int)((ent >> 8) & 0xffu);
                const _Float16* kp;
                const _Float16* vp;
                if (have_new && s == p.T - 1) {
                    const size_t off = ((size_t)(b * p.W + slot) * p.Hkv + g) * D + c * 8;
                    kp = p.k_new + off;
                    vp = p.v_new + off;
                } else {
                    const size_t off = (((size_t)s * N + b * p.W + slot) * p.Hkv + g) * D + c * 8;
                    kp = p.resp_k + off;
                    vp = p.resp_v + off;
                }
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    t.k[u][v] = load16_stream(kp + v * (LPR * 8));
                    t.v[u][v] = load16_stream(vp + v * (LPR * 8));
                }
                t.meta[u] = ((uint32_t)(Lp + s) << 8) | (ok ? (ent & 0xffu) : 0u);
            }
        };
        stream_tiles_impl<Tile>(fetch, consume, wave, n_tiles);
    }

    // ---- merge the lane groups that hold different rows of the same head ----
#pragma unroll
    for (int off = LPR * HP; off < 64; off <<= 1) {
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            const float mo = __shfl_xor(m[qi], off);
            const float lo = __shfl_xor(l[qi], off);
            const float mn = fmaxf(m[qi], mo);
            const float a = fast_exp2(m[qi] - mn);
            const float bb = fast_exp2(mo - mn);
            l[qi] = l[qi] * a + lo * bb;
            m[qi] = mn;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float ao = __shfl_xor(acc[qi][e], off);
                acc[qi][e] = acc[qi][e] * a + ao * bb;
            }
        }
    }

    // ---- merge the waves through LDS (reuses the response-list storage) ----
    __syncthreads();
    if (rl == 0) {
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            if (c == 0) {
                smem.merge.ml[wave][hl][qi][0] = m[qi];
                smem.merge.ml[wave][hl][qi][1] = l[qi];
            }
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    smem.merge.acc[wave][hl][qi][v * (LPR * 8) + c * 8 + e] = acc[qi][v * 8 + e];
        }
    }
    __syncthreads();

    const int NQ = N * p.Hq;
    for (int idx = tid; idx < HP * QB * D; idx += kThreads) {
        const int d = idx % D;
        const int qi = (idx / D) % QB;
        const int h = idx / (D * QB);
        const int lq = qb * QB + qi;
        if (lq >= p.nq) continue;
        float mm = smem.merge.ml[0][h][qi][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) mm = fmaxf(mm, smem.merge.ml[w][h][qi][0]);
        float ll = 0.0f, aa = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float f = fast_exp2(smem.merge.ml[w][h][qi][0] - mm);
            ll += smem.merge.ml[w][h][qi][1] * f;
            aa += smem.merge.acc[w][h][qi][d] * f;
        }
        const int j = lq / p.G;
        const int hq = (gb * HP + h) * p.G + (lq % p.G);
        const size_t qidx = (size_t)(b * p.W + j) * p.Hq + hq;
        if (direct_out) {
            p.out[qidx * D + d] = (_Float16)(aa / ll);
        } else {
            p.ws_acc[((size_t)chunk * NQ + qidx) * D + d] = aa;
            if (d == 0) {
                p.ws_ml[((size_t)chunk * NQ + qidx) * 2 + 0] = mm;
                p.ws_ml[((size_t)chunk * NQ + qidx) * 2 + 1] = ll;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Merge pass over chunks (Section 3.3: the partial contexts are accumulated
// together): out = sum_c acc_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
// One thread per (query row, 4 consecutive head-dim elements).
// ---------------------------------------------------------------------------
// BATCH chunks are combined per pass with every load of the pass in flight at
// once (first all (m, l) pairs, then all accumulator slices), so a merge of up
// to BATCH chunks costs two memory round trips.  The launcher picks the smallest
// BATCH in {4, 8, 16} that covers the chunk count (slots past the last chunk
// re-read it and are ignored).
template <int BATCH>
__global__ __launch_bounds__(256) void sdpa_merge_kernel(_Float16* out, const float* ws_ml,
                                                         const float* ws_acc, int NQ, int D,
                                                         int n_chunks)
{
    const int per_row = D / 4;
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (size_t)NQ * per_row) return;
    const size_t qidx = gid / per_row;
    const int d4 = (int)(gid % per_row) * 4;
    float mm = kEmptyMax;
    float ll = 0.0f;
    float4_t aa = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int c0 = 0; c0 < n_chunks; c0 += BATCH) {
        float2 ml[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int ch = min(c0 + u, n_chunks - 1);
            ml[u] = *reinterpret_cast<const float2*>(ws_ml + ((size_t)ch * NQ + qidx) * 2);
        }
        float4_t a[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int ch = min(c0 + u, n_chunks - 1);
            a[u] = *reinterpret_cast<const float4_t*>(ws_acc + ((size_t)ch * NQ + qidx) * D + d4);
        }
        float m_new = mm;
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (c0 + u < n_chunks) m_new = fmaxf(m_new, ml[u].x);
        const float corr = fast_exp2(mm - m_new);
        ll *= corr;
        aa *= corr;
        mm = m_new;
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            if (c0 + u < n_chunks) {
                const float f = fast_exp2(ml[u].x - mm);
                ll += ml[u].y * f;
                aa += a[u] * f;
            }
        }
    }
    const float inv = 1.0f / ll;
    half4_t o;
    o.x = (_Float16)(aa.x * inv);
    o.y = (_Float16)(aa.y * inv);
    o.z = (_Float16)(aa.z * inv);
    o.w = (_Float16)(aa.w * inv);
    *reinterpret_cast<half4_t*>(out + qidx * D + d4) = o;
}

// ---------------------------------------------------------------------------
// Append (Section 3.1): row t of the response buffers := the step's K/V.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void append_kv_kernel(uint4* __restrict__ dst_k,
                                                        uint4* __restrict__ dst_v,
                                                        const uint4* __restrict__ src_k,
                                                        const uint4* __restrict__ src_v,
                                                        size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
        dst_k[i] = src_k[i];
        dst_v[i] = src_v[i];
    }
}

// ---------------------------------------------------------------------------
// Streaming-read probe: the practical HBM read ceiling.  Every work-group
// sweeps its own contiguous slice with eight non-temporal 128-bit loads in
// flight per lane -- the friendliest shape this device has for a pure read.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_probe_kernel(const u32x4_t* __restrict__ src,
                                                                size_t n_vec, uint32_t* sink)
{
    constexpr int kInFlight = 8;
    const size_t per_group = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_group;
    const size_t hi = lo + per_group < n_vec ? lo + per_group : n_vec;
    uint32_t x = 0;
    size_t i = lo + threadIdx.x;
    for (; i + (kInFlight - 1) * 256 < hi; i += kInFlight * 256) {
        u32x4_t v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += 256) {
        const u32x4_t a = __builtin_nontemporal_load(src + i);
        x ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    // one word per work-group; the xor keeps every load live
    __shared__ uint32_t red[256];
    red[threadIdx.x] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t y = 0;
        for (int k = 0; k < 256; ++k) y ^= red[k];
        sink[blockIdx.x] = y;
    }
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
template <int D, int QB, int HP>
static hipError_t launch_one(const SdpaParams& p, unsigned grid, hipStream_t st)
{
    return SEGKV_LAUNCH((sdpa_decode_alu_kernel<D, QB, HP>), dim3(grid), dim3(kThreads), st, p);
}

template <int D, int QB>
static hipError_t launch_hp(const SdpaParams& p, int HP, unsigned grid, hipStream_t st)
{
    switch (HP) {
        case 1: return launch_one<D, QB, 1>(p, grid, st);
        case 2: return launch_one<D, QB, 2>(p, grid, st);
        case 4: return launch_one<D, QB, 4>(p, grid, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sdpa_decode(const SdpaParams& p, int D, int QB, int HP, unsigned grid,
                              hipStream_t st)
{
    if (QB != 1 && QB != 4) return hipErrorInvalidValue;
    switch (D) {
        case 64:  return QB == 1 ? launch_hp<64, 1>(p, HP, grid, st) : launch_hp<64, 4>(p, HP, grid, st);
        case 128: return QB == 1 ? launch_hp<128, 1>(p, HP, grid, st) : launch_hp<128, 4>(p, HP, grid, st);
        case 256: return QB == 1 ? launch_hp<256, 1>(p, HP, grid, st) : launch_hp<256, 4>(p, HP, grid, st);
        default:  return hipErrorInvalidValue;
    }
}

hipError_t launch_sdpa_merge(_Float16* out, const float* ws_ml, const float* ws_acc, int NQ, int D,
                             int n_chunks, hipStream_t st)
{
    const size_t threads = (size_t)NQ * (D / 4);
    const unsigned grid = (unsigned)((threads + 255) / 256);
    if (n_chunks <= 4)
        return SEGKV_LAUNCH(sdpa_merge_kernel<4>, dim3(grid), dim3(256), st, out, ws_ml, ws_acc, NQ, D,
                            n_chunks);
    if (n_chunks <= 8)
        return SEGKV_LAUNCH(sdpa_merge_kernel<8>, dim3(grid), dim3(256), st, out, ws_ml, ws_acc, NQ, D,
                            n_chunks);
    return SEGKV_LAUNCH(sdpa_merge_kernel<16>, dim3(grid), dim3(256), st, out, ws_ml, ws_acc, NQ, D,
                        n_chunks);
}

hipError_t launch_append_kv(void* dst_k, void* dst_v, const void* src_k, const void* src_v,
                            size_t bytes, hipStream_t st)
{
    const size_t n_vec = bytes / 16;
    unsigned grid = (unsigned)((n_vec + 255) / 256);
    if (grid > 2048u) grid = 2048u;
    if (grid == 0) grid = 1;
    return SEGKV_LAUNCH(append_kv_kernel, dim3(grid), dim3(256), st, (uint4*)dst_k, (uint4*)dst_v,
                        (const uint4*)src_k, (const uint4*)src_v, n_vec);
}

hipError_t launch_stream_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st)
{
    return SEGKV_LAUNCH(stream_read_probe_kernel, dim3(kProbeGroups), dim3(256), st,
                        (const u32x4_t*)src, bytes / 16, (uint32_t*)sink);
}

}  // namespace segkv
