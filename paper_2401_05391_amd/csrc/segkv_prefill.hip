// libsegkv device code: prefill-phase attention (arxiv 2401.05391, Section 3.1
// prefill phase; Section 3.3: prefill is the decode kernel restricted to the
// query and the prompt key/value).  Batch-first tensors,
// no transposes: q/out [B, N0, Hq, D], k/v [B, N0, Hkv, D]; k/v ARE the prompt
// segment that the decode kernel reads afterwards.  Causal: token i sees keys
// 0..i of its own request.
//
// Compute-bound, so everything runs on the matrix cores, with the same operand
// orientation as the decode kernel:
//     S^T[key][query]  = K[key][:]   . Q^T[:][query]
//     O^T[d][query]   += V^T[d][key] . P^T[key][query]
// A work-group of 4 waves (8 at D = 256) owns 128 (256) consecutive query tokens
// of one (request, query head); each wave holds 32 of them as the N dimension
// (Q^T operand in registers) and walks the key tiles 0 .. its own diagonal.  K/V
// tiles of 32 keys are shared by the group's waves through LDS (one barrier per
// tile); the V^T operand comes out of LDS with the transposing read.  Two
// kernels: sdpa_prefill_direct_kernel<D> (D = 128, 256) copies the tiles from
// global memory straight into LDS, three tiles deep, and stores its output from
// registers; sdpa_prefill_mfma_kernel<D> stages them through registers into
// double-buffered LDS (D = 64, a zero scale, and the tests' second
// implementation).  The order in which the (request, head, query block) items
// are taken is described at prefill_work_item.
#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include "segkv_common.h"
#include "segkv_launch.h"
#include "segkv_device.h"
#include "segkv_mfma_tile.h"

namespace segkv {

// The kernels keep the logits in the units of the raw products and divide the bias by the
// scale.  Below this |scale * log2 e| the product's share of a logit is far under fp32
// resolution next to any bias, the division would overflow, and the scale counts as zero.
constexpr float kTinyScale2 = 1.0e-30f;

// Waves per work-group (each holds 32 query tokens).  D <= 128: four, two
// work-groups per CU, so that one group's barrier waits overlap the other's
// work.  D = 256: eight -- the accumulators leave room for two waves per SIMD
// only within one work-group's LDS, and K/V tiles are shared by twice the queries.
constexpr int prefill_waves(int D) { return D <= 128 ? 4 : 8; }

// Work order.  The query blocks of one (request, query head) re-read the same K/V rows
// (block j needs keys 0 .. its own end), so they should run on one XCD at about the same
// time: the re-reads are then served by its L2 instead of HBM.  Later blocks have more keys
// to visit, and a long block that starts last leaves most of the chip idle while it
// finishes.  Both are met as follows.  The heads are split evenly among the 8 XCDs (the
// hardware sends work-group i to XCD i mod 8; the grid is padded to 8 equal shares and the
// surplus work-groups leave at once).  Each XCD takes its heads in groups of about as many
// as fill its work-group slots twice (heads_per_group x blocks per head), and deals each
// group's blocks longest first ACROSS the group's heads: what runs together still belongs
// to those few heads, and every group -- the XCD's last one too -- ends with its shortest
// blocks.  Heads that share a KV head (grouped queries) are neighbours within a group.
struct PrefillWorkItem { int b, hq, qblk; bool valid; };
__host__ __device__ inline int prefill_grid_size(int n_heads, int n_qblocks)
{
    return kNumXcd * ((n_heads + kNumXcd - 1) / kNumXcd) * n_qblocks;
}
__device__ __forceinline__ PrefillWorkItem prefill_work_item(const PrefillParams& p, int n_qblocks)
{
    const int xcd = blockIdx.x % kNumXcd;
    const int k = blockIdx.x / kNumXcd;                        // this XCD's k-th work-group
    const int n_heads = p.B * p.Hq;
    const int heads_lo = n_heads / kNumXcd, rem = n_heads % kNumXcd;
    const int first_head = xcd * heads_lo + min(xcd, rem);     // the XCD's heads
    const int heads_x = heads_lo + (xcd < rem ? 1 : 0);
    if (k >= heads_x * n_qblocks) return {0, 0, 0, false};
    // groups of nearly equal size, about heads_per_group heads each
    const int n_groups = max(1, (heads_x + p.heads_per_group / 2) / p.heads_per_group);
    const int small = heads_x / n_groups, n_big = heads_x % n_groups;   // n_big groups hold small + 1
    const int big_items = (small + 1) * n_qblocks;
    int group_first, heads_here, r;
    if (k < n_big * big_items) {
        const int gi = k / big_items;
        r = k - gi * big_items;
        heads_here = small + 1;
        group_first = gi * (small + 1);
    } else {
        const int k2 = k - n_big * big_items;
        const int gi = k2 / (small * n_qblocks);
        r = k2 - gi * (small * n_qblocks);
        heads_here = small;
        group_first = n_big * (small + 1) + gi * small;
    }
    const int head = first_head + group_first + r % heads_here;
    return {head / p.Hq, head % p.Hq, n_qblocks - 1 - r / heads_here, true};
}

// Two work-groups per CU (two waves per SIMD) for D <= 128, so that one wave's
// softmax arithmetic overlaps the other's MFMAs.
template <int D>
__global__ __launch_bounds__(prefill_waves(D) * 64) __attribute__((amdgpu_waves_per_eu(2)))
void sdpa_prefill_mfma_kernel(PrefillParams p)
{
    using Geo = MfmaGeometry<D>;
    constexpr int CPR = Geo::CPR, NKS = Geo::NKS, NDB = Geo::NDB;
    constexpr int ROWB = Geo::ROWB, TILEB = Geo::TILEB;
    // V rows 32 bytes apart modulo 256: the four rows of a transposing read (32
    // bytes each) fall into different banks.  (4-8% over the decode kernel's
    // pitch here, where LDS reads are half of the CU's busy cycles.)
    constexpr int VROWB = D * 2 + 32, VTILEB = kKeyTile * VROWB;
    constexpr int kPrefillWaves = prefill_waves(D);
    constexpr int kPrefillQueries = kPrefillWaves * kQueryTile;   // query tokens per work-group
    constexpr int NT = kPrefillWaves * 64;
    constexpr int STAGEB = TILEB + VTILEB;
    constexpr int kVecPerTile = kKeyTile * CPR;            // 16-byte vectors of one operand tile
    constexpr int kVecPerThread = (kVecPerTile + NT - 1) / NT;
    constexpr int OROWB = D * 2 + 16;                      // output staging row pitch

    constexpr int OUTB = kPrefillWaves * kQueryTile * OROWB;          // output staging reuses the tiles
    constexpr int STAGE_PITCH = (2 * STAGEB >= OUTB) ? STAGEB : (OUTB + 1) / 2;
    __shared__ __align__(16) unsigned char s_stage[2][STAGE_PITCH];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31;
    const int h = lane >> 5;

    // ---- work item (see prefill_work_item for the order) ----
    const int n_qblocks = (p.N0 + kPrefillQueries - 1) / kPrefillQueries;
    const PrefillWorkItem item = prefill_work_item(p, n_qblocks);
    if (!item.valid) return;                  // padding of the grid: the whole work-group leaves
    const int qblk = item.qblk, hq = item.hq, b = item.b;
    const int g = hq / p.G;
    const int q0 = qblk * kPrefillQueries;
    const int wq0 = q0 + wave * kQueryTile;   // first query token of this wave
    const int qi = wq0 + n;                   // this lane's query token
    const float slope2 = p.slopes ? p.slopes[hq] * kLog2e : 0.0f;
    // the scale enters as |scale| (its sign is moved into Q), so that the maximum of
    // the raw products of a tile is the maximum of its scaled logits
    const float scale2 = fabsf(p.scale2);
    // Logits are kept in the units of the raw products, raw + bias / |scale|, and the scale is
    // applied inside the exponent's multiply-add.  A zero scale leaves only the bias: then
    // every tile takes the masked path, which drops the product (raw_w = 0) and keeps the
    // bias in final units (mult = 1).
    const bool zero_scale = scale2 < kTinyScale2;
    const float raw_w = zero_scale ? 0.0f : 1.0f;
    const float bias_raw = zero_scale ? slope2 : slope2 / scale2;
    const float mult = zero_scale ? 1.0f : scale2;

    // ---- Q^T operand: this lane's query row, 8 halves per k-step, in registers ----
    half8_t qreg[NKS];
    {
        const int qrow = min(qi, p.N0 - 1);
        const _Float16* qp = p.q + (((size_t)b * p.N0 + qrow) * p.Hq + hq) * D;
        const uint32_t flip = p.scale2 < 0.0f ? 0x80008000u : 0u;
#pragma unroll
        for (int t = 0; t < NKS; ++t) {
            u32x4_t w = load16(qp + 16 * t + 8 * h);
            w.x ^= flip; w.y ^= flip; w.z ^= flip; w.w ^= flip;
            qreg[t] = __builtin_bit_cast(half8_t, w);
        }
    }

    // ---- cooperative K/V tile staging ----
    const int k_end = min(q0 + kPrefillQueries, p.N0);     // keys this block may need
    const int n_tiles = (k_end + kKeyTile - 1) / kKeyTile;
    const uint32_t row_stride = (uint32_t)p.Hkv * D;
    u32x4_t sk[kVecPerThread], sv[kVecPerThread];
    // a thread's offsets within a tile are fixed; the tile's base address is uniform
    uint32_t lane_off[kVecPerThread];
#pragma unroll
    for (int c = 0; c < kVecPerThread; ++c) {
        const int i = tid + c * NT;
        lane_off[c] = (uint32_t)((i / CPR) % kKeyTile) * row_stride + (i % CPR) * 8;
    }
    auto fetch = [&](int ti) __attribute__((always_inline)) {
        const int base = ti * kKeyTile;
        const int lim = p.N0 - 1 - base;                   // last valid row of the tile
        const size_t tile_off = (((size_t)b * p.N0 + base) * p.Hkv + g) * D;
        const _Float16* const kb = p.k + tile_off;
        const _Float16* const vb = p.v + tile_off;
        if (lim >= kKeyTile - 1) {
#pragma unroll
            for (int c = 0; c < kVecPerThread; ++c) {
                sk[c] = load16(kb + lane_off[c]);
                sv[c] = load16(vb + lane_off[c]);
            }
        } else {                                           // ragged last tile: rows past the end repeat the last one
#pragma unroll
            for (int c = 0; c < kVecPerThread; ++c) {
                const int i = tid + c * NT;
                const int row = min((i / CPR) % kKeyTile, lim);
                const uint32_t off = (uint32_t)row * row_stride + (i % CPR) * 8;
                sk[c] = load16(kb + off);
                sv[c] = load16(vb + off);
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kVecPerThread; ++c) {
            const int i = tid + c * NT;
            if (i < kVecPerTile) {
                const int row = i / CPR, ch = i % CPR;
                *reinterpret_cast<u32x4_t*>(s_stage[buf] + row * ROWB + (ch << 4)) = sk[c];
                *reinterpret_cast<u32x4_t*>(s_stage[buf] + TILEB + row * VROWB + (ch << 4)) = sv[c];
            }
        }
    };

    // ---- running state ----
    float m_ref = kEmptyMax;
    float l_part = 0.0f;
    float16_t o_acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.0f;

    const int grp = lane >> 4;
    const int li = lane & 15;
    const int tr_base = (4 * h + (li >> 2)) * VROWB + ((16 * (grp & 1) + 4 * (li & 3)) << 1);

    auto compute_tile = [&](const unsigned char* k_tile, const unsigned char* v_tile, int base,
                            bool diagonal) __attribute__((always_inline)) {
        float16_t s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
        for (int t = 0; t < NKS; ++t) {
            const half8_t a =
                *reinterpret_cast<const half8_t*>(k_tile + n * ROWB + ((2 * t + h) << 4));
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[t], s, 0, 0, 0);
        }
        // s holds the raw products; tiles with a mask or a bias bring their logits into the
        // same raw units (bias divided by the scale, masked keys at minus infinity), and the
        // scale is applied inside the exponent's multiply-add
        if (diagonal || p.slopes != nullptr || zero_scale) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = base + 8 * (r >> 2) + 4 * h + (r & 3);
                const float z = __builtin_fmaf(s[r], raw_w, bias_raw * (float)(key - qi));
                s[r] = (key <= qi) ? z : -INFINITY;       // causal; also hides keys >= N0
            }
        }
        float m_tile = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, s[r]);
        m_tile *= mult;
        // The two lanes that share a query (keys 4h..) see different keys, but the
        // vote is wave-wide: their maxima are only exchanged when the reference moves.
        if (__any(m_tile > m_ref + kRescaleSlack)) {
            m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
            const float m_new = fmaxf(m_ref, m_tile);
            const float corr = fast_exp2(m_ref - m_new);
            m_ref = m_new;
            l_part *= corr;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= corr;
        }
        half8_t pb[2];
        const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(__builtin_fmaf(s[r], mult, -m_ref));
            const float p1 = fast_exp2(__builtin_fmaf(s[r + 1], mult, -m_ref));
            const half2_t pp = {(_Float16)p0, (_Float16)p1};
            // the row sum adds what the P.V product will see: the rounded pair, in one instruction
            l_part = __builtin_amdgcn_fdot2(pp, ones, l_part, false);
            pb[r >> 3][r & 7] = pp.x;
            pb[r >> 3][(r & 7) + 1] = pp.y;
        }
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
            if (NDB > 4) __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop over key tiles: one barrier per tile, loads one tile ahead ----
    fetch(0);
    stage(0);
    __syncthreads();
    for (int ti = 0; ti < n_tiles; ++ti) {
        const int buf = ti & 1;
        if (ti + 1 < n_tiles) fetch(ti + 1);
        const int base = ti * kKeyTile;
        // tiles entirely above this wave's last query are skipped (uniform per wave)
        if (base <= wq0 + kQueryTile - 1)
            compute_tile(s_stage[buf], s_stage[buf] + TILEB, base, base + kKeyTile - 1 > wq0);
        if (ti + 1 < n_tiles) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise, transpose through LDS, store rows with 128-bit writes ----
    l_part += __shfl_xor(l_part, 32);
    const float inv = 1.0f / l_part;
    unsigned char* const obuf = &s_stage[0][0] + wave * (kQueryTile * OROWB);
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half4_t o4;
            o4.x = (_Float16)(o_acc[db][4 * i + 0] * inv);
            o4.y = (_Float16)(o_acc[db][4 * i + 1] * inv);
            o4.z = (_Float16)(o_acc[db][4 * i + 2] * inv);
            o4.w = (_Float16)(o_acc[db][4 * i + 3] * inv);
            *reinterpret_cast<half4_t*>(obuf + n * OROWB + ((32 * db + 8 * i + 4 * h) << 1)) = o4;
        }
    // the wave reads back only what it wrote itself
    wave_lds_exchange_point();
    constexpr int kRowsPerPass = 64 / CPR;
#pragma unroll
    for (int r0 = 0; r0 < kQueryTile; r0 += kRowsPerPass) {
        const int row = r0 + lane / CPR;
        const int ch = lane % CPR;
        const int tok = wq0 + row;
        const u32x4_t w = *reinterpret_cast<const u32x4_t*>(obuf + row * OROWB + (ch << 4));
        if (tok < p.N0)
            store16(p.out + (((size_t)b * p.N0 + tok) * p.Hq + hq) * D + ch * 8, w);
    }
}

// ---------------------------------------------------------------------------
// D = 128 variant whose K/V tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: lane i's 16 bytes land at base + 16 i, no registers
// and no LDS store instructions in between), three tiles deep.
//
// A copy instruction fills 1 KB = 4 whole rows without padding, so rows are 256
// bytes apart and bank conflicts are avoided by permuting the 16-byte chunks of
// a row instead: the lane that fills position c' of row r fetches chunk
//     K tile:  c = c' ^ (r & 15)                 (16 consecutive rows reading one
//                                                 chunk hit 16 different positions)
//     V tile:  c = (((c' >> 1) ^ (r & 7)) << 1) | (c' & 1)
//                                                (the 4 rows of a transposing read,
//                                                 32 bytes each, hit 4 different ones)
// and the operand reads apply the same permutation.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void copy16_to_lds(const _Float16* gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory");
}

// The same with a uniform base address in scalar registers and a 32-bit byte offset per lane.
__device__ __forceinline__ void copy16_to_lds(const _Float16* base, uint32_t byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_base)
                 : "memory");
}

// D = 128: four waves, three work-groups per CU (the register budget of three waves per SIMD
// is part of the design).  D = 256: eight waves and one work-group per CU; rows are 512 bytes
// and the same permutations act on the low four bits of the chunk index.
constexpr int direct_waves(int D) { return D == 256 ? 8 : 4; }
template <int D>
__global__ __launch_bounds__(direct_waves(D) * 64) __attribute__((amdgpu_waves_per_eu(D == 256 ? 2 : 3)))
void sdpa_prefill_direct_kernel(PrefillParams p)
{
    constexpr int CPR = D / 8, NKS = D / 16, NDB = D / 32;
    constexpr int ROWB = D * 2;                            // no padding: see above
    constexpr int TILEB = kKeyTile * ROWB, STAGEB = 2 * TILEB, NSTAGE = 3;
    constexpr int RPI = 64 / CPR;                          // rows per copy instruction
    constexpr int NINS = kKeyTile / RPI;                   // copy instructions per operand tile
    constexpr int NWAVES = direct_waves(D), INS_PER_WAVE = NINS / NWAVES;
    constexpr int kQueries = NWAVES * kQueryTile;
    static_assert(INS_PER_WAVE * NWAVES == NINS && INS_PER_WAVE >= 1, "the waves share a tile's copies evenly");
    __shared__ __align__(256) unsigned char s_stage[NSTAGE * STAGEB];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31;
    const int h = lane >> 5;

    const int n_qblocks = (p.N0 + kQueries - 1) / kQueries;
    const PrefillWorkItem item = prefill_work_item(p, n_qblocks);
    if (!item.valid) return;                  // padding of the grid: the whole work-group leaves
    const int qblk = item.qblk, hq = item.hq, b = item.b;
    const int g = hq / p.G;
    const int q0 = qblk * kQueries;
    const int wq0 = q0 + wave * kQueryTile;
    const int qi = wq0 + n;
    const float slope2 = p.slopes ? p.slopes[hq] * kLog2e : 0.0f;
    // the scale enters as |scale| (its sign is moved into Q), so that the maximum of
    // the raw products of a tile is the maximum of its scaled logits
    const float scale2 = fabsf(p.scale2);

    // ---- tile copies: this wave's share is INS_PER_WAVE instructions per operand ----
    const int k_end = min(q0 + kQueries, p.N0);
    const int n_tiles = (k_end + kKeyTile - 1) / kKeyTile;
    const uint32_t row_stride = (uint32_t)p.Hkv * D;
    const unsigned lds0 =
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)s_stage;
    const int crow = lane / CPR;                          // row within the instruction's 4
    const int cpos = lane % CPR;                          // chunk position filled by this lane
    // A lane's byte offset within a tile is fixed (row, permuted chunk); the tile's base
    // address is uniform and travels in scalar registers, one tile stride further per turn.
    auto chunk_k = [&](int r) __attribute__((always_inline)) { return cpos ^ (r & 15); };
    auto chunk_v = [&](int r) __attribute__((always_inline)) {
        return (((cpos >> 1) ^ (r & 7)) << 1) | (cpos & 1);
    };
    uint32_t lane_off_k[INS_PER_WAVE], lane_off_v[INS_PER_WAVE];
#pragma unroll
    for (int j = 0; j < INS_PER_WAVE; ++j) {
        const int r = RPI * (wave * INS_PER_WAVE + j) + crow;
        lane_off_k[j] = ((uint32_t)r * row_stride + chunk_k(r) * 8) * 2;
        lane_off_v[j] = ((uint32_t)r * row_stride + chunk_v(r) * 8) * 2;
    }
    const size_t head_off = ((size_t)b * p.N0 * p.Hkv + g) * D;
    const size_t tile_stride = (size_t)kKeyTile * row_stride;
    auto issue = [&](int ti, int stage) __attribute__((always_inline)) {
        const int lim = p.N0 - 1 - ti * kKeyTile;         // last valid row of the tile
        const _Float16* const k_tile = p.k + head_off + ti * tile_stride;
        const _Float16* const v_tile = p.v + head_off + ti * tile_stride;
        const unsigned sbase = lds0 + stage * STAGEB + wave * INS_PER_WAVE * 1024;
        if (lim >= kKeyTile - 1) {
#pragma unroll
            for (int j = 0; j < INS_PER_WAVE; ++j) {
                copy16_to_lds(k_tile, lane_off_k[j], sbase + j * 1024);
                copy16_to_lds(v_tile, lane_off_v[j], sbase + TILEB + j * 1024);
            }
        } else {                                          // ragged last tile: rows past the end repeat the last one
#pragma unroll
            for (int j = 0; j < INS_PER_WAVE; ++j) {
                const int r = RPI * (wave * INS_PER_WAVE + j) + crow;
                const uint32_t roff = (uint32_t)min(r, lim) * row_stride;
                copy16_to_lds(k_tile, (roff + chunk_k(r) * 8) * 2, sbase + j * 1024);
                copy16_to_lds(v_tile, (roff + chunk_v(r) * 8) * 2, sbase + TILEB + j * 1024);
            }
        }
    };
    // all three stages are free at the start: the first three tiles go out together, ahead of Q
    issue(0, 0);
    if (n_tiles > 1) issue(1, 1);
    if (n_tiles > 2) issue(2, 2);

    // ---- Q^T operand in registers ----
    half8_t qreg[NKS];
    {
        const int qrow = min(qi, p.N0 - 1);
        const _Float16* qp = p.q + (((size_t)b * p.N0 + qrow) * p.Hq + hq) * D;
        const uint32_t flip = p.scale2 < 0.0f ? 0x80008000u : 0u;
#pragma unroll
        for (int t = 0; t < NKS; ++t) {
            u32x4_t w = load16(qp + 16 * t + 8 * h);
            w.x ^= flip; w.y ^= flip; w.z ^= flip; w.w ^= flip;
            qreg[t] = __builtin_bit_cast(half8_t, w);
        }
        // The compiler's wait for these loads must sit here and not inside the tile
        // loop, where it would also wait for the tile copies in flight (which it
        // does not know of).
#pragma unroll
        for (int t = 0; t < NKS; ++t) asm volatile("" : "+v"(qreg[t]));
    }

    float m_ref = kEmptyMax;
    float l_part = 0.0f;
    float16_t o_acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.0f;

    const int grp = lane >> 4;
    const int li = lane & 15;
    const int kx = (n & 15) << 4;                                      // K chunk permutation of row n
    const int vrow = 4 * h + (li >> 2);                                // first V row of this lane
    const int vy = ((grp & 1) ^ (vrow & 7)) << 5;                      // V pair permutation
    const int tr_base = vrow * ROWB + 8 * (li & 3);

    // Lane-constant LDS addresses of the operand reads; the stage is a compile-time
    // constant of each copy of the loop body below, so it travels in the instructions'
    // immediate offsets and no address is computed per tile.
    // (finished values the compiler may not take apart again into a shared base plus a part
    // that it would then add back before every read)
    // (The permutations touch address bits 4-7 only: k-step t + 8 and block db + 4 of a
    // 512-byte row are their partners' addresses plus 256, one more immediate.)
    constexpr int NKA = NKS < 8 ? NKS : 8, NVA = NDB < 4 ? NDB : 4;
    int k_addr[NKA], v_addr[NVA];
#pragma unroll
    for (int t = 0; t < NKA; ++t) {
        k_addr[t] = n * ROWB + (((2 * t + h) << 4) ^ kx);
        asm volatile("" : "+v"(k_addr[t]));
    }
#pragma unroll
    for (int db = 0; db < NVA; ++db) {
        v_addr[db] = TILEB + tr_base + ((db * 64) ^ vy);
        asm volatile("" : "+v"(v_addr[db]));
    }
    const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};

    // Softmax of one tile and its P.V product.  s holds the raw products; tiles with a
    // mask or a bias first bring their logits into the same raw units (bias divided by the
    // scale, masked keys at minus infinity), so that one copy of the code below serves
    // both and the scale is applied inside the exponent's multiply-add.
    const float bias_raw = slope2 / scale2;
    auto finish_tile = [&](float16_t& s, int base, bool plain, auto stage_c) __attribute__((always_inline)) {
        constexpr int SOFF = decltype(stage_c)::value * STAGEB;
        if (!plain) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = base + 8 * (r >> 2) + 4 * h + (r & 3);
                const float z = s[r] + bias_raw * (float)(key - qi);
                s[r] = (key <= qi) ? z : -INFINITY;       // causal; also hides keys >= N0
            }
        }
        float m_tile = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, s[r]);
        m_tile *= scale2;
        const float mult = scale2;
        // The two lanes that share a query see different keys, but the vote is wave-wide:
        // their maxima are only exchanged when the reference moves.
        if (__any(m_tile > m_ref + kRescaleSlack)) {
            m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
            const float m_new = fmaxf(m_ref, m_tile);
            const float corr = fast_exp2(m_ref - m_new);
            m_ref = m_new;
            l_part *= corr;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= corr;
        }
        half8_t pb[2];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(__builtin_fmaf(s[r], mult, -m_ref));
            const float p1 = fast_exp2(__builtin_fmaf(s[r + 1], mult, -m_ref));
            const half2_t pp = {(_Float16)p0, (_Float16)p1};
            // the row sum adds what the P.V product will see: the rounded pair, in one instruction
            l_part = __builtin_amdgcn_fdot2(pp, ones, l_part, false);
            pb[r >> 3][r & 7] = pp.x;
            pb[r >> 3][(r & 7) + 1] = pp.y;
        }
        if constexpr (D == 256) {
            // as for the K operands: the V^T operands (two transposing reads each) run
            // V_AHEAD products ahead of their MFMAs
            constexpr int V_AHEAD = 4;
            half4_t va[2 * NDB][2];
#pragma unroll
            for (int i = 0; i < 2 * NDB; ++i) {
                const int db = i >> 1, u = i & 1;
                va[i][0] = lds_read_tr16(s_stage + v_addr[db % NVA] + (SOFF + (db / NVA) * 256 + (16 * u) * ROWB));
                va[i][1] = lds_read_tr16(s_stage + v_addr[db % NVA] + (SOFF + (db / NVA) * 256 + (16 * u + 8) * ROWB));
            }
#pragma unroll
            for (int i = 0; i < 2 * NDB; ++i) {
                const half4_t lo = va[i][0], hi = va[i][1];
                const half8_t a = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                o_acc[i >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[i & 1], o_acc[i >> 1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * V_AHEAD, 0);
#pragma unroll
            for (int i = 0; i < 2 * NDB - V_AHEAD; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, V_AHEAD, 0);
        } else {
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const half4_t lo = lds_read_tr16(s_stage + v_addr[db % NVA] + (SOFF + (db / NVA) * 256 + (16 * u) * ROWB));
                    const half4_t hi = lds_read_tr16(s_stage + v_addr[db % NVA] + (SOFF + (db / NVA) * 256 + (16 * u + 8) * ROWB));
                    const half8_t a = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[u], o_acc[db], 0, 0, 0);
                }
            }
        }
    };

    // ---- a wave's output, written from registers: the two lanes of a query hold alternating
    // 8-byte pieces of its row; they swap every other piece, so that each stores 16 contiguous
    // bytes.  No LDS and no barrier after the last tile.
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    auto store_output = [&]() __attribute__((always_inline)) {
        const float l_row = l_part + __shfl_xor(l_part, 32);
        const float inv = 1.0f / l_row;
        _Float16* const row = p.out + (((size_t)b * p.N0 + min(qi, p.N0 - 1)) * p.Hq + hq) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int ip = 0; ip < 4; ip += 2) {
                uint32_t w[2][2];                      // [piece ip, ip + 1][its two words]
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const half2_t lo = {(_Float16)(o_acc[db][4 * (ip + j) + 0] * inv),
                                        (_Float16)(o_acc[db][4 * (ip + j) + 1] * inv)};
                    const half2_t hi = {(_Float16)(o_acc[db][4 * (ip + j) + 2] * inv),
                                        (_Float16)(o_acc[db][4 * (ip + j) + 3] * inv)};
                    w[j][0] = __builtin_bit_cast(uint32_t, lo);
                    w[j][1] = __builtin_bit_cast(uint32_t, hi);
                }
                // upper-half lanes of the first operand <-> lower-half lanes of the second:
                // lane n keeps its piece ip and receives lane n+32's piece ip (the next 8 bytes);
                // lane n+32 receives lane n's piece ip+1 and keeps its own
                const u32x2_t x0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                const u32x2_t x1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                const u32x4_t v = {x0.x, x1.x, x0.y, x1.y};
                if (qi < p.N0) store16(row + 32 * db + 8 * (ip + h), v);
            }
    };

    // ---- one turn of the main loop: tile ti is computed out of stage STAGE while ti+1
    // and ti+2 are on their way.  s_waitcnt immediates: vmcnt in bits 3:0, no wait on the
    // other counters. ----
    const bool alibi = p.slopes != nullptr;
    auto turn = [&](int ti, auto stage_c) __attribute__((always_inline)) {
        constexpr int STAGE = decltype(stage_c)::value;
        constexpr int SOFF = STAGE * STAGEB;
        // this wave's copies of tile ti have landed (the 2 * INS_PER_WAVE newest belong to ti+1)
        if (ti + 1 < n_tiles) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * INS_PER_WAVE));
        else                  __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();      // everybody's have; and everybody is done with tile ti-1's stage
        if (ti > 0 && ti + 2 < n_tiles) issue(ti + 2, (STAGE + 2) % NSTAGE);   // (tile 2 went out with 0 and 1)
        const int base = ti * kKeyTile;
        if (base <= wq0 + kQueryTile - 1) {
            // (the wave that is about to issue the dependent Q.K^T chain goes first on its SIMD:
            // +0.2-1 %; the same around the P.V product measured 3 % slower)
            __builtin_amdgcn_s_setprio(2);
            float16_t s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.0f;
            if constexpr (D == 256) {
                // Two waves per SIMD here: an LDS read takes longer than the two MFMAs the
                // compiler would leave between a read and its use, so the K operands run
                // four reads ahead (the groups below fix that order).
                constexpr int AHEAD = 3;
                half8_t a[NKS];
#pragma unroll
                for (int t = 0; t < NKS; ++t)
                    a[t] = *reinterpret_cast<const half8_t*>(s_stage + k_addr[t % NKA] + (SOFF + (t / NKA) * 256));
#pragma unroll
                for (int t = 0; t < NKS; ++t) s = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t], qreg[t], s, 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
                for (int t = 0; t < NKS - AHEAD; ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
            } else {
#pragma unroll
                for (int t = 0; t < NKS; ++t) {
                    const half8_t a = *reinterpret_cast<const half8_t*>(s_stage + k_addr[t % NKA] + (SOFF + (t / NKA) * 256));
                    s = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[t], s, 0, 0, 0);
                }
            }
            __builtin_amdgcn_s_setprio(0);
            finish_tile(s, base, !alibi && base + kKeyTile - 1 <= wq0, stage_c);
        }
    };
    // (one copy of the loop body per stage: the stage's LDS offset is an immediate)
    for (int ti = 0; ti < n_tiles; ti += NSTAGE) {
        turn(ti, std::integral_constant<int, 0>{});
        if (ti + 1 < n_tiles) turn(ti + 1, std::integral_constant<int, 1>{});
        if (ti + 2 < n_tiles) turn(ti + 2, std::integral_constant<int, 2>{});
    }
    store_output();
}

hipError_t launch_sdpa_prefill(const PrefillParams& p, int D, hipStream_t st)
{
    if (D != 64 && D != 128 && D != 256) return hipErrorInvalidValue;
    // tiles copied straight into LDS at D = 128 and 256 (a zero scale goes the other way: the
    // direct kernels divide the bias by the scale); the test-only override keeps the
    // register-staged kernels
    const bool direct = (D == 128 || D == 256) && !tuning().prefill_regs && fabsf(p.scale2) >= kTinyScale2;
    const int nw = direct ? direct_waves(D) : prefill_waves(D);
    const int n_qblocks = (p.N0 + nw * kQueryTile - 1) / (nw * kQueryTile);
    const unsigned grid = (unsigned)prefill_grid_size(p.B * p.Hq, n_qblocks);
    const dim3 block(nw * 64);
    // work-group slots of one XCD (32 CUs; work-groups per CU as the kernels' registers and
    // LDS allow: 4 / 3 / 1 at D = 64 / 128 / 256), the measure of a group of heads
    PrefillParams q = p;
    const int slots_per_xcd = 32 * (D == 64 ? 4 : D == 128 ? 3 : 1);
    // Two rounds of slots per group measured best on the multi-head shapes (one: -1 %, four: -4
    // to -8 %, the K/V of too many heads then compete for the L2); query heads that share a KV head
    // cost the L2 nothing extra, so grouped-query shapes take G times as many (70B-2k: +4 %).
    q.heads_per_group = std::max(1, 2 * slots_per_xcd / n_qblocks) * std::max(1, p.G);
    switch (D) {
        case 64:  return SEGKV_LAUNCH(sdpa_prefill_mfma_kernel<64>, dim3(grid), block, st, q);
        case 128:
            if (direct) return SEGKV_LAUNCH(sdpa_prefill_direct_kernel<128>, dim3(grid), block, st, q);
            return SEGKV_LAUNCH(sdpa_prefill_mfma_kernel<128>, dim3(grid), block, st, q);
        default:
            if (direct) return SEGKV_LAUNCH(sdpa_prefill_direct_kernel<256>, dim3(grid), block, st, q);
            return SEGKV_LAUNCH(sdpa_prefill_mfma_kernel<256>, dim3(grid), block, st, q);
    }
}

}  // namespace segkv
