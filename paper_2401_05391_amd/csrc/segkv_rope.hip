// libsegkv device code: the producer step ahead of the decode attention
// (arxiv 2401.05391, Section 3.1): rotary position embedding of the step's
// query and key, fused with the append of the step's key/value to their row of
// the sequence-first response buffers -- one launch instead of RoPE(q), RoPE(k)
// and two copies.
//
// One work-group per beam row.  The row's cos/sin table (rotary_dim/2 angles,
// evaluated in double precision: positions reach thousands of radians) is built
// once in LDS, then every thread rotates 16-byte pieces of the row's heads.
#include "segkv_common.h"
#include "segkv_launch.h"
#include "segkv_device.h"

namespace segkv {

constexpr int kRopeThreads = 256;
constexpr int kRopeMaxPairs = 128;   // rotary_dim <= 256

template <bool INTERLEAVED>
__global__ __launch_bounds__(kRopeThreads) void rope_append_kernel(RopeParams p)
{
    __shared__ float s_cos[kRopeMaxPairs];
    __shared__ float s_sin[kRopeMaxPairs];

    const int n = blockIdx.x;                    // beam row
    const int tid = threadIdx.x;
    const int D = p.D, R = p.R;
    const int pos = p.positions ? p.positions[n / p.W] : p.pos_default;

    // theta_i = base^(-2i/R); angle = pos * theta_i
    for (int i = tid; i < R / 2; i += kRopeThreads) {
        const double theta = exp2(-2.0 * (double)i / (double)R * p.log2_base);
        double sn, cs;
        sincos((double)pos * theta, &sn, &cs);
        s_cos[i] = (float)cs;
        s_sin[i] = (float)sn;
    }
    __syncthreads();

    // A rotation item covers 8 pairs in the half convention (the 16-byte piece at
    // 8i and its partner at R/2 + 8i) and 4 pairs in the interleaved one (the
    // piece at 8i holds its own partners).
    const int items_per_head = INTERLEAVED ? R / 8 : R / 16;
    const int tail_per_head = (D - R) / 8;       // 16-byte pieces past the rotary part
    const int q_items = p.Hq * items_per_head;
    const int k_items = p.Hkv * items_per_head;

    _Float16* const q_row = p.q + (size_t)n * p.Hq * D;
    const _Float16* const k_src = p.k_new + (size_t)n * p.Hkv * D;
    _Float16* const k_dst = p.resp_k_row + (size_t)n * p.Hkv * D;

    for (int it = tid; it < q_items + k_items; it += kRopeThreads) {
        const bool is_q = it < q_items;
        const int local = is_q ? it : it - q_items;
        const int head = local / items_per_head;
        const int i = local % items_per_head;
        const _Float16* src = (is_q ? q_row : k_src) + (size_t)head * D;
        _Float16* dst = (is_q ? q_row : k_dst) + (size_t)head * D;
        if (INTERLEAVED) {
            const u32x4_t w = load16(src + 8 * i);
            const uint32_t in[4] = {w.x, w.y, w.z, w.w};
            uint32_t out[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t ab = as_half2(in[j]);
                const float a = (float)ab.x, b = (float)ab.y;
                const float c = s_cos[4 * i + j], s = s_sin[4 * i + j];
                const half2_t r = {(_Float16)(a * c - b * s), (_Float16)(b * c + a * s)};
                out[j] = __builtin_bit_cast(uint32_t, r);
            }
            store16(dst + 8 * i, u32x4_t{out[0], out[1], out[2], out[3]});
        } else {
            const u32x4_t wa = load16(src + 8 * i);
            const u32x4_t wb = load16(src + R / 2 + 8 * i);
            const uint32_t ina[4] = {wa.x, wa.y, wa.z, wa.w};
            const uint32_t inb[4] = {wb.x, wb.y, wb.z, wb.w};
            uint32_t oa[4], ob[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t a2 = as_half2(ina[j]), b2 = as_half2(inb[j]);
                const float c0 = s_cos[8 * i + 2 * j], s0 = s_sin[8 * i + 2 * j];
                const float c1 = s_cos[8 * i + 2 * j + 1], s1 = s_sin[8 * i + 2 * j + 1];
                const float a0 = (float)a2.x, a1 = (float)a2.y, b0 = (float)b2.x, b1 = (float)b2.y;
                const half2_t ra = {(_Float16)(a0 * c0 - b0 * s0), (_Float16)(a1 * c1 - b1 * s1)};
                const half2_t rb = {(_Float16)(b0 * c0 + a0 * s0), (_Float16)(b1 * c1 + a1 * s1)};
                oa[j] = __builtin_bit_cast(uint32_t, ra);
                ob[j] = __builtin_bit_cast(uint32_t, rb);
            }
            store16(dst + 8 * i, u32x4_t{oa[0], oa[1], oa[2], oa[3]});
            store16(dst + R / 2 + 8 * i, u32x4_t{ob[0], ob[1], ob[2], ob[3]});
        }
    }

    // elements past the rotary part of K are copied (Q is rotated in place: nothing to do)
    for (int it = tid; it < p.Hkv * tail_per_head; it += kRopeThreads) {
        const int head = it / tail_per_head;
        const int off = head * D + R + 8 * (it % tail_per_head);
        store16(k_dst + off, load16(k_src + off));
    }
    // V: plain append
    const _Float16* const v_src = p.v_new + (size_t)n * p.Hkv * D;
    _Float16* const v_dst = p.resp_v_row + (size_t)n * p.Hkv * D;
    for (int it = tid; it < p.Hkv * D / 8; it += kRopeThreads)
        store16(v_dst + 8 * it, load16(v_src + 8 * it));
}

hipError_t launch_rope_append(const RopeParams& p, int interleaved, int rows, hipStream_t st)
{
    if (interleaved)
        return SEGKV_LAUNCH(rope_append_kernel<true>, dim3(rows), dim3(kRopeThreads), st, p);
    return SEGKV_LAUNCH(rope_append_kernel<false>, dim3(rows), dim3(kRopeThreads), st, p);
}

}  // namespace segkv
