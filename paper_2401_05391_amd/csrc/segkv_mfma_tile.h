// Tile geometry and LDS helpers shared by the matrix-core kernels (decode and
// prefill): 32-key x 32-query tiles for v_mfma_f32_32x32x16_f16.
#pragma once
#include "segkv_common.h"

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
    // Row pitch of the LDS tiles: 16 bytes of padding make it 16 mod 256, so the
    // 16 consecutive rows that read the same 16-byte column (QK^T operands) fall
    // into 16 different bank groups, and every operand address stays "lane base
    // + constant".  The V tile uses the same pitch: wider paddings (32, 48) that
    // would also separate the 4 rows of a transposing read measured ~15% slower
    // end to end on MI355X.
    static constexpr int ROWB = D * 2 + 16;
    static constexpr int VROWB = D * 2 + 16;
    static constexpr int TILEB = kKeyTile * ROWB;     // bytes of a K tile
    static constexpr int VTILEB = kKeyTile * VROWB;   // bytes of a V tile
    static constexpr int MROW = D + 4;                // floats per query row in the merge layout
    static constexpr int MERGEB = kQueryTile * MROW * 4;
    static constexpr int REGIONB = (TILEB + VTILEB > MERGEB) ? TILEB + VTILEB : MERGEB;  // per wave
};

// 64-bit LDS read with a 16-bit transpose across each group of 16 lanes.
__device__ __forceinline__ half4_t lds_read_tr16(const unsigned char* lds_ptr)
{
    typedef short short4_t __attribute__((ext_vector_type(4)));
    const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4_t*)(lds_ptr));
    return __builtin_bit_cast(half4_t, r);
}

}  // namespace segkv
