// Internal interface between the C-ABI layer (segkv_api.hip) and the device
// code (segkv_kernels.hip).  Not installed; not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace segkv {

// Launches a kernel and returns the status of THIS launch: the thread's sticky
// error is cleared first, so that an error some earlier HIP call of the caller
// left behind is not mistaken for a rejected launch.
template <typename... KArgs, typename... Args>
inline hipError_t launch_checked(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                                 Args... args)
{
    (void)hipGetLastError();
    kernel<<<grid, block, 0, stream>>>(args...);
    return hipGetLastError();
}
#define SEGKV_LAUNCH(kernel, grid, block, stream, ...) \
    ::segkv::launch_checked(kernel, grid, block, stream, __VA_ARGS__)

}  // namespace segkv

namespace segkv {

// Planner overrides for tests and A/B measurements, read from the environment
// ONCE (first use) and again only on segkv_reload_tuning(): see include/segkv.h.
struct Tuning {
    int path;            // SEGKV_PATH: 0 planner's choice, 1 "alu", 2 "mfma"
    int pair_heads;      // SEGKV_PAIR_HEADS: -1 planner's choice, 0, 1
    int target_groups;   // SEGKV_TARGET_GROUPS: 0 = default
    int min_pchunk;      // SEGKV_MIN_PCHUNK: 0 = default
    int mfma_waves;      // SEGKV_MFMA_WAVES: 0 = planner's choice, 4, 8
    int heads_per_wave;  // SEGKV_HEADS_PER_WAVE: 0 = planner's choice
    int xcd_head_order;  // SEGKV_XCD_HEAD_ORDER: 0 keeps consecutive heads on consecutive XCDs, default on
    int prefill_regs;    // SEGKV_PREFILL=regs: 1 keeps the register-staged prefill kernel at D = 128
};
const Tuning& tuning();
void reload_tuning();

struct SdpaParams {
    const _Float16* q;
    _Float16* out;
    const _Float16* prompt_k;
    const _Float16* prompt_v;
    _Float16* resp_k;
    _Float16* resp_v;
    const int32_t* parent;
    const _Float16* k_new;
    const _Float16* v_new;
    const float* slopes;
    const int32_t* prompt_lens;   // [B] valid prompt rows per request, or null (all Lp)
    int32_t* anc_out;
    float* ws_ml;    // [n_chunks][NQ][2]
    float* ws_acc;   // [n_chunks][NQ][D]
    float scale2;    // scale * log2(e)
    int B, W, Hq, Hkv, G, Lp, T;
    int nq;          // W * G queries per unit
    int n_qblocks;
    int merged;      // 1: a single work-group per (unit, qblock) covers prompt and response
    int n_chunks;    // partials per query (1 => the main kernel writes `out` itself)
    int pchunk;      // prompt positions per chunk
    int rchunk;      // response steps per chunk (<= kMaxStepsPerChunk)
    int n_rchunks;   // response chunks come first in the chunk index
    uint32_t prompt_row_stride;   // elements between consecutive keys of one request and head
    size_t prompt_req_stride;     // elements between the first keys of consecutive requests
    const uint32_t* lineage;      // null, or the per-request lineage lists (see segkv_lineage.hip)
    int lineage_stride;           // 32-bit words per request: header + capacity
    int head_pairs;     // 1: every row holds two adjacent heads of D/2 elements (D = 128 kernel, 64-wide heads)
    uint32_t head_perm8;  // matrix-core kernel: nibble j = KV head (mod 8) that position j of a run of eight takes
    int resp_in_last;   // 1: no response chunks; the last chunk walks its prompt rows and the whole response
};


struct PrefillParams {
    const _Float16* q;    // [B, N0, Hq, D]
    const _Float16* k;    // [B, N0, Hkv, D]
    const _Float16* v;    // [B, N0, Hkv, D]
    _Float16* out;        // [B, N0, Hq, D]
    const float* slopes;  // [Hq] or null
    float scale2;         // scale * log2(e)
    int B, N0, Hq, Hkv, G;
    int heads_per_group;  // work order: query heads whose blocks are dealt long-first together (set by the launcher)
};

struct RopeParams {
    _Float16* q;               // [rows, Hq, D], rotated in place
    const _Float16* k_new;     // [rows, Hkv, D]
    const _Float16* v_new;     // [rows, Hkv, D]
    _Float16* resp_k_row;      // row t of resp_k: [rows, Hkv, D]
    _Float16* resp_v_row;
    const int32_t* positions;  // [B] or null
    int pos_default;           // Lp + t
    int W, Hq, Hkv, D;
    int R;                     // rotary dimension
    double log2_base;
};

constexpr int kMaxStepsPerChunk = 256;   // response steps one work-group can resolve
constexpr int kMaxListEntries = 1024;    // (step, slot) rows of one chunk: steps * beam <= this
// LDS budget of the matrix-core decode kernel: 8 waves with the whole 160 KB of a
// CU, or 4 waves with half of it so that two work-groups share a CU.  Whatever
// the tiles, the Q tile and the merge statistics leave is the response list,
// whose capacity bounds the response steps one work-group can walk.
constexpr int mfma_key_tile(int D) { return D == 256 ? 16 : 32; }
constexpr int mfma_region_bytes(int D, int QT)
{
    const int tiles = 2 * mfma_key_tile(D) * (2 * D + 16);
    const int merge = QT * (D + 4) * 4;
    return tiles > merge ? tiles : merge;
}
constexpr int mfma_list_capacity(int D, int QT, int NW, int heads_per_row = 1)
{
    const int fixed = NW * mfma_region_bytes(D, QT) + QT * (2 * D + 16) +
                      NW * heads_per_row * QT * 8 + 64;
    const int budget = (NW == 8 ? 160 : 80) * 1024 - 256;
    const int cap = (budget - fixed) / 4;
    return cap < 64 ? 0 : ((cap > 16384 ? 16384 : cap) & ~63);
}
// A request's lineage list: {entries, steps covered, 0, 0} ahead of the entries.
constexpr int kLineageHeaderWords = 4;
constexpr int kProbeGroups = 4096;       // work-groups (and sink words) of the read probe

hipError_t launch_sdpa_decode(const SdpaParams& p, int D, int QB, int HP, unsigned grid,
                              hipStream_t st);
hipError_t launch_sdpa_decode_mfma(const SdpaParams& p, int D, int QT, int NW, unsigned grid,
                                   hipStream_t st);
hipError_t launch_sdpa_prefill(const PrefillParams& p, int D, hipStream_t st);
hipError_t launch_mfma_rate_probe(const void* operands, float* out, unsigned long long* clocks,
                                  int n_groups, int iters, hipStream_t st);
hipError_t launch_sdpa_merge(_Float16* out, const float* ws_ml, const float* ws_acc, int NQ, int D,
                             int n_chunks, hipStream_t st);
hipError_t launch_append_kv(void* dst_k, void* dst_v, const void* src_k, const void* src_v,
                            size_t bytes, hipStream_t st);
hipError_t launch_lineage_update(uint32_t* lineage, const int32_t* parent_row, int B, int W, int t,
                                 int stride, hipStream_t st);
hipError_t launch_rope_append(const RopeParams& p, int interleaved, int rows, hipStream_t st);
hipError_t launch_stream_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st);

}  // namespace segkv
