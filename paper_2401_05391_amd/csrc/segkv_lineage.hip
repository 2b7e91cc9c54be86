// libsegkv device code: the per-request lineage list kept across decode steps
// (arxiv 2401.05391, Section 3.3: the kernel's index tensor says which response
// row every beam reads at every past step, and is brought up to date once per
// generated token, the way FasterTransformer keeps its beam-search cache
// indirection).  Here the tensor is held with equal rows merged: one entry
//     (step << 16) | (slot << 8) | mask      mask bit j: beam j reads the row
// per distinct (step, slot) row that some beam of the request still descends
// from, ordered by step and by slot within a step -- the list the attention
// kernel otherwise derives from the raw parent table in every work-group of
// every layer.
//
// One generated token: beam j now reads, at every earlier step, what beam
// parent[j] read before.  An entry keeps the beams whose parent was among its
// readers and is dropped when none was; the new step adds one row per beam.
// O(entries) work, no dependency between entries: one work-group per request
// re-maps 256 entries at a time and compacts them in place (an entry only ever
// moves towards the front, behind positions that were read in the same or an
// earlier pass).
#include "segkv_common.h"
#include "segkv_launch.h"

namespace segkv {

constexpr int kLineageThreads = 256;

__global__ __launch_bounds__(kLineageThreads) void lineage_update_kernel(uint32_t* lineage,
                                                                          const int32_t* parent_row,
                                                                          int W, int t, int stride)
{
    __shared__ int s_kept[kLineageThreads / 64];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    uint32_t* const hdr = lineage + (size_t)b * stride;
    uint32_t* const ent = hdr + kLineageHeaderWords;
    const int room = stride - kLineageHeaderWords - W;       // entries that may survive
    const int n_old = (t > 0) ? min((int)hdr[0], room) : 0;

    // the step's parent row, one byte per beam (entries are trusted to lie in
    // [0, W); clamping keeps a bad row from selecting bits outside the mask)
    int par[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        par[j] = (j < W && t > 0 && parent_row) ? min(max(parent_row[b * W + j], 0), W - 1) : j;

    int out = 0;
    for (int base = 0; base < n_old; base += kLineageThreads) {
        const int i = base + tid;
        const uint32_t e = (i < n_old) ? ent[i] : 0u;
        uint32_t mask = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < W && ((e >> par[j]) & 1u)) mask |= 1u << j;
        const bool keep = mask != 0;
        const unsigned long long votes = __ballot(keep);
        const int rank = __popcll(votes & ((1ull << lane) - 1ull));
        __syncthreads();                     // this pass's entries are all in registers
        if (lane == 0) s_kept[wave] = __popcll(votes);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kLineageThreads / 64; ++w) {
            if (w < wave) before += s_kept[w];
            total += s_kept[w];
        }
        if (keep) ent[out + before + rank] = (e & ~0xffu) | mask;
        out += total;
    }
    __syncthreads();
    if (tid < W) ent[out + tid] = ((uint32_t)t << 16) | ((uint32_t)tid << 8) | (1u << tid);
    if (tid == 0) {
        hdr[0] = (uint32_t)(out + W);        // entries
        hdr[1] = (uint32_t)(t + 1);          // steps covered
    }
}

hipError_t launch_lineage_update(uint32_t* lineage, const int32_t* parent_row, int B, int W, int t,
                                 int stride, hipStream_t st)
{
    return SEGKV_LAUNCH(lineage_update_kernel, dim3(B), dim3(kLineageThreads), st, lineage, parent_row,
                        W, t, stride);
}

}  // namespace segkv
