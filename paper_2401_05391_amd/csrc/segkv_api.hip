// libsegkv C-ABI layer: argument validation, launch planning, kernel launches.
// Declarations and the full contract are in include/segkv.h.
#include "segkv.h"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "segkv_launch.h"

// Scratch of segkv_sdpa_decode_static_scratch: one copy per GPU the library runs
// on, held until the process ends.  The name is a host-side stand-in, not a
// device address: host code only ever uses the pointer hipGetSymbolAddress
// returns for the current device (static_scratch_ptr below).
static __device__ __align__(256) unsigned char scratch[SEGKV_STATIC_SCRATCH_BYTES];

namespace {

using segkv::SdpaParams;

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
// Allocates nothing.  Null on failure.
void* static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // a racing thread stores the same value
    return ptr;
}

struct Plan {
    int G, nq, QB, n_qblocks;
    int HP;   // adjacent KV heads handled by one wave-wide load (ALU path)
    int mfma; // 1: matrix-core kernel, 0: vector-ALU kernel
    int NW;   // waves per work-group of the matrix-core kernel
    int merged, n_chunks, pchunk, rchunk, n_rchunks, n_pchunks, resp_in_last;
    size_t ws_ml_bytes, ws_acc_bytes;
    int pair;           // 1: two adjacent 64-wide heads per 256-byte row, run as D = 128 (see make_plan)
    int D, Hq, Hkv;     // the dimensions the kernel is launched with (halved head counts when pair)
    unsigned grid;
};

int env_int(const char* name)
{
    const char* s = std::getenv(name);
    if (!s || !*s) return 0;
    const long v = std::strtol(s, nullptr, 10);
    return v > 0 ? (int)v : 0;
}

segkv::Tuning read_tuning_from_environment()
{
    segkv::Tuning t{};
    const char* path = std::getenv("SEGKV_PATH");
    t.path = (path && path[0] == 'a') ? 1 : (path && path[0] == 'm') ? 2 : 0;
    const char* pair = std::getenv("SEGKV_PAIR_HEADS");
    t.pair_heads = (pair && *pair) ? (pair[0] != '0' ? 1 : 0) : -1;
    t.target_groups = env_int("SEGKV_TARGET_GROUPS");
    t.min_pchunk = env_int("SEGKV_MIN_PCHUNK");
    t.mfma_waves = env_int("SEGKV_MFMA_WAVES");
    t.heads_per_wave = env_int("SEGKV_HEADS_PER_WAVE");
    const char* xho = std::getenv("SEGKV_XCD_HEAD_ORDER");
    t.xcd_head_order = (xho && xho[0] == '0') ? 0 : 1;
    const char* prefill = std::getenv("SEGKV_PREFILL");
    t.prefill_regs = (prefill && prefill[0] == 'r') ? 1 : 0;
    return t;
}

std::mutex g_tuning_mutex;
std::atomic<bool> g_tuning_ready{false};
segkv::Tuning g_tuning;

// Text of the last HIP error a launch of this thread returned (segkv_status_string).
thread_local hipError_t t_last_hip_error = hipSuccess;
inline int hip_status(hipError_t e)
{
    if (e == hipSuccess) return SEGKV_OK;
    t_last_hip_error = e;
    return SEGKV_HIP_ERROR;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

constexpr int kResponseGrowthStep = 16;   // Section 3.2: response capacity grows by 16 rows

bool dims_ok(const segkv_dims* d)
{
    return d && d->B >= 1 && d->beam >= 1 && d->Hkv >= 1 && d->Hq >= 1 && d->Hq % d->Hkv == 0 &&
           d->D >= 1 && d->Lp >= 0 && d->T >= 1 && d->T <= d->Tcap;
}

bool dims_supported(const segkv_dims* d)
{
    return (d->D == 64 || d->D == 128 || d->D == 256) && d->beam <= 8;
}

// Which kernel.  The matrix-core kernel, always: its tile stream (one tile in
// flight per wave, operands through LDS) is HBM-bound from a single query per
// K/V row up, and measured faster than the vector-ALU kernel at every shape
// tried, greedy decode included (Llama2-7B shape, one query per row: 10.9
// against 14.9 us at batch 1, 27 against 31 us at batch 8, 90 against 98 us at
// batch 31; the one exception found, D = 256 with one query per row and 128
// units, is 5% the other way).  The vector-ALU kernel stays in the library as
// the second implementation the tests compare (the test-only override selects it).
bool want_mfma(int /*nq*/, long /*kv_units*/)
{
    return segkv::tuning().path != 1;
}

// How the keys of one (request, KV head) unit are cut into work-groups.
// Enough work-groups to occupy 256 CUs, but chunks long enough that the fp32
// partials written per chunk stay small next to the K/V bytes the chunk reads.
//
// Multi-head attention with D = 64 is run as D = 128 with half the heads: Q, K, V
// and the output of two adjacent heads are one contiguous 256-byte row each, and
// the kernel's head-pair variant keeps the two heads' products and softmax
// states apart.  K/V rows then arrive in 256-byte instead of 128-byte pieces
// (the same bytes laid out as D = 128 stream 10-20% faster).  Pairing halves the
// number of units, so it is only done when enough remain to fill the device:
// measured faster from 384 (request, head) units up (+21% at 4096, +8% at 384 to
// 1024), slower at 256 and below.  The test-only override forces the choice.
Plan make_plan(const segkv_dims* d_in)
{
    Plan pl{};
    segkv_dims dd = *d_in;
    const segkv::Tuning& tune = segkv::tuning();
    const bool pair_possible = dd.D == 64 && dd.Hq == dd.Hkv && dd.Hkv % 2 == 0 && want_mfma(dd.beam, 0);
    const bool pair_wanted = tune.pair_heads >= 0 ? tune.pair_heads != 0 : (long)dd.B * dd.Hkv >= 384;
    pl.pair = (pair_possible && pair_wanted) ? 1 : 0;
    if (pl.pair) {
        dd.D = 128;
        dd.Hq /= 2;
        dd.Hkv /= 2;
    }
    const segkv_dims* const d = &dd;
    const int heads_per_row = pl.pair ? 2 : 1;
    pl.D = dd.D;
    pl.Hq = dd.Hq;
    pl.Hkv = dd.Hkv;
    pl.G = d->Hq / d->Hkv;
    pl.nq = d->beam * pl.G;
    pl.mfma = want_mfma(pl.nq, (long)d->B * d->Hkv) ? 1 : 0;
    int target_groups, min_pchunk;
    if (pl.mfma) {
        // query slots per work-group: the 16-slot shape when it holds all queries
        // of a unit, and always at D = 256 (accumulator registers)
        pl.QB = (pl.nq <= 16 || d->D == 256) ? 16 : 32;
        pl.HP = 1;
        target_groups = tune.target_groups ? tune.target_groups : 256;
        min_pchunk = tune.min_pchunk ? tune.min_pchunk : 256;   // one 32-key tile per wave
    } else {
        pl.QB = (pl.nq == 1) ? 1 : 4;
        // Adjacent KV heads per wave-wide load: 4 give 1 KB-contiguous reads,
        // the best streaming shape, but also 4x fewer, 4x longer units.  Keep at
        // least ~128 units; below that fall back to 2 or 1 heads per load
        // (measured: GPT-J shape fastest with 2, batch-1 shapes with 1).
        const int hp_env = tune.heads_per_wave;
        pl.HP = hp_env ? hp_env : 4;
        while (pl.HP > 1 &&
               (d->Hkv % pl.HP != 0 || (pl.HP != 2 && pl.HP != 4) ||
                (!hp_env && (long)d->B * (d->Hkv / pl.HP) * ceil_div(pl.nq, pl.QB) < 128)))
            pl.HP >>= 1;
        target_groups = tune.target_groups ? tune.target_groups : 1024;
        min_pchunk = tune.min_pchunk ? tune.min_pchunk : 64 * pl.QB;
    }
    pl.n_qblocks = ceil_div(pl.nq, pl.QB);
    const long units = (long)d->B * (d->Hkv / pl.HP) * pl.n_qblocks;

    // response steps one work-group may own.  Matrix-core kernel: one wave resolves
    // them window by window into an LDS list sized by what the tiles leave free
    // (worst case W distinct rows per step).  Vector-ALU kernel: one list thread
    // per step, at most kMaxListEntries (step, slot) rows.
    int max_steps, max_steps_merged;
    if (pl.mfma) {
        // Four-wave work-groups, two per CU, when there are more units than CUs: one
        // group's start-up and merge then overlap the other's streaming.
        pl.NW = 8;
        const long kv_units = (long)d->B * d->Hkv * ceil_div(pl.nq, pl.QB);
        const int nw_env = tune.mfma_waves;
        if (pl.QB == 16 && d->D <= 128 &&
            (nw_env == 4 || (nw_env == 0 && kv_units > 256 &&
                             d->T * d->beam <=
                                 segkv::mfma_list_capacity(d->D, pl.QB, 4, heads_per_row))))
            pl.NW = 4;
        max_steps_merged = segkv::mfma_list_capacity(d->D, pl.QB, pl.NW, heads_per_row) / d->beam;
        if (max_steps_merged > 65535) max_steps_merged = 65535;
        max_steps = max_steps_merged < segkv::kMaxStepsPerChunk ? max_steps_merged
                                                                : segkv::kMaxStepsPerChunk;
    } else {
        max_steps = segkv::kMaxListEntries / d->beam;
        if (max_steps > segkv::kMaxStepsPerChunk) max_steps = segkv::kMaxStepsPerChunk;
        max_steps_merged = max_steps;
    }

    if (d->T <= max_steps_merged && units >= target_groups) {
        pl.merged = 1;
        pl.n_chunks = 1;
        pl.n_rchunks = 1;
        pl.rchunk = d->T;
        pl.n_pchunks = d->Lp > 0 ? 1 : 0;
        pl.pchunk = d->Lp > 0 ? d->Lp : 1;
    } else if (pl.mfma && d->T <= max_steps_merged) {
        // Too few units to fill the device, response short enough for one list: cut
        // the unit's rows (prompt rows plus the distinct response rows expected)
        // into equal runs.  The last run takes the tail of the prompt and the whole
        // response, so that no work-group is left with the response alone.
        long resp_rows = d->beam == 1 ? d->T : (long)d->T + d->T / 8 + 8;
        if (resp_rows > (long)d->T * d->beam) resp_rows = (long)d->T * d->beam;
        const long total = d->Lp + resp_rows;
        // as many runs as fit the device in one round (one work-group per CU): a few
        // work-groups left over for a second round would cost a whole run's time
        const long want = target_groups / units > 1 ? target_groups / units : 1;
        long run = (total + want - 1) / want;
        if (run < min_pchunk) run = min_pchunk;
        run = (run + 31) / 32 * 32;
        const int np = d->Lp > 0 ? ceil_div(d->Lp, (int)run) : 0;
        const long last_prompt = np > 0 ? d->Lp - (long)(np - 1) * run : 0;
        const bool fold = np > 0 && last_prompt + resp_rows <= run + run / 4;
        pl.resp_in_last = 1;
        pl.n_rchunks = 0;
        pl.rchunk = d->T;
        pl.pchunk = (int)run;
        pl.n_pchunks = np;
        pl.n_chunks = fold ? np : np + 1;
        pl.merged = pl.n_chunks == 1 ? 1 : 0;
    } else {
        pl.merged = 0;
        pl.n_rchunks = ceil_div(d->T, max_steps);
        pl.rchunk = ceil_div(d->T, pl.n_rchunks);
        if (d->Lp > 0) {
            long want = (target_groups + units - 1) / units - pl.n_rchunks;
            const int most = ceil_div(d->Lp, min_pchunk);
            if (want < 1) want = 1;
            if (want > most) want = most;
            pl.pchunk = ceil_div(ceil_div(d->Lp, (int)want), 32) * 32;
            pl.n_pchunks = ceil_div(d->Lp, pl.pchunk);
        } else {
            pl.pchunk = 1;
            pl.n_pchunks = 0;
        }
        pl.n_chunks = pl.n_rchunks + pl.n_pchunks;
    }
    const size_t NQ = (size_t)d->B * d->beam * d->Hq;
    if (pl.n_chunks > 1) {
        pl.ws_ml_bytes =
            ((size_t)pl.n_chunks * NQ * heads_per_row * 2 * sizeof(float) + 15) & ~(size_t)15;
        pl.ws_acc_bytes = (size_t)pl.n_chunks * NQ * d->D * sizeof(float);
    }
    pl.grid = (unsigned)(units * pl.n_chunks);
    return pl;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// XCD-aware placement of KV heads for the matrix-core kernel.  Work-group i runs
// on XCD i % 8 and consecutive work-groups take consecutive KV heads, so with a
// multiple of eight heads every XCD streams the same heads (mod 8) of every
// request, i.e. fixed 256-byte columns of the K/V rows.  Two things are uneven on
// MI355X, both measured with per-work-group time stamps on the Llama2-70B shape
// (256 work-groups, one per CU): the columns whose address bits 9:8 are 01 are
// served more slowly (a head that streams one finishes 3-4 us later than one
// that streams none), and the odd-numbered XCDs get a smaller share of the HBM
// bandwidth than the even ones (about 2 us between their means).  The kernel
// ends with its slowest work-group, so the heads with slow columns go to the
// even XCDs.  Returns nibble j = head (mod 8) for position j of every aligned
// run of eight heads; the identity when nothing is known to be uneven.
uint32_t xcd_aware_head_order(const void* k_base, const void* v_base, int head_bytes)
{
    constexpr uint32_t kIdentity = 0x76543210u;
    if (!k_base || !v_base || head_bytes < 128 || head_bytes > 1024) return kIdentity;
    int score[8];
    for (int j = 0; j < 8; ++j) {
        score[j] = 0;
        for (int off = 0; off < head_bytes; off += 128) {
            const uintptr_t ak = (uintptr_t)k_base + (uintptr_t)j * head_bytes + off;
            const uintptr_t av = (uintptr_t)v_base + (uintptr_t)j * head_bytes + off;
            score[j] += (((ak >> 8) & 3u) == 1u) + (((av >> 8) & 3u) == 1u);
        }
    }
    int heads[8] = {0, 1, 2, 3, 4, 5, 6, 7};
    // stable insertion sort, slowest first
    for (int i = 1; i < 8; ++i)
        for (int k = i; k > 0 && score[heads[k]] > score[heads[k - 1]]; --k) {
            const int t = heads[k];
            heads[k] = heads[k - 1];
            heads[k - 1] = t;
        }
    static const int kXcdFastFirst[8] = {0, 2, 4, 6, 1, 3, 5, 7};
    uint32_t perm = 0;
    for (int k = 0; k < 8; ++k) perm |= (uint32_t)heads[k] << (4 * kXcdFastFirst[k]);
    return perm;
}

// A lineage list of `capacity` entries per request can hold `steps` steps of this beam width.
bool lineage_ok(int32_t capacity, int32_t steps, const segkv_dims* d)
{
    return d && d->B >= 1 && d->beam >= 1 && d->beam <= 8 && capacity >= 4 && capacity % 4 == 0 &&
           steps >= 1 && steps < (1 << 16) && (long)steps * d->beam <= capacity;
}

}  // namespace

namespace segkv {

const Tuning& tuning()
{
    if (!g_tuning_ready.load(std::memory_order_acquire)) reload_tuning();
    return g_tuning;
}

void reload_tuning()
{
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    g_tuning = read_tuning_from_environment();
    g_tuning_ready.store(true, std::memory_order_release);
}

}  // namespace segkv

extern "C" {

void segkv_reload_tuning(void) { segkv::reload_tuning(); }

const char* segkv_status_string(int status)
{
    switch (status) {
        case SEGKV_OK: return "ok";
        case SEGKV_INVALID_ARG: return "invalid argument";
        case SEGKV_UNSUPPORTED: return "unsupported head dimension or beam width";
        case SEGKV_MISALIGNED: return "tensor pointer is not 16-byte aligned";
        case SEGKV_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SEGKV_HIP_ERROR: {
            // the runtime's own text for the launch this thread last had rejected
            static thread_local char text[160];
            std::snprintf(text, sizeof text, "HIP runtime rejected a kernel launch: %s",
                          t_last_hip_error == hipSuccess ? "no launch of this thread has failed"
                                                         : hipGetErrorString(t_last_hip_error));
            return text;
        }
        case SEGKV_STATIC_SCRATCH_EXCEEDED:
            return "these dimensions need more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

size_t segkv_workspace_bytes(const segkv_dims* d)
{
    if (!dims_ok(d) || !dims_supported(d)) return 0;
    const Plan pl = make_plan(d);
    return pl.ws_ml_bytes + pl.ws_acc_bytes;
}

size_t segkv_value_stagger_bytes(const segkv_dims* d)
{
    if (!dims_ok(d) || !dims_supported(d)) return 0;
    // only the per-head column streams of the matrix-core kernel gain from it:
    // 256 to step off the slow address class, 4096 to part row i of K from row i of V
    const Plan pl = make_plan(d);
    return (pl.mfma && pl.D * 2 == 256) ? 4096 + 256 : 0;
}

int segkv_append_kv(void* resp_k, void* resp_v, const void* k_new, const void* v_new, int32_t t,
                    const segkv_dims* d, void* stream)
{
    if (!d || !resp_k || !resp_v || !k_new || !v_new) return SEGKV_INVALID_ARG;
    if (d->B < 1 || d->beam < 1 || d->Hkv < 1 || d->D < 1 || d->Tcap < 1) return SEGKV_INVALID_ARG;
    if (t < 0 || t >= d->Tcap) return SEGKV_INVALID_ARG;
    if ((d->D % 8) != 0) return SEGKV_UNSUPPORTED;
    if (misaligned(resp_k) || misaligned(resp_v) || misaligned(k_new) || misaligned(v_new))
        return SEGKV_MISALIGNED;
    const size_t row_bytes = (size_t)d->B * d->beam * d->Hkv * d->D * 2;
    char* dk = (char*)resp_k + (size_t)t * row_bytes;
    char* dv = (char*)resp_v + (size_t)t * row_bytes;
    const hipError_t e = segkv::launch_append_kv(dk, dv, k_new, v_new, row_bytes, (hipStream_t)stream);
    return hip_status(e);
}

int segkv_sdpa_decode(void* out, const void* q, const void* prompt_k, const void* prompt_v,
                      void* resp_k, void* resp_v, const int32_t* parent, const void* k_new,
                      const void* v_new, const float* alibi_slopes, int32_t* anc_out,
                      void* workspace, size_t workspace_bytes, float scale, const segkv_dims* d,
                      void* stream)
{
    return segkv_sdpa_decode_ragged(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, k_new, v_new,
                                    alibi_slopes, nullptr, anc_out, workspace, workspace_bytes, scale,
                                    d, stream);
}

namespace {

// prompt_seq_first: prompt_k / prompt_v are [Lp, B, Hkv, D] instead of [B, Lp, Hkv, D]
int sdpa_decode_impl(void* out, const void* q, const void* prompt_k, const void* prompt_v,
                     void* resp_k, void* resp_v, const int32_t* parent, const void* k_new,
                     const void* v_new, const float* alibi_slopes, const int32_t* prompt_lens,
                     bool prompt_seq_first, int32_t* anc_out, void* workspace,
                     size_t workspace_bytes, float scale, const segkv_dims* d, void* stream,
                     const void* lineage = nullptr, int32_t lineage_capacity = 0)
{
    if (!dims_ok(d)) return SEGKV_INVALID_ARG;
    if (lineage && !lineage_ok(lineage_capacity, d->T, d)) return SEGKV_INVALID_ARG;
    if (!out || !q || !resp_k || !resp_v) return SEGKV_INVALID_ARG;
    if (d->Lp > 0 && (!prompt_k || !prompt_v)) return SEGKV_INVALID_ARG;
    if (d->beam > 1 && !parent && !lineage) return SEGKV_INVALID_ARG;
    if ((k_new == nullptr) != (v_new == nullptr)) return SEGKV_INVALID_ARG;
    if (!dims_supported(d)) return SEGKV_UNSUPPORTED;
    if ((long)d->B * d->beam * d->Hq > (1L << 28)) return SEGKV_UNSUPPORTED;
    // a tile's rows are addressed with 32-bit element offsets from the tile's base
    if ((long)d->Hkv * d->D > (1L << 25)) return SEGKV_UNSUPPORTED;
    if (prompt_seq_first && (long)d->B * d->Hkv * d->D > (1L << 25)) return SEGKV_UNSUPPORTED;
    if (misaligned(out) || misaligned(q) || misaligned(resp_k) || misaligned(resp_v) ||
        (d->Lp > 0 && (misaligned(prompt_k) || misaligned(prompt_v))) ||
        (k_new && (misaligned(k_new) || misaligned(v_new))) || misaligned(workspace) ||
        ((uintptr_t)parent & 3u) || ((uintptr_t)alibi_slopes & 3u) || ((uintptr_t)anc_out & 3u) ||
        ((uintptr_t)prompt_lens & 3u))
        return SEGKV_MISALIGNED;

    if (misaligned(lineage)) return SEGKV_MISALIGNED;
    const Plan pl = make_plan(d);
    if (lineage && !pl.mfma) return SEGKV_UNSUPPORTED;      // the vector-ALU kernel resolves parents only
    const size_t need = pl.ws_ml_bytes + pl.ws_acc_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need)) return SEGKV_WORKSPACE_TOO_SMALL;

    SdpaParams p{};
    p.q = (const _Float16*)q;
    p.out = (_Float16*)out;
    p.prompt_k = (const _Float16*)prompt_k;
    p.prompt_v = (const _Float16*)prompt_v;
    p.resp_k = (_Float16*)resp_k;
    p.resp_v = (_Float16*)resp_v;
    p.parent = parent;
    p.k_new = (const _Float16*)k_new;
    p.v_new = (const _Float16*)v_new;
    p.slopes = alibi_slopes;
    p.prompt_lens = prompt_lens;
    p.lineage = (const uint32_t*)lineage;
    p.lineage_stride = segkv::kLineageHeaderWords + lineage_capacity;
    if (prompt_seq_first) {
        p.prompt_row_stride = (uint32_t)d->B * d->Hkv * d->D;
        p.prompt_req_stride = (size_t)d->Hkv * d->D;
    } else {
        p.prompt_row_stride = (uint32_t)d->Hkv * d->D;
        p.prompt_req_stride = (size_t)d->Lp * d->Hkv * d->D;
    }
    p.anc_out = anc_out;
    p.ws_ml = need ? (float*)workspace : nullptr;
    p.ws_acc = need ? (float*)((char*)workspace + pl.ws_ml_bytes) : nullptr;
    p.scale2 = scale * 1.4426950408889634f;
    p.B = d->B; p.W = d->beam; p.Hq = pl.Hq; p.Hkv = pl.Hkv; p.G = pl.G; p.Lp = d->Lp; p.T = d->T;
    p.head_pairs = pl.pair;
    p.nq = pl.nq;
    p.n_qblocks = pl.n_qblocks;
    p.merged = pl.merged;
    p.n_chunks = pl.n_chunks;
    p.pchunk = pl.pchunk;
    p.rchunk = pl.rchunk;
    p.n_rchunks = pl.n_rchunks;
    p.resp_in_last = pl.resp_in_last;
    p.head_perm8 = 0x76543210u;
    if (pl.mfma && pl.Hkv % 8 == 0 && segkv::tuning().xcd_head_order)
        p.head_perm8 = d->Lp > 0 ? xcd_aware_head_order(prompt_k, prompt_v, pl.D * 2)
                                 : xcd_aware_head_order(resp_k, resp_v, pl.D * 2);

    hipStream_t st = (hipStream_t)stream;
    hipError_t e = pl.mfma ? segkv::launch_sdpa_decode_mfma(p, pl.D, pl.QB, pl.NW, pl.grid, st)
                           : segkv::launch_sdpa_decode(p, d->D, pl.QB, pl.HP, pl.grid, st);
    if (e != hipSuccess) return hip_status(e);
    if (pl.n_chunks > 1) {
        e = segkv::launch_sdpa_merge(p.out, p.ws_ml, p.ws_acc, d->B * d->beam * d->Hq, d->D,
                                     pl.n_chunks, st);
        if (e != hipSuccess) return hip_status(e);
    }
    return SEGKV_OK;
}

}  // namespace

int segkv_sdpa_decode_ragged(void* out, const void* q, const void* prompt_k, const void* prompt_v,
                             void* resp_k, void* resp_v, const int32_t* parent, const void* k_new,
                             const void* v_new, const float* alibi_slopes,
                             const int32_t* prompt_lens, int32_t* anc_out, void* workspace,
                             size_t workspace_bytes, float scale, const segkv_dims* d, void* stream)
{
    return sdpa_decode_impl(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, k_new, v_new,
                            alibi_slopes, prompt_lens, false, anc_out, workspace, workspace_bytes,
                            scale, d, stream);
}

int segkv_sdpa_decode_static_scratch(void* out, const void* q, const void* prompt_k,
                                     const void* prompt_v, void* resp_k, void* resp_v,
                                     const int32_t* parent, const void* k_new, const void* v_new,
                                     const float* alibi_slopes, int32_t* anc_out, float scale,
                                     const segkv_dims* d, void* stream)
{
    if (!dims_ok(d)) return SEGKV_INVALID_ARG;
    if (!dims_supported(d)) return SEGKV_UNSUPPORTED;
    // the size check comes before anything touches the device
    const Plan pl = make_plan(d);
    const size_t need = pl.ws_ml_bytes + pl.ws_acc_bytes;
    if (need > (size_t)SEGKV_STATIC_SCRATCH_BYTES) return SEGKV_STATIC_SCRATCH_EXCEEDED;
    void* ptr = nullptr;
    if (need > 0) {
        ptr = static_scratch_ptr();
        if (!ptr) return hip_status(hipErrorInvalidSymbol);
    }
    // The partials need no clearing: every chunk's work-group writes its whole
    // slice before the merge pass reads it.
    return sdpa_decode_impl(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, k_new, v_new,
                            alibi_slopes, nullptr, false, anc_out, ptr, need, scale, d, stream);
}

int segkv_sdpa_decode_lineage(void* out, const void* q, const void* prompt_k, const void* prompt_v,
                              void* resp_k, void* resp_v, const void* lineage,
                              int32_t lineage_capacity, const void* k_new, const void* v_new,
                              const float* alibi_slopes, const int32_t* prompt_lens, void* workspace,
                              size_t workspace_bytes, float scale, const segkv_dims* d, void* stream)
{
    if (!lineage) return SEGKV_INVALID_ARG;
    return sdpa_decode_impl(out, q, prompt_k, prompt_v, resp_k, resp_v, nullptr, k_new, v_new,
                            alibi_slopes, prompt_lens, false, nullptr, workspace, workspace_bytes,
                            scale, d, stream, lineage, lineage_capacity);
}

size_t segkv_lineage_bytes(const segkv_dims* d, int32_t lineage_capacity)
{
    if (!d || d->B < 1 || lineage_capacity < 4 || lineage_capacity % 4 != 0) return 0;
    return (size_t)d->B * (segkv::kLineageHeaderWords + (size_t)lineage_capacity) * sizeof(uint32_t);
}

int segkv_lineage_update(void* lineage, int32_t lineage_capacity, const int32_t* parent_row,
                         int32_t t, const segkv_dims* d, void* stream)
{
    if (!lineage || t < 0 || !lineage_ok(lineage_capacity, t + 1, d)) return SEGKV_INVALID_ARG;
    if (t > 0 && d->beam > 1 && !parent_row) return SEGKV_INVALID_ARG;
    if (misaligned(lineage) || ((uintptr_t)parent_row & 3u)) return SEGKV_MISALIGNED;
    const hipError_t e = segkv::launch_lineage_update(
        (uint32_t*)lineage, parent_row, d->B, d->beam, t,
        segkv::kLineageHeaderWords + lineage_capacity, (hipStream_t)stream);
    return hip_status(e);
}

int segkv_sdpa_decode_seq_first_prompt(void* out, const void* q, const void* prompt_k,
                                       const void* prompt_v, void* resp_k, void* resp_v,
                                       const int32_t* parent, const void* k_new, const void* v_new,
                                       const float* alibi_slopes, const int32_t* prompt_lens,
                                       int32_t* anc_out, void* workspace, size_t workspace_bytes,
                                       float scale, const segkv_dims* d, void* stream)
{
    return sdpa_decode_impl(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, k_new, v_new,
                            alibi_slopes, prompt_lens, true, anc_out, workspace, workspace_bytes,
                            scale, d, stream);
}

int segkv_rope_append(void* q, const void* k_new, const void* v_new, void* resp_k, void* resp_v,
                      const int32_t* positions, int32_t t, float rope_base, int32_t rotary_dim,
                      int32_t interleaved, const segkv_dims* d, void* stream)
{
    if (!d || !q || !k_new || !v_new || !resp_k || !resp_v) return SEGKV_INVALID_ARG;
    if (d->B < 1 || d->beam < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1 || d->Lp < 0 || d->Tcap < 1)
        return SEGKV_INVALID_ARG;
    if (t < 0 || t >= d->Tcap) return SEGKV_INVALID_ARG;
    if (!(rope_base > 0.0f) || rotary_dim < 0 || rotary_dim > d->D) return SEGKV_INVALID_ARG;
    if ((d->D % 8) != 0 || rotary_dim > 256 || (rotary_dim % (interleaved ? 8 : 16)) != 0)
        return SEGKV_UNSUPPORTED;
    if (misaligned(q) || misaligned(k_new) || misaligned(v_new) || misaligned(resp_k) ||
        misaligned(resp_v) || ((uintptr_t)positions & 3u))
        return SEGKV_MISALIGNED;
    const size_t row_elems = (size_t)d->B * d->beam * d->Hkv * d->D;
    segkv::RopeParams p{};
    p.q = (_Float16*)q;
    p.k_new = (const _Float16*)k_new;
    p.v_new = (const _Float16*)v_new;
    p.resp_k_row = (_Float16*)resp_k + (size_t)t * row_elems;
    p.resp_v_row = (_Float16*)resp_v + (size_t)t * row_elems;
    p.positions = positions;
    p.pos_default = d->Lp + t;
    p.W = d->beam; p.Hq = d->Hq; p.Hkv = d->Hkv; p.D = d->D;
    p.R = rotary_dim;
    p.log2_base = std::log2((double)rope_base);
    const hipError_t e =
        segkv::launch_rope_append(p, interleaved ? 1 : 0, d->B * d->beam, (hipStream_t)stream);
    return hip_status(e);
}

int segkv_sdpa_prefill(void* out, const void* q, const void* k, const void* v,
                       const float* alibi_slopes, float scale, const segkv_dims* d, void* stream)
{
    if (!d || !out || !q || !k || !v) return SEGKV_INVALID_ARG;
    if (d->B < 1 || d->Hkv < 1 || d->Hq < 1 || d->Hq % d->Hkv != 0 || d->D < 1 || d->Lp < 1)
        return SEGKV_INVALID_ARG;
    if (d->D != 64 && d->D != 128 && d->D != 256) return SEGKV_UNSUPPORTED;
    if ((long)d->B * d->Hq * ((d->Lp + 127) / 128) > (1L << 30)) return SEGKV_UNSUPPORTED;
    if (misaligned(out) || misaligned(q) || misaligned(k) || misaligned(v) ||
        ((uintptr_t)alibi_slopes & 3u))
        return SEGKV_MISALIGNED;
    segkv::PrefillParams p{};
    p.q = (const _Float16*)q;
    p.k = (const _Float16*)k;
    p.v = (const _Float16*)v;
    p.out = (_Float16*)out;
    p.slopes = alibi_slopes;
    p.scale2 = scale * 1.4426950408889634f;
    p.B = d->B; p.N0 = d->Lp; p.Hq = d->Hq; p.Hkv = d->Hkv; p.G = d->Hq / d->Hkv;
    const hipError_t e = segkv::launch_sdpa_prefill(p, d->D, (hipStream_t)stream);
    return hip_status(e);
}

int segkv_probe_mfma_rate(const void* operands, void* out, void* clocks, int32_t n_groups, int32_t iters,
                          void* stream)
{
    if (!operands || !out || !clocks) return SEGKV_INVALID_ARG;
    if (n_groups <= 0 || iters <= 0 || n_groups > (1 << 20)) return SEGKV_INVALID_ARG;
    if (((uintptr_t)operands & 15u) || ((uintptr_t)out & 3u) || ((uintptr_t)clocks & 7u)) return SEGKV_MISALIGNED;
    return hip_status(segkv::launch_mfma_rate_probe(operands, (float*)out, (unsigned long long*)clocks,
                                                    n_groups, iters, (hipStream_t)stream));
}

uint64_t segkv_cache_token_bytes(int32_t L, int32_t H, int32_t D, int32_t elem_bytes)
{
    if (L <= 0 || H <= 0 || D <= 0 || elem_bytes <= 0) return 0;
    return 2ull * (uint64_t)L * (uint64_t)H * (uint64_t)D * (uint64_t)elem_bytes;
}

int32_t segkv_response_capacity(int32_t n_response)
{
    if (n_response <= 0) return 0;
    return (int32_t)(((int64_t)n_response + kResponseGrowthStep - 1) / kResponseGrowthStep *
                     kResponseGrowthStep);
}

uint64_t segkv_cache_standard_bytes(int32_t BS, int32_t BW, int32_t n_prompt, int32_t n_response,
                                    uint64_t token_bytes)
{
    if (BS <= 0 || BW <= 0 || n_prompt < 0 || n_response < 0) return 0;
    return (uint64_t)BS * (uint64_t)BW * ((uint64_t)n_prompt + (uint64_t)n_response) * token_bytes;
}

uint64_t segkv_cache_segment_bytes(int32_t BS, int32_t BW, int32_t n_prompt, int32_t n_response,
                                   uint64_t token_bytes)
{
    if (BS <= 0 || BW <= 0 || n_prompt < 0 || n_response < 0) return 0;
    const uint64_t cap = (uint64_t)segkv_response_capacity(n_response);
    return (uint64_t)BS * ((uint64_t)n_prompt + (uint64_t)BW * cap) * token_bytes;
}

int segkv_grow_response(void* new_k, void* new_v, const void* old_k, const void* old_v,
                        int32_t tcap_new, const segkv_dims* d, void* stream)
{
    if (!d || !new_k || !new_v || !old_k || !old_v) return SEGKV_INVALID_ARG;
    if (d->B < 1 || d->beam < 1 || d->Hkv < 1 || d->D < 1) return SEGKV_INVALID_ARG;
    if (d->T < 0 || d->T > d->Tcap || tcap_new < d->Tcap) return SEGKV_INVALID_ARG;
    if ((d->D % 8) != 0) return SEGKV_UNSUPPORTED;
    if (misaligned(new_k) || misaligned(new_v) || misaligned(old_k) || misaligned(old_v))
        return SEGKV_MISALIGNED;
    if (d->T == 0) return SEGKV_OK;
    const size_t bytes = (size_t)d->T * d->B * d->beam * d->Hkv * d->D * 2;
    const hipError_t e = segkv::launch_append_kv(new_k, new_v, old_k, old_v, bytes, (hipStream_t)stream);
    return hip_status(e);
}

int segkv_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || (bytes & 15u)) return SEGKV_INVALID_ARG;
    if (misaligned(src) || ((uintptr_t)sink & 3u)) return SEGKV_MISALIGNED;
    const hipError_t e = segkv::launch_stream_read_probe(src, bytes, sink, (hipStream_t)stream);
    return hip_status(e);
}

}  // extern "C"
