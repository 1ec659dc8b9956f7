// extern "C" entry points of libffsnap.so (see include/ffsnap.h for the contract).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/ffsnap.h"
#include "gf2.h"
#include "fused.hpp"
#include "kernels.hpp"
#include "layout.hpp"

using namespace ffsnap;

// ---- scratch of ff_crc32c_noalloc ---------------------------------------------------------------
// The reduction tables of the tile kernel (kTabWords entries) followed by one CRC register per
// 1 MiB tile of the buffer.  The array lives in every GPU's memory from the moment the library is
// loaded there until the process ends.  In host code `scratch` only names the symbol: the device
// address is looked up once per device (scratch_for_current_device) and that pointer is what the
// kernels, and the one-time table upload, are given.
constexpr uint32_t kNoallocTileRows = 1024;  // 1 MiB per tile, as in ff_crc32c
constexpr uint64_t kNoallocMaxTiles = FF_CRC32C_NOALLOC_MAX_BYTES / (1024ull * kNoallocTileRows);
static __device__ __align__(256) uint32_t scratch[kTabWords + kNoallocMaxTiles];

// Nothing in a plan changes after ff_snapshot_plan has returned: every call reads it, and the
// device tables behind it, only.  What a call needs beyond them travels in kernel arguments or
// lives in the caller's own output arrays.
struct ff_plan {
    Layout layout;
    bool host_only = false;
    int device = -1;
    void* dev_block = nullptr;  // one allocation holding every device table
    TileTables tables;
    // A pass that only reads (verify) runs fastest on larger tiles than one that also writes:
    // it folds verify_group consecutive tiles as one.
    uint32_t verify_group = 1;
    uint32_t affine = 0;  // preset/complement term of a chunk_bytes-long CRC
    // fused optimizer step (only when every parameter group is complete)
    const WorkTile* work = nullptr;
    uint32_t n_work = 0;        // all work tiles: parameter tiles first, then RAW tiles
    uint32_t n_work_param = 0;
    uint32_t fused_xcd_group = 4;  // XCD-aware order of the fused step's tiles (kernels.hpp)
    uint32_t mix_xcd_group = 16;   // ... and of the bare traffic pattern (its own best)
    // entry k: first parameter tile of parameter group k * kGradsPerLaunch; last entry: n_work_param
    std::vector<uint32_t> group_tile_begin;
    const uint32_t* fused_tabs = nullptr;
};

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e)
{
    std::snprintf(g_hip_error, sizeof(g_hip_error), "%s", hipGetErrorString(e));
    return FF_ERR_HIP;
}

#define FF_HIP_TRY(expr)                       \
    do {                                       \
        hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) return hip_fail(e_); \
    } while (0)

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t* g_scratch_ptr[kMaxDevices] = {};  // per device: address of `scratch`, tables uploaded

// Device address of `scratch` on the current device; on the first call per device the reduction
// tables are written behind it (a synchronous copy: no allocation, no stream involved).
int scratch_for_current_device(uint32_t** out)
{
    int dev = -1;
    FF_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return FF_ERR_INVALID;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        uint32_t* ptr = nullptr;
        FF_HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) return FF_ERR_HIP;
        uint32_t tab[kTabWords];
        build_tab_u(tab);
        FF_HIP_TRY(hipMemcpy(ptr, tab, sizeof(tab), hipMemcpyHostToDevice));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FF_OK;
}


int upload_tables(ff_plan* p)
{
    const Layout& L = p->layout;
    const uint64_t n = L.segs.size();
    const uint64_t o_off = 0;
    const uint64_t o_ptr = align_up(o_off + (n + 1) * 8, 256);
    const uint64_t o_first = align_up(o_ptr + n * 8, 256);
    const uint64_t o_tab = align_up(o_first + L.n_tiles * 4, 256);
    std::vector<WorkTile> work;
    if (L.adam_ok && !L.params.empty()) build_work_tiles(L, work);
    if (work.size() > 0xFFFFFFF0ull) return FF_ERR_INVALID;
    const uint64_t o_work = align_up(o_tab + kTabWords * 4, 256);
    const uint64_t o_ftabs = align_up(o_work + work.size() * sizeof(WorkTile), 256);
    const uint64_t o_tbase = align_up(o_ftabs + kFusedTabWords * 4, 256);
    const uint64_t o_shift = align_up(o_tbase + L.n_tiles * 8, 256);
    const uint64_t total = align_up(o_shift + uint64_t(L.tiles_per_chunk) * 4, 256);

    std::vector<unsigned char> host(total, 0);
    uint64_t* h_off = reinterpret_cast<uint64_t*>(host.data() + o_off);
    uint64_t* h_ptr = reinterpret_cast<uint64_t*>(host.data() + o_ptr);
    for (uint64_t i = 0; i < n; i++) {
        h_off[i] = L.segs[i].off;
        h_ptr[i] = L.segs[i].ptr;
    }
    h_off[n] = L.payload;
    std::memcpy(host.data() + o_first, L.tile_first_seg.data(), L.n_tiles * 4);
    std::memcpy(host.data() + o_tbase, L.tile_base.data(), L.n_tiles * 8);
    {
        // x^(32 + 8 * bytes behind tile k of a chunk), from the last tile (x^32) backwards: the
        // factor x^32 is the one a tile's register lacks
        uint32_t* h_shift = reinterpret_cast<uint32_t*>(host.data() + o_shift);
        const uint32_t x_tile = gf2_xpow(8 * L.tile_bytes);
        uint32_t v = kX32;
        for (uint32_t k = L.tiles_per_chunk; k-- > 0;) {
            h_shift[k] = v;
            v = gf2_mul(v, x_tile);
        }
    }
    build_tab_u(reinterpret_cast<uint32_t*>(host.data() + o_tab));
    if (!work.empty()) std::memcpy(host.data() + o_work, work.data(), work.size() * sizeof(WorkTile));
    build_fused_tabs(reinterpret_cast<uint32_t*>(host.data() + o_ftabs));

    FF_HIP_TRY(hipGetDevice(&p->device));
    hipError_t e = hipMalloc(&p->dev_block, total);
    if (e == hipErrorOutOfMemory) return FF_ERR_NOMEM;
    FF_HIP_TRY(e);
    FF_HIP_TRY(hipMemcpy(p->dev_block, host.data(), total, hipMemcpyHostToDevice));

    unsigned char* d = static_cast<unsigned char*>(p->dev_block);
    TileTables& t = p->tables;
    t.seg_off = reinterpret_cast<const uint64_t*>(d + o_off);
    t.seg_ptr = reinterpret_cast<const uint64_t*>(d + o_ptr);
    t.tile_first_seg = reinterpret_cast<const uint32_t*>(d + o_first);
    t.tile_base = reinterpret_cast<const uint64_t*>(d + o_tbase);
    t.tile_shift = reinterpret_cast<const uint32_t*>(d + o_shift);
    t.tab_u = reinterpret_cast<const uint32_t*>(d + o_tab);
    p->work = reinterpret_cast<const WorkTile*>(d + o_work);
    p->n_work = static_cast<uint32_t>(work.size());
    p->n_work_param = 0;
    for (const WorkTile& w : work) p->n_work_param += (w.kind == kWorkParam) ? 1u : 0u;
    // the parameter tiles are sorted by parameter group: where each launch of the fused step begins
    p->group_tile_begin.clear();
    for (uint32_t i = 0; i < p->n_work_param; i++)
        while (p->group_tile_begin.size() <= work[i].grad_index / kGradsPerLaunch)
            p->group_tile_begin.push_back(i);
    while (p->group_tile_begin.size() <= (L.params.size() + kGradsPerLaunch - 1) / kGradsPerLaunch)
        p->group_tile_begin.push_back(p->n_work_param);
    p->fused_tabs = reinterpret_cast<const uint32_t*>(d + o_ftabs);
    return FF_OK;
}

int check_device_call(const ff_plan* p)
{
    if (!p) return FF_ERR_NULL;
    if (p->host_only) return FF_ERR_HOST_ONLY;
    // the plan's tables live on the device that was current when it was built
    int dev = -1;
    FF_HIP_TRY(hipGetDevice(&dev));
    if (dev != p->device) return FF_ERR_INVALID;
    return FF_OK;
}

}  // namespace

extern "C" {

int ff_snapshot_plan(const ff_segment* segs, uint64_t n_segs, uint64_t chunk_bytes, uint32_t flags,
                     ff_plan** out)
{
    if (!out) return FF_ERR_NULL;
    *out = nullptr;
    // bits 8..15 of flags: log2 of the tile size in bytes (0 = default), a tuning knob
    const unsigned tile_log2 = (flags >> 8) & 0xFFu;
    if (flags & ~(FF_PLAN_HOST_ONLY | 0xFF00u | 0x70000u | 0xF80000u)) return FF_ERR_INVALID;
    ff_plan* p = new (std::nothrow) ff_plan();
    if (!p) return FF_ERR_NOMEM;
    int rc;
    try {
        rc = build_layout(segs, n_segs, chunk_bytes, tile_log2, p->layout);
    } catch (const std::bad_alloc&) {
        rc = FF_ERR_NOMEM;
    }
    if (rc != FF_OK) {
        delete p;
        return rc;
    }
    const Layout& L = p->layout;
    p->host_only = (flags & FF_PLAN_HOST_ONLY) != 0;
    p->affine = crc_affine_term(L.chunk_bytes);
    while (L.tile_bytes * p->verify_group < kVerifyTileBytes &&
           p->verify_group * 2 <= L.tiles_per_chunk)
        p->verify_group *= 2;  // tiles_per_chunk is a power of two
    TileTables& t = p->tables;
    t.payload = L.payload;
    t.total_rows = L.buffer_bytes / 1024;
    t.n_seg = static_cast<uint32_t>(L.segs.size());
    t.tile_rows = static_cast<uint32_t>(L.tile_bytes / 1024);
    t.lead_rows = 0;
    t.n_tiles = static_cast<uint32_t>(L.n_tiles);
    t.tiles_per_chunk = L.tiles_per_chunk;
    while ((1u << t.tpc_log2) < L.tiles_per_chunk) t.tpc_log2++;
    // bits 16..18: bit 18 set = take bits 16..17 as the cache-hint selector (tuning knob)
    if (flags & 0x40000u) t.hint = (flags >> 16) & 3u;
    // bits 19..23: 0 = default, else log2(xcd_group) + 1, 31 = no regrouping (tuning knob)
    {
        const unsigned xg = (flags >> 19) & 31u;
        if (xg == 30u) {  // 8 * 2^29 workgroups per round does not fit the 32-bit launch index
            delete p;
            return FF_ERR_INVALID;
        }
        if (xg == 31u) t.xcd_group = p->fused_xcd_group = p->mix_xcd_group = 0;
        else if (xg) t.xcd_group = p->fused_xcd_group = p->mix_xcd_group = 1u << (xg - 1);
    }
    if (L.n_tiles > 0xFFFFFFF0ull) {
        delete p;
        return FF_ERR_INVALID;
    }
    if (!p->host_only) {
        try {
            rc = upload_tables(p);
        } catch (const std::bad_alloc&) {
            rc = FF_ERR_NOMEM;
        }
        if (rc != FF_OK) {
            if (p->dev_block) (void)hipFree(p->dev_block);
            delete p;
            return rc;
        }
    }
    *out = p;
    return FF_OK;
}

void ff_plan_destroy(ff_plan* plan)
{
    if (!plan) return;
    if (plan->dev_block) (void)hipFree(plan->dev_block);
    delete plan;
}

uint64_t ff_plan_payload_bytes(const ff_plan* p) { return p ? p->layout.payload : 0; }
uint64_t ff_plan_num_chunks(const ff_plan* p) { return p ? p->layout.n_chunks : 0; }
uint64_t ff_plan_buffer_bytes(const ff_plan* p) { return p ? p->layout.buffer_bytes : 0; }
uint64_t ff_plan_chunk_bytes(const ff_plan* p) { return p ? p->layout.chunk_bytes : 0; }
uint64_t ff_plan_num_segments(const ff_plan* p) { return p ? p->layout.segs.size() : 0; }
uint64_t ff_plan_num_params(const ff_plan* p) { return p ? p->layout.params.size() : 0; }
uint32_t ff_plan_layout_id(const ff_plan* p) { return p ? p->layout.layout_id : 0; }

int ff_plan_segment_range(const ff_plan* p, uint64_t i, uint64_t* begin, uint64_t* end)
{
    if (!p || !begin || !end) return FF_ERR_NULL;
    if (i >= p->layout.segs.size()) return FF_ERR_INVALID;
    *begin = p->layout.segs[i].off;
    *end = p->layout.segs[i].off + p->layout.segs[i].nbytes;
    return FF_OK;
}

int ff_razor_select(const ff_segment* segs, uint64_t n_segs, const ff_razor_config* cfg,
                    uint32_t which, uint64_t* out_indices, uint64_t* n_out)
{
    if ((n_segs && !segs) || !cfg || !out_indices || !n_out) return FF_ERR_NULL;
    if (cfg->dp_degree == 0 || cfg->distributed_optimizer > 1 || which > FF_RAZOR_REDUNDANT)
        return FF_ERR_INVALID;
    const bool weights_redundant = cfg->dp_degree > 1;                                 // rule 1
    const bool optimizer_redundant = cfg->dp_degree > 1 && !cfg->distributed_optimizer;  // rule 2
    uint64_t n = 0;
    for (uint64_t i = 0; i < n_segs; i++) {
        bool redundant;
        switch (segs[i].kind) {
        case FF_KIND_RAW: redundant = false; break;
        case FF_KIND_W16: redundant = weights_redundant; break;
        case FF_KIND_MASTER:
        case FF_KIND_M:
        case FF_KIND_V: redundant = optimizer_redundant; break;
        default: return FF_ERR_INVALID;
        }
        if (redundant == (which == FF_RAZOR_REDUNDANT)) out_indices[n++] = i;
    }
    *n_out = n;
    return FF_OK;
}

int ff_pack(const ff_plan* p, void* chunks, uint32_t* crcs, void* hip_stream)
{
    int rc = check_device_call(p);
    if (rc != FF_OK) return rc;
    if (!chunks || !crcs) return FF_ERR_NULL;
    if (reinterpret_cast<uint64_t>(chunks) % 16 || reinterpret_cast<uint64_t>(crcs) % 4)
        return FF_ERR_INVALID;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    TileTables t = p->tables;
    t.acc = crcs;
    FF_HIP_TRY(launch_preset(crcs, nullptr, 0, p->layout.n_chunks, p->affine, nullptr, nullptr, s));
    FF_HIP_TRY(launch_tiles(kPack, t, chunks, s));
    return FF_OK;
}

}  // extern "C"

namespace {

// Verify (and scatter) either every chunk or the chunks of `list` (at most kMaxListedChunks; a
// longer selection is a sequence of these).  clear_n_bad: this call starts the count.
int restore_impl(const ff_plan* p, const void* chunks, const uint32_t* crcs, uint32_t* bad,
                 uint64_t* n_bad, uint32_t flags, const ChunkList* list, bool clear_n_bad,
                 hipStream_t s)
{
    const Layout& L = p->layout;
    TileTables t = p->tables;
    t.acc = bad;  // the tiles' registers are summed in the caller's bad[]
    void* buf = const_cast<void*>(chunks);
    const bool verify_only = (flags & FF_RESTORE_VERIFY_ONLY) != 0;
    const bool skip_bad = (flags & FF_RESTORE_SKIP_BAD) != 0;
    if ((verify_only || skip_bad) && !list && verify_chunks_applicable(L.chunk_bytes, L.n_chunks) &&
        L.tile_bytes <= L.chunk_bytes / 8 && L.tile_bytes <= (1u << 16) &&
        (1u << 16) % L.tile_bytes == 0) {
        // pass 1 over a whole buffer of many chunks: one workgroup per chunk
        FF_HIP_TRY(launch_verify_chunks(t, L.chunk_bytes, static_cast<uint32_t>(L.tile_bytes),
                                        L.tiles_per_chunk, p->affine, buf, crcs, bad, n_bad,
                                        L.n_chunks, s));
        if (verify_only) return FF_OK;
        t.acc = nullptr;
        t.skip_bad = bad;
        FF_HIP_TRY(launch_tiles(kRestore, t, buf, s, nullptr));
        return FF_OK;
    }
    FF_HIP_TRY(launch_preset(bad, crcs, 0, L.n_chunks, p->affine, clear_n_bad ? n_bad : nullptr, list, s));
    if (verify_only || skip_bad) {
        // pass 1: read and fold only; over the whole buffer it runs on grouped tiles
        TileTables v = t;
        if (!list) {
            v.tile_rows *= p->verify_group;
            v.n_tiles /= p->verify_group;
            v.tiles_per_chunk /= p->verify_group;
            v.tpc_log2 = 0;
            while ((1u << v.tpc_log2) < v.tiles_per_chunk) v.tpc_log2++;
            v.shift_stride = p->verify_group;
        }
        FF_HIP_TRY(launch_tiles(kVerify, v, buf, s, list));
        FF_HIP_TRY(launch_finish_verify(bad, L.n_chunks, n_bad, list, s));
        if (verify_only) return FF_OK;
        // pass 2: scatter the tiles of the chunks that verified; nothing is folded
        t.acc = nullptr;
        t.skip_bad = bad;
        FF_HIP_TRY(launch_tiles(kRestore, t, buf, s, list));
        return FF_OK;
    }
    FF_HIP_TRY(launch_tiles(kRestore, t, buf, s, list));
    FF_HIP_TRY(launch_finish_verify(bad, L.n_chunks, n_bad, list, s));
    return FF_OK;
}

int check_restore_args(const ff_plan* p, const void* chunks, const uint32_t* crcs, uint32_t* bad,
                       uint64_t* n_bad, uint32_t flags)
{
    int rc = check_device_call(p);
    if (rc != FF_OK) return rc;
    if (!chunks || !crcs || !bad || !n_bad) return FF_ERR_NULL;
    if (flags & ~(FF_RESTORE_VERIFY_ONLY | FF_RESTORE_SKIP_BAD)) return FF_ERR_INVALID;
    if (reinterpret_cast<uint64_t>(chunks) % 16 || reinterpret_cast<uint64_t>(crcs) % 4 ||
        reinterpret_cast<uint64_t>(bad) % 4 || reinterpret_cast<uint64_t>(n_bad) % 8)
        return FF_ERR_INVALID;
    return FF_OK;
}

// prev: null for the in-place step; else the snapshot that holds the old master, m and v.
int adam_impl(const ff_plan* p, const void* const* grads, const ff_adam_hparams* hp,
              uint32_t half_dtype, float inv_scale, uint64_t* n_nonfinite, const void* prev,
              void* chunks, uint32_t* crcs, hipStream_t s, bool bare = false)
{
    int rc = check_device_call(p);
    if (rc != FF_OK) return rc;
    if (!grads || !hp || !chunks || (!crcs && !bare)) return FF_ERR_NULL;
    const Layout& L = p->layout;
    if (!L.adam_ok || L.params.empty() || hp->step == 0) return FF_ERR_INVALID;
    if (L.half_dtype != half_dtype) return FF_ERR_INVALID;  // bf16 plan <-> fp16 call or vice versa
    if (reinterpret_cast<uint64_t>(chunks) % 16 || reinterpret_cast<uint64_t>(crcs) % 4)
        return FF_ERR_INVALID;
    if (prev) {
        // the two snapshots must be different buffers: elements of `prev` are read while
        // neighbouring ones of `chunks` are already written
        const uint64_t a = reinterpret_cast<uint64_t>(prev), b = reinterpret_cast<uint64_t>(chunks);
        if (a % 16 || (a < b ? b - a : a - b) < L.buffer_bytes) return FF_ERR_INVALID;
    }
    for (size_t i = 0; i < L.params.size(); i++) {
        if (!grads[i]) return FF_ERR_NULL;
        if (reinterpret_cast<uint64_t>(grads[i]) % 2) return FF_ERR_INVALID;
    }
    FusedConsts c;
    {
        // shared scalars: evaluated in double from the fp32 hyper-parameters, rounded once
        const double lr = hp->lr, b1 = hp->beta1, b2 = hp->beta2, wd = hp->weight_decay;
        const double t = static_cast<double>(hp->step);
        c.adam.decay = static_cast<float>(1.0 - lr * wd);
        c.adam.b1 = hp->beta1;
        c.adam.omb1 = static_cast<float>(1.0 - b1);
        c.adam.b2 = hp->beta2;
        c.adam.omb2 = static_cast<float>(1.0 - b2);
        c.adam.step_size = static_cast<float>(lr / (1.0 - std::pow(b1, t)));
        c.adam.bc2s = static_cast<float>(std::sqrt(1.0 - std::pow(b2, t)));
        c.adam.eps = hp->eps;
    }
    c.inv_scale = inv_scale;
    c.xcd_group = bare ? p->mix_xcd_group : p->fused_xcd_group;
    c.n_nonfinite = n_nonfinite;
    c.prev = static_cast<const uint8_t*>(prev);
    FF_HIP_TRY(launch_fused(half_dtype == FF_F16, p->work, p->n_work_param,
                            p->n_work - p->n_work_param, grads,
                            static_cast<uint32_t>(L.params.size()), p->group_tile_begin.data(),
                            p->fused_tabs, chunks, crcs, L.n_chunks, L.payload, L.buffer_bytes,
                            p->affine, c, bare, s));
    return FF_OK;
}


}  // namespace

extern "C" {

int ff_pack_to_host(const ff_plan* p, void* chunks, uint32_t* crcs, void* host_chunks,
                    uint32_t* host_crcs, uint64_t slice_chunks, void* pack_stream,
                    void* copy_stream)
{
    int rc = check_device_call(p);
    if (rc != FF_OK) return rc;
    if (!chunks || !crcs || !host_chunks || !host_crcs) return FF_ERR_NULL;
    if (reinterpret_cast<uint64_t>(chunks) % 16 || reinterpret_cast<uint64_t>(crcs) % 4 ||
        slice_chunks == 0)
        return FF_ERR_INVALID;
    const Layout& L = p->layout;
    hipStream_t ps = static_cast<hipStream_t>(pack_stream);
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    const uint64_t n_slices = (L.n_chunks + slice_chunks - 1) / slice_chunks;
    uint8_t* d = static_cast<uint8_t*>(chunks);
    uint8_t* h = static_cast<uint8_t*>(host_chunks);
    for (uint64_t k = 0; k < n_slices; k++) {
        const uint64_t j0 = k * slice_chunks;
        const uint64_t nj = std::min(slice_chunks, L.n_chunks - j0);
        TileTables t = p->tables;
        t.acc = crcs;
        t.tile_begin = static_cast<uint32_t>(j0 * L.tiles_per_chunk);
        t.n_list = static_cast<uint32_t>(nj * L.tiles_per_chunk);
        FF_HIP_TRY(launch_preset(crcs, nullptr, j0, nj, p->affine, nullptr, nullptr, ps));
        FF_HIP_TRY(launch_tiles(kPack, t, chunks, ps));
        // the copy stream waits for this slice; the event belongs to this call alone and is
        // released as soon as the wait has been queued (the runtime keeps it until then)
        hipEvent_t done;
        FF_HIP_TRY(hipEventCreateWithFlags(&done, hipEventDisableTiming));
        hipError_t e = hipEventRecord(done, ps);
        if (e == hipSuccess) e = hipStreamWaitEvent(cs, done, 0);
        const hipError_t e2 = hipEventDestroy(done);
        FF_HIP_TRY(e);
        FF_HIP_TRY(e2);
        FF_HIP_TRY(hipMemcpyAsync(h + j0 * L.chunk_bytes, d + j0 * L.chunk_bytes,
                                  nj * L.chunk_bytes, hipMemcpyDeviceToHost, cs));
        FF_HIP_TRY(hipMemcpyAsync(host_crcs + j0, crcs + j0, nj * 4, hipMemcpyDeviceToHost, cs));
    }
    return FF_OK;
}

int ff_restore(const ff_plan* p, const void* chunks, const uint32_t* crcs, uint32_t* bad,
               uint64_t* n_bad, uint32_t flags, void* hip_stream)
{
    int rc = check_restore_args(p, chunks, crcs, bad, n_bad, flags);
    if (rc != FF_OK) return rc;
    return restore_impl(p, chunks, crcs, bad, n_bad, flags, nullptr, true,
                        static_cast<hipStream_t>(hip_stream));
}

int ff_restore_checked(const ff_plan* p, uint32_t sender_layout_id, const void* chunks,
                       const uint32_t* crcs, uint32_t* bad, uint64_t* n_bad, uint32_t flags,
                       void* hip_stream)
{
    int rc = check_restore_args(p, chunks, crcs, bad, n_bad, flags);
    if (rc != FF_OK) return rc;
    if (sender_layout_id != p->layout.layout_id) return FF_ERR_LAYOUT;  // nothing enqueued
    return restore_impl(p, chunks, crcs, bad, n_bad, flags, nullptr, true,
                        static_cast<hipStream_t>(hip_stream));
}

int ff_restore_chunks(const ff_plan* p, const void* chunks, const uint32_t* crcs,
                      const uint64_t* chunk_ids, uint64_t n_ids, uint32_t* bad, uint64_t* n_bad,
                      uint32_t flags, void* hip_stream)
{
    int rc = check_restore_args(p, chunks, crcs, bad, n_bad, flags);
    if (rc != FF_OK) return rc;
    if (n_ids && !chunk_ids) return FF_ERR_NULL;
    const Layout& L = p->layout;
    if (n_ids > L.n_chunks) return FF_ERR_INVALID;
    for (uint64_t k = 0; k < n_ids; k++) {
        if (chunk_ids[k] >= L.n_chunks) return FF_ERR_INVALID;
        if (k && chunk_ids[k] <= chunk_ids[k - 1]) return FF_ERR_INVALID;  // strictly ascending
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (n_ids == 0) {
        FF_HIP_TRY(launch_zero_u64(n_bad, s));
        return FF_OK;
    }
    // the ids go to the kernels inside their arguments, kMaxListedChunks at a time
    for (uint64_t k0 = 0; k0 < n_ids; k0 += kMaxListedChunks) {
        ChunkList list;
        list.n = static_cast<uint32_t>(std::min<uint64_t>(kMaxListedChunks, n_ids - k0));
        for (uint32_t k = 0; k < kMaxListedChunks; k++)
            list.id[k] = k < list.n ? static_cast<uint32_t>(chunk_ids[k0 + k]) : 0u;
        rc = restore_impl(p, chunks, crcs, bad, n_bad, flags, &list, k0 == 0, s);
        if (rc != FF_OK) return rc;
    }
    return FF_OK;
}

int ff_plan_chunk_span(const ff_plan* p, uint64_t chunk, uint64_t* first_seg, uint64_t* n_seg,
                       uint64_t* begin, uint64_t* end)
{
    if (!p || !first_seg || !n_seg || !begin || !end) return FF_ERR_NULL;
    const Layout& L = p->layout;
    if (chunk >= L.n_chunks) return FF_ERR_INVALID;
    const uint64_t lo = chunk * L.chunk_bytes;
    const uint64_t hi = std::min(lo + L.chunk_bytes, L.payload);
    // first segment whose end is beyond lo (segments are sorted by offset)
    size_t a = 0, b = L.segs.size();
    while (a < b) {
        const size_t mid = (a + b) / 2;
        if (L.segs[mid].off + L.segs[mid].nbytes <= lo) a = mid + 1; else b = mid;
    }
    size_t e = a;
    while (e < L.segs.size() && L.segs[e].off < hi) e++;
    *first_seg = a;
    *n_seg = e - a;
    *begin = lo;
    *end = hi;
    return FF_OK;
}

int ff_adam_step_snapshot(const ff_plan* p, const void* const* grads, const ff_adam_hparams* hp,
                          void* chunks, uint32_t* crcs, void* hip_stream)
{
    return adam_impl(p, grads, hp, FF_BF16, 1.0f, nullptr, nullptr, chunks, crcs,
                     static_cast<hipStream_t>(hip_stream));
}

int ff_adam_step_snapshot_f16(const ff_plan* p, const void* const* grads,
                              const ff_adam_hparams* hp, float inv_loss_scale,
                              uint64_t* n_nonfinite, void* chunks, uint32_t* crcs,
                              void* hip_stream)
{
    if (reinterpret_cast<uint64_t>(n_nonfinite) % 8) return FF_ERR_INVALID;
    return adam_impl(p, grads, hp, FF_F16, inv_loss_scale, n_nonfinite, nullptr, chunks, crcs,
                     static_cast<hipStream_t>(hip_stream));
}

int ff_adam_step_chained(const ff_plan* p, const void* const* grads, const ff_adam_hparams* hp,
                         float inv_loss_scale, uint64_t* n_nonfinite, const void* prev_chunks,
                         void* chunks, uint32_t* crcs, void* hip_stream)
{
    if (!p) return FF_ERR_NULL;
    if (!prev_chunks) return FF_ERR_NULL;
    const uint32_t half = p->layout.half_dtype;
    if (half != FF_F16 && (inv_loss_scale != 1.0f || n_nonfinite)) return FF_ERR_INVALID;
    if (reinterpret_cast<uint64_t>(n_nonfinite) % 8) return FF_ERR_INVALID;
    return adam_impl(p, grads, hp, half == FF_F16 ? FF_F16 : FF_BF16, inv_loss_scale, n_nonfinite,
                     prev_chunks, chunks, crcs, static_cast<hipStream_t>(hip_stream));
}

int ff_mix_ceiling(const ff_plan* p, const void* const* grads, const void* prev_chunks,
                   void* chunks, void* hip_stream)
{
    if (!p) return FF_ERR_NULL;
    const ff_adam_hparams hp = {0.f, 0.f, 0.f, 0.f, 0.f, 1u};  // unused by the bare pattern
    const uint32_t half = p->layout.half_dtype == FF_F16 ? FF_F16 : FF_BF16;
    return adam_impl(p, grads, &hp, half, 1.0f, nullptr, prev_chunks, chunks, nullptr,
                     static_cast<hipStream_t>(hip_stream), true);
}

int ff_crc32c(const void* dev_buf, uint64_t nbytes, uint32_t* dev_out, void* hip_stream)
{
    if (!dev_out || (nbytes && !dev_buf)) return FF_ERR_NULL;
    if (reinterpret_cast<uint64_t>(dev_buf) % 16 || reinterpret_cast<uint64_t>(dev_out) % 4)
        return FF_ERR_INVALID;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint64_t rows = nbytes / 1024;
    const uint32_t tile_rows = 1024;
    if ((rows + tile_rows - 1) / tile_rows > 0xFFFFFFF0ull) return FF_ERR_INVALID;
    TileTables t;
    t.total_rows = rows;
    t.tile_rows = tile_rows;
    t.n_tiles = static_cast<uint32_t>((rows + tile_rows - 1) / tile_rows);
    t.lead_rows = static_cast<uint32_t>(static_cast<uint64_t>(t.n_tiles) * tile_rows - rows);
    t.payload = rows * 1024;

    // scratch: byte tables + one register per tile
    const uint64_t scratch_bytes = kTabWords * 4 + (static_cast<uint64_t>(t.n_tiles) + 1) * 4;
    void* scratch = nullptr;
    hipError_t e = hipMalloc(&scratch, scratch_bytes);
    if (e == hipErrorOutOfMemory) return FF_ERR_NOMEM;
    FF_HIP_TRY(e);
    uint32_t tab[kTabWords];
    build_tab_u(tab);
    int rc = FF_OK;
    do {
        if ((e = hipMemcpyAsync(scratch, tab, sizeof(tab), hipMemcpyHostToDevice, s)) != hipSuccess) break;
        t.tab_u = static_cast<const uint32_t*>(scratch);
        t.partial = static_cast<uint32_t*>(scratch) + kTabWords;
        if ((e = launch_tiles(kVerify, t, const_cast<void*>(dev_buf), s)) != hipSuccess) break;
        const uint8_t* tail = static_cast<const uint8_t*>(dev_buf) + rows * 1024;
        e = launch_finish_crc(t.partial, t.n_tiles, gf2_xpow(8ull * 1024 * tile_rows), tail,
                              static_cast<uint32_t>(nbytes - rows * 1024), crc_affine_term(nbytes),
                              dev_out, s);
    } while (0);
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(scratch);
    if (e != hipSuccess) rc = hip_fail(e);
    else if (e2 != hipSuccess) rc = hip_fail(e2);
    return rc;
}

int ff_crc32c_noalloc(const void* dev_buf, uint64_t nbytes, uint32_t* dev_out, void* hip_stream)
{
    if (!dev_out || (nbytes && !dev_buf)) return FF_ERR_NULL;
    if (reinterpret_cast<uint64_t>(dev_buf) % 16 || reinterpret_cast<uint64_t>(dev_out) % 4)
        return FF_ERR_INVALID;
    if (nbytes > FF_CRC32C_NOALLOC_MAX_BYTES) return FF_ERR_TOO_LARGE;
    uint32_t* ptr = nullptr;
    const int rc = scratch_for_current_device(&ptr);
    if (rc != FF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint64_t rows = nbytes / 1024;
    TileTables t;
    t.total_rows = rows;
    t.tile_rows = kNoallocTileRows;
    t.n_tiles = static_cast<uint32_t>((rows + kNoallocTileRows - 1) / kNoallocTileRows);
    t.lead_rows = static_cast<uint32_t>(static_cast<uint64_t>(t.n_tiles) * kNoallocTileRows - rows);
    t.payload = rows * 1024;
    t.tab_u = ptr;
    // every tile of this call stores its register before the finishing kernel reads it, so what
    // an earlier (possibly longer) call left behind is never looked at and nothing needs clearing
    t.partial = ptr + kTabWords;
    FF_HIP_TRY(launch_tiles(kVerify, t, const_cast<void*>(dev_buf), s));
    const uint8_t* tail = static_cast<const uint8_t*>(dev_buf) + rows * 1024;
    FF_HIP_TRY(launch_finish_crc(t.partial, t.n_tiles, gf2_xpow(8ull * 1024 * kNoallocTileRows), tail,
                                 static_cast<uint32_t>(nbytes - rows * 1024),
                                 crc_affine_term(nbytes), dev_out, s));
    return FF_OK;
}

int ff_copy_ceiling(void* dst, const void* src, uint64_t nbytes, void* hip_stream)
{
    if (!dst || !src) return FF_ERR_NULL;
    if (reinterpret_cast<uint64_t>(dst) % 16 || reinterpret_cast<uint64_t>(src) % 16 || nbytes % 16)
        return FF_ERR_INVALID;
    FF_HIP_TRY(launch_copy(dst, src, nbytes, static_cast<hipStream_t>(hip_stream)));
    return FF_OK;
}

const char* ff_strerror(int status)
{
    static thread_local char buf[320];
    switch (status) {
    case FF_OK: return "ok";
    case FF_ERR_NULL: return "a required pointer is NULL";
    case FF_ERR_INVALID: return "invalid argument";
    case FF_ERR_EMPTY: return "the segments hold no bytes";
    case FF_ERR_NOMEM: return "out of memory";
    case FF_ERR_HOST_ONLY: return "device work asked of a host-only plan";
    case FF_ERR_TOO_LARGE: return "input larger than the fixed scratch array allows";
    case FF_ERR_LAYOUT: return "the sender's layout id differs from the plan's";
    case FF_ERR_HIP:
        std::snprintf(buf, sizeof(buf), "HIP error: %s", g_hip_error);
        return buf;
    default: return "unknown status";
    }
}

}  // extern "C"
