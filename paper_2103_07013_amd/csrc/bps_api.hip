// Host side of the C ABI declared in include/bps.h: renderer object, scene table, request
// staging and launch planning.  All rendering arithmetic is in raster_kernels.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/bps.h"
#include "clusters.h"
#include "raster_kernels.h"

namespace {

constexpr int kMaxScenes = 4096;
constexpr int kRing = 4;          // request staging slots in flight
constexpr int kXcds = 8;          // work-groups are dealt round-robin to 8 accelerator dies
constexpr size_t kMaxProfiled = 4096;   // profiled requests remembered between two reads of the totals

thread_local std::string g_create_error = "";

// ---- scratch of bps_render_static, the entry point that allocates nothing ------------------------
// Work items as staged, work items in launch order, and one cost word per item.
constexpr uint32_t kStaticMaxItems = bps::kMaxPlannedItems;
constexpr size_t kStaticScratchBytes = (size_t)kStaticMaxItems * (2 * sizeof(bps::WorkItem) + sizeof(uint32_t));
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// In host code the array's name is only a stand-in: its address on each device is looked up once
// (bps_create, with that device current) and used from then on.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
// what the array on each device holds: the renderer and plan whose work items were unpacked last
const void* g_scratch_owner[kMaxDevices] = {};
uint64_t g_scratch_plan[kMaxDevices] = {};

// Device memory of one scene: a single allocation holding every array, so that loading is one
// asynchronous copy and retiring a scene can hand the block to the next load.
struct Arena {
    void* ptr = nullptr;
    size_t bytes = 0;
};

struct HostScene {
    bool live = false;
    bps::SceneDev dev{};
    Arena arena;
    uint64_t bytes = 0;
    bool has_colors = false;
    hipEvent_t ready = nullptr;   // copy finished (asynchronous loads); null once known complete
    uint64_t last_use = 0;        // sequence number of the last request that referenced the scene
};

struct Retired {      // device block or table slot that queued requests may still read
    Arena arena;
    int slot = -1;
    uint64_t last_use = 0;
    hipEvent_t upload = nullptr;   // the scene's own upload, if it was still in flight when the scene was retired
};

struct Staging {      // pinned host image of a scene being copied
    void* ptr = nullptr;
    size_t bytes = 0;
    hipEvent_t done = nullptr;
};

struct RingSlot {
    unsigned char* host = nullptr;   // pinned
    unsigned char* dev = nullptr;
    size_t capacity = 0;
    hipEvent_t done = nullptr;
    hipEvent_t planned = nullptr;    // launch plan ready (only used when planning runs on the renderer's own stream)
    bool pending = false;
    uint64_t seq = 0;
    uint64_t items_version = 0;      // plan whose work items the device buffer holds (0 = none)
};

}  // namespace

struct bps_renderer {
    bps_config cfg{};
    int device = 0;
    int num_cu = 0;
    int threads = 512;
    int ss = 1, rw = 64, rh = 64;     // supersampling factor and rendered frame size
    float* ss_depth = nullptr;        // [max_batch][rh][rw] when supersampling
    uint8_t* ss_rgb = nullptr;
    int tile_w = 64, tile_h = 64, tiles = 1;
    int list_cap = 2048;
    int round_target = 2048, first_round = 192;
    size_t lds = 0;
    size_t max_lds = 0;
    std::string error = "";
    std::mutex err_mu;                // guards `error` alone (failures are also reported from outside `mu`)
    std::vector<HostScene> scenes;
    std::vector<uint32_t> gens;       // generation of every table slot: part of the handle, so that a stale handle is refused
    std::vector<Retired> retired;     // waiting for the requests that used them
    std::vector<Arena> arena_pool;    // free device blocks, reused by later loads
    std::vector<Staging> staging;     // pinned images, reused once their copy has finished
    hipStream_t load_stream = nullptr;   // used by the synchronous bps_load_scene
    hipStream_t plan_stream = nullptr;   // staging + launch planning of requests whose inputs are complete at the call
    uint64_t seq = 0, done_seq = 0;   // requests issued / known complete
    uint64_t arena_allocs = 0;        // device blocks allocated so far (reuse keeps this flat)
    std::mutex mu;                    // guards all state: one loader thread may run beside the render thread
    bps::SceneDev* d_scenes = nullptr;
    RingSlot ring[kRing];
    int ring_next = 0;
    unsigned long long* gvis = nullptr;   // [max_batch][H][W], only for split frames
    uint32_t* ids = nullptr;              // [max_batch][H][W], RGB-D requests without a caller id buffer
    uint32_t* shade_queue = nullptr;      // queues of the pixels whose winner needs the clipper, then two counter blocks
    uint32_t shade_parity = 0;            // which of the two counters the next RGB-D request uses
    unsigned long long* d_stats = nullptr;   // diagnostics block: 8 counters + one duration per work-group
    size_t stats_cap = 0;
    bool want_stats = false;
    int stats_mode = 0;                   // 0 counters + timeline, 1 phase timers, 2 / 3 path tallies
    std::vector<hipEvent_t> ev;           // profiling: pairs (start, stop), one pair per request
    size_t ev_used = 0;
    bool profiling = false;
    uint32_t profile_every = 1, profile_count = 0;   // every n-th request is timed
    // cached plan: valid while the scene ids and split count repeat
    std::vector<bps_scene> plan_ids;
    int plan_splits = 0;
    uint64_t plan_version = 0;        // counts the plans made; ring slots remember which one they hold
    std::vector<bps::WorkItem> plan_items;
    std::vector<bps_scene> call_slots;    // table slots of the current request's scene handles (keeps its capacity)
    uint64_t last_splits = 0, last_groups = 0;
    unsigned char* static_scratch = nullptr;   // this device's copy of the static scratch array (bps_render_static)
    // last request that used a buffer every request shares (ids, gvis, ss_*, d_stats): a later one on
    // another stream waits for it
    hipEvent_t shared_done = nullptr;
    hipStream_t shared_stream = nullptr;
};

namespace {

bps_status fail(bps_renderer* r, bps_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (r) {
        std::lock_guard<std::mutex> g(r->err_mu);
        r->error = buf;
    } else {
        g_create_error = buf;
    }
    return code;
}

#define BPS_HIP(r, call)                                                                      \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail((r), e_ == hipErrorOutOfMemory ? BPS_ERR_OOM : BPS_ERR_HIP, "%s: %s", \
                        #call, hipGetErrorString(e_));                                        \
    } while (0)

// A scene handle is its table slot (low 12 bits) and the slot's generation at load time above it.
constexpr int kSlotBits = 12;
static_assert((1 << kSlotBits) == kMaxScenes, "a handle holds the table slot in its low bits");
bps_scene make_handle(const bps_renderer* r, int slot) { return (bps_scene)((uint32_t)slot | (r->gens[slot] << kSlotBits)); }
// Table slot of a live handle, -1 for anything else (never loaded, retired, or retired and the slot reused).
int slot_of(const bps_renderer* r, bps_scene h) {
    if (h < 0) return -1;
    const size_t slot = (uint32_t)h & (uint32_t)(kMaxScenes - 1);
    if (slot >= r->scenes.size() || !r->scenes[slot].live || r->gens[slot] != ((uint32_t)h >> kSlotBits)) return -1;
    return (int)slot;
}

void free_scene(HostScene& s) {
    if (s.arena.ptr) (void)hipFree(s.arena.ptr);
    if (s.ready) (void)hipEventDestroy(s.ready);
    s = HostScene{};
}

// Learn which requests have finished (never blocks) and recycle what they were holding.
// Requests on different streams can finish out of order: everything up to the oldest request still
// pending is complete (every request in flight holds a ring slot).
void note_completions(bps_renderer* r) {
    uint64_t all_done = r->seq;
    for (const RingSlot& s : r->ring)
        if (s.pending) all_done = std::min(all_done, s.seq - 1);
    r->done_seq = std::max(r->done_seq, all_done);
}

void collect(bps_renderer* r) {
    for (RingSlot& s : r->ring)
        if (s.pending && hipEventQuery(s.done) == hipSuccess) s.pending = false;
    (void)hipGetLastError();
    note_completions(r);
    for (size_t i = 0; i < r->retired.size();) {
        Retired& x = r->retired[i];
        if (x.upload && hipEventQuery(x.upload) == hipSuccess) {
            (void)hipEventDestroy(x.upload);
            x.upload = nullptr;
        }
        (void)hipGetLastError();
        if (x.last_use <= r->done_seq && !x.upload) {
            if (r->retired[i].arena.ptr) r->arena_pool.push_back(r->retired[i].arena);
            r->retired[i] = r->retired.back();
            r->retired.pop_back();
        } else {
            ++i;
        }
    }
}

bool slot_busy(const bps_renderer* r, int slot) {
    for (const Retired& x : r->retired)
        if (x.slot == slot) return true;
    return false;
}

bool fp_cull_enabled(const bps_renderer* r) { return !(r->cfg.flags & BPS_FLAG_NO_CLUSTER_CULL); }

// Choose how many work-groups share one environment: enough groups to fill the device a few
// times over when the batch is small, one group per environment when the batch is large.
int plan_splits(const bps_renderer* r, uint32_t B, uint32_t min_clusters) {
    if (r->cfg.splits > 0) return r->cfg.splits;
    int waves = r->threads / 64;
    int want_groups = 4 * r->num_cu;
    int s = 1;
    int groups = (int)B * r->tiles;
    if (groups < 2 * r->num_cu) s = (want_groups + groups - 1) / groups;
    int max_s = std::max(1, (int)(min_clusters / (uint32_t)(8 * waves)));   // >= 8 clusters per wave
    return std::max(1, std::min(s, max_s));
}

// The launch plan: one work item per (environment, tile, slice of its scene's clusters);
// environments of one scene are kept on one accelerator die so its L2 serves every re-read of that
// scene.  Cached while the scene ids and the split count repeat.
void make_plan(bps_renderer* r, const bps_scene* scene_ids, uint32_t B, int S) {
    bool replan = r->plan_splits != S || r->plan_ids.size() != B || std::memcmp(r->plan_ids.data(), scene_ids, B * sizeof(bps_scene)) != 0;
    if (replan) {
        std::vector<uint32_t> order(B);
        for (uint32_t b = 0; b < B; ++b) order[b] = b;
        std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return scene_ids[a] < scene_ids[b]; });
        std::vector<bps::WorkItem> sorted;
        sorted.reserve((size_t)B * S * r->tiles);
        for (uint32_t k = 0; k < B; ++k) {
            uint32_t b = order[k];
            uint32_t C = r->scenes[scene_ids[b]].dev.n_clusters;
            (void)C;
            for (int tile = 0; tile < r->tiles; ++tile)
                for (int s = 0; s < S; ++s) {
                    bps::WorkItem it;
                    it.env = b;
                    it.scene = (uint32_t)scene_ids[b];
                    it.split_of = ((uint32_t)S << 16) | (uint32_t)s;
                    it.tile = (uint32_t)tile;
                    sorted.push_back(it);
                }
        }
        const size_t n = sorted.size();
        r->plan_items.resize(n);
        // block i runs on die i % 8: give die x the x-th contiguous chunk of the sorted list
        size_t start = 0;
        for (int x = 0; x < kXcds; ++x) {
            size_t cnt = n / kXcds + ((size_t)x < n % kXcds ? 1 : 0);
            for (size_t k = 0; k < cnt; ++k) r->plan_items[x + k * kXcds] = sorted[start + k];
            start += cnt;
        }
        r->plan_ids.assign(scene_ids, scene_ids + B);
        r->plan_splits = S;
        ++r->plan_version;
    }
}

bps::FrameParams frame_params(const bps_renderer* r, int S) {
    bps::FrameParams fp;
    fp.H = r->rh;
    fp.W = r->rw;
    fp.tile_w = r->tile_w;
    fp.tile_h = r->tile_h;
    fp.sx = 128.0f * (float)fp.W;
    fp.sy = 128.0f * (float)fp.H;
    fp.xmax = 2.0f * fp.sx + 64.0f;
    fp.ymax = 2.0f * fp.sy + 64.0f;
    fp.background = r->cfg.background_depth;
    fp.merge = S > 1 ? 1 : 0;
    fp.cull = (r->cfg.flags & BPS_FLAG_NO_CLUSTER_CULL) ? 0 : (r->cfg.flags & BPS_FLAG_NO_OCCLUSION_CULL) ? 1 : 2;
    fp.list_cap = r->list_cap;
    fp.round_target = r->round_target;
    fp.first_round = r->first_round;
    fp.phase_timers = r->want_stats ? r->stats_mode : 0;
    fp.bilinear = (r->cfg.flags & BPS_FLAG_BILINEAR) ? 1 : 0;
    return fp;
}

}  // namespace

extern "C" {

const char* bps_last_error(const bps_renderer* r) {
    if (!r) return g_create_error.c_str();
    // a copy per calling thread: another thread's failure cannot change the text while the caller reads it
    thread_local std::string text;
    std::lock_guard<std::mutex> g(const_cast<bps_renderer*>(r)->err_mu);
    text = r->error;
    return text.c_str();
}

bps_status bps_create(const bps_config* cfg, bps_renderer** out) {
    if (!cfg || !out) return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: null argument");
    *out = nullptr;
    if (cfg->max_batch < 1) return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: max_batch must be >= 1");
    if (cfg->supersample != 0 && cfg->supersample != 1 && cfg->supersample != 2)
        return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: supersample must be 0, 1 or 2");
    const int ss = cfg->supersample == 2 ? 2 : 1;
    if (cfg->height < 8 || cfg->height * ss > 128 || cfg->height % 8 || cfg->width < 8 || cfg->width * ss > 128 || cfg->width % 8)
        return fail(nullptr, BPS_ERR_INVALID_ARG,
                    "bps_create: height and width must be multiples of 8, at least 8 and at most 128 after supersampling");
    if (cfg->mode != BPS_MODE_DEPTH && cfg->mode != BPS_MODE_RGBD)
        return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: unknown mode %d", cfg->mode);
    if (cfg->threads != 0 && cfg->threads != 256 && cfg->threads != 384 && cfg->threads != 512 && cfg->threads != 1024)
        return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: threads must be 0, 256, 384, 512 or 1024");
    if (cfg->splits < 0 || cfg->splits > 0xFFFF) return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: splits must be 0..65535");
    if (cfg->flags & ~(uint32_t)(BPS_FLAG_NO_CLUSTER_CULL | BPS_FLAG_NO_OCCLUSION_CULL | BPS_FLAG_NO_DISPATCH_ORDER | BPS_FLAG_INPUTS_READY | BPS_FLAG_BILINEAR)) return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: unknown flag bits 0x%x", cfg->flags);
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0)
        return fail(nullptr, BPS_ERR_HIP, "bps_create: no HIP device available (this library has no CPU path)");
    if (cfg->device < 0 || cfg->device >= ndev)
        return fail(nullptr, BPS_ERR_INVALID_ARG, "bps_create: device %d out of range (0..%d)", cfg->device, ndev - 1);

    bps_renderer* r = new (std::nothrow) bps_renderer();
    if (!r) return fail(nullptr, BPS_ERR_OOM, "bps_create: out of host memory");
    r->cfg = *cfg;
    r->device = cfg->device;
    bps_status st = BPS_OK;
    auto bail = [&](bps_status code) {
        g_create_error = r->error;
        bps_destroy(r);
        return code;
    };
    auto step = [&]() -> bps_status {
        BPS_HIP(r, hipSetDevice(r->device));
        hipDeviceProp_t prop;
        BPS_HIP(r, hipGetDeviceProperties(&prop, r->device));
        r->num_cu = prop.multiProcessorCount;
        int lds_optin = 0;
        if (hipDeviceGetAttribute(&lds_optin, hipDeviceAttributeSharedMemPerBlockOptin, r->device) != hipSuccess) lds_optin = 0;
        (void)hipGetLastError();
        r->max_lds = std::max<size_t>(prop.sharedMemPerBlock, (size_t)std::max(lds_optin, 0));
        // a work-group owns one tile of the frame: the whole frame up to 64 pixels per side,
        // otherwise the frame is cut into equal tiles of at most 64 pixels
        auto tile_of = [](int n) { int parts = (n + 63) / 64; return (n + parts - 1) / parts; };
        r->ss = ss;
        r->rw = cfg->width * ss;      // rendered size; the output is rw / ss by rh / ss
        r->rh = cfg->height * ss;
        r->tile_w = tile_of(r->rw);
        r->tile_h = tile_of(r->rh);
#ifdef BPS_TUNING_KNOBS      // experiments only: not compiled into the library that ships
        if (const char* e = std::getenv("BPS_TILE")) {   // force a tile size
            int v = std::atoi(e);
            if (v >= 8 && v <= 64) { r->tile_w = std::min(v, r->rw); r->tile_h = std::min(v, r->rh); }
        }
#endif
        r->tiles = ((r->rw + r->tile_w - 1) / r->tile_w) * ((r->rh + r->tile_h - 1) / r->tile_h);
        // the raster kernel's depth tiles and footprint records are laid out for windows of at most 64x64 pixels
        if (r->tile_w > 64 || r->tile_h > 64 || ((r->tile_w + 7) / 8) * ((r->tile_h + 7) / 8) > bps::kHizTiles)
            return fail(r, BPS_ERR_UNSUPPORTED, "bps_create: window %dx%d exceeds what the raster kernel is laid out for", r->tile_w, r->tile_h);
        // preferred work-group size whose LDS footprint leaves room for a useful survivor list
        const int order[4] = {512, 384, 256, 1024};
        r->threads = 0;
        auto fit_cap = [&](int t) -> int {
            size_t fixed = bps::lds_bytes(r->tile_h, r->tile_w, t, 0);
            if (fixed >= r->max_lds) return 0;
            // two work-groups per compute unit when the frame allows it
            size_t budget = fixed * 2 + 2 * 12 * 512 <= r->max_lds ? r->max_lds / 2 : r->max_lds;
            size_t cap = std::min<size_t>(2048, (budget - fixed) / 12);
            return (int)(cap & ~(size_t)63);
        };
        if (cfg->threads) {
            if (fit_cap(cfg->threads) >= 128) r->threads = cfg->threads;
        } else {
            for (int t : order)
                if (fit_cap(t) >= 512) { r->threads = t; break; }
        }
        if (!r->threads)
            return fail(r, BPS_ERR_UNSUPPORTED, "bps_create: a %dx%d frame needs %zu bytes of LDS, device offers %zu",
                        r->rh, r->rw, bps::lds_bytes(r->tile_h, r->tile_w, cfg->threads ? cfg->threads : 256, 512),
                        r->max_lds);
        r->list_cap = fit_cap(r->threads);
        r->round_target = r->list_cap;
#ifdef BPS_TUNING_KNOBS
        if (const char* e = std::getenv("BPS_ROUND_TARGET")) r->round_target = std::max(1, std::atoi(e));
        if (const char* e = std::getenv("BPS_FIRST_ROUND")) r->first_round = std::max(1, std::atoi(e));
#endif
        r->lds = bps::lds_bytes(r->tile_h, r->tile_w, r->threads, r->list_cap);
        BPS_HIP(r, bps::prepare_raster(r->threads, r->lds));
        BPS_HIP(r, hipMalloc((void**)&r->d_scenes, sizeof(bps::SceneDev) * kMaxScenes));
        BPS_HIP(r, hipMemset(r->d_scenes, 0, sizeof(bps::SceneDev) * kMaxScenes));
        for (RingSlot& s : r->ring) {
            BPS_HIP(r, hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
            BPS_HIP(r, hipEventCreateWithFlags(&s.planned, hipEventDisableTiming));
        }
        BPS_HIP(r, hipStreamCreateWithFlags(&r->load_stream, hipStreamNonBlocking));
        {   // address of the static scratch array on this device (every device holds its own copy)
            std::lock_guard<std::mutex> g(g_scratch_mu);
            if (r->device < kMaxDevices) {
                if (!g_scratch_ptr[r->device]) {
                    void* ptr = nullptr;
                    BPS_HIP(r, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
                    g_scratch_ptr[r->device] = ptr;
                }
                r->static_scratch = (unsigned char*)g_scratch_ptr[r->device];
            }
        }
        return BPS_OK;
    };
    st = step();
    if (st != BPS_OK) return bail(st);
    *out = r;
    return BPS_OK;
}

void bps_destroy(bps_renderer* r) {
    if (!r) return;
    (void)hipSetDevice(r->device);
    (void)hipDeviceSynchronize();
    for (HostScene& s : r->scenes) free_scene(s);
    for (Retired& x : r->retired) {
        if (x.arena.ptr) (void)hipFree(x.arena.ptr);
        if (x.upload) (void)hipEventDestroy(x.upload);
    }
    for (Arena& x : r->arena_pool) (void)hipFree(x.ptr);
    for (Staging& x : r->staging) {
        (void)hipHostFree(x.ptr);
        (void)hipEventDestroy(x.done);
    }
    if (r->load_stream) (void)hipStreamDestroy(r->load_stream);
    if (r->plan_stream) (void)hipStreamDestroy(r->plan_stream);
    for (RingSlot& s : r->ring) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.dev) (void)hipFree(s.dev);
        if (s.done) (void)hipEventDestroy(s.done);
        if (s.planned) (void)hipEventDestroy(s.planned);
    }
    if (r->gvis) (void)hipFree(r->gvis);
    if (r->ids) (void)hipFree(r->ids);
    if (r->shade_queue) (void)hipFree(r->shade_queue);
    if (r->ss_depth) (void)hipFree(r->ss_depth);
    if (r->ss_rgb) (void)hipFree(r->ss_rgb);
    if (r->d_stats) (void)hipFree(r->d_stats);
    if (r->d_scenes) (void)hipFree(r->d_scenes);
    for (hipEvent_t e : r->ev) (void)hipEventDestroy(e);
    delete r;
}

namespace {

struct TextureArg {
    const float* uvs = nullptr;        // [V][2]
    const uint8_t* texels = nullptr;   // [h][w][3]
    uint32_t w = 0, h = 0;
};

// Shared by the synchronous and asynchronous entry points: validate, cluster, lay every array out
// in one pinned image, copy it into one device block on `stream`, update the scene table on the
// same stream and record the scene's ready event.
bps_status load_scene_on(bps_renderer* r, const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T,
                         const uint8_t* colors, const TextureArg& tex, hipStream_t stream, bps_scene* out_handle) {
    if (!vertices || !indices || !out_handle) return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: null argument");
    const bool textured = tex.uvs != nullptr || tex.texels != nullptr;
    if (textured) {
        if (!tex.uvs || !tex.texels) return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: uvs and texels go together");
        if (tex.w == 0 || tex.h == 0 || tex.w > 4096 || tex.h > 4096 || (tex.w & (tex.w - 1)) || (tex.h & (tex.h - 1)))
            return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: texture sides must be powers of two up to 4096 (got %ux%u)", tex.w, tex.h);
    }
    if (V == 0 || T == 0) return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: empty mesh (V=%u, T=%u)", V, T);
    for (size_t i = 0; i < 3 * (size_t)T; ++i)
        if (indices[i] >= V)
            return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: index %u of triangle %zu is >= V=%u", indices[i], i / 3, V);
    for (size_t i = 0; i < 3 * (size_t)V; ++i)
        if (!std::isfinite(vertices[i]))
            return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: vertex %zu has a non-finite coordinate", i / 3);
    BPS_HIP(r, hipSetDevice(r->device));
    // the long host-side steps (clustering, filling the pinned image) run without the lock
    bps::ClusterSet cs;
    try {
        cs = bps::build_clusters(vertices, V, indices, T);
    } catch (const std::bad_alloc&) {
        return fail(r, BPS_ERR_OOM, "bps_load_scene: out of host memory while clustering");
    }
    // (the raster kernel's survivor records keep 23 bits for the cluster)
    if (cs.count == 0 || cs.count >= (1u << 23)) return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene: unsupported cluster count %u", cs.count);

    // ---- layout of the block (every array 256-byte aligned), scene-table record last
    const uint32_t c_stride = (cs.count + 63u) & ~63u, nblocks = c_stride / 64u;
    size_t off = 0;
    auto place = [&](size_t bytes) { size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
    const size_t o_cverts = place(cs.verts.size() * 4), o_ctris = place(cs.tris.size() * 4), o_ids = place(cs.tri_id.size() * 4);
    const size_t o_verts = place((size_t)V * 12), o_idx = place((size_t)T * 12), o_col = colors ? place((size_t)V * 3) : 0;
    const size_t o_cb = place((size_t)6 * c_stride * 4), o_bb = place((size_t)6 * nblocks * 4);
    // texture: uv per vertex, then every mip level as RGBA8 texels, level after level
    size_t pyramid_texels = 0;
    uint32_t tex_levels = 0;
    if (textured)
        for (uint32_t a_ = tex.w, b_ = tex.h;; a_ = a_ > 1 ? a_ / 2 : 1, b_ = b_ > 1 ? b_ / 2 : 1) {
            pyramid_texels += (size_t)a_ * b_;
            ++tex_levels;
            if (a_ == 1 && b_ == 1) break;
        }
    const size_t o_uv = textured ? place((size_t)V * 8) : 0, o_tex = textured ? place(pyramid_texels * 4) : 0;
    const size_t copy_bytes = off;      // what the pinned image holds and the upload copies
    // per-triangle shading records (64 B each), built on the device from the uploaded arrays
    const bool shaded = colors != nullptr || textured;
    const size_t o_trirec = shaded ? place((size_t)T * 64) : 0;
    const size_t dev_bytes = off;
    off = copy_bytes;
    const size_t o_rec = place(sizeof(bps::SceneDev));
    const size_t img_bytes = off;

    // ---- pinned image: reuse one whose copy has finished, else allocate
    Staging stg;
    std::unique_lock<std::mutex> lock(r->mu);
    for (size_t i = 0; i < r->staging.size(); ++i)
        if (r->staging[i].bytes >= img_bytes && hipEventQuery(r->staging[i].done) == hipSuccess) {
            stg = r->staging[i];
            r->staging[i] = r->staging.back();
            r->staging.pop_back();
            break;
        }
    (void)hipGetLastError();
    lock.unlock();
    if (!stg.ptr) {
        BPS_HIP(r, hipHostMalloc(&stg.ptr, img_bytes, hipHostMallocDefault));
        stg.bytes = img_bytes;
        hipError_t e = hipEventCreateWithFlags(&stg.done, hipEventDisableTiming);
        if (e != hipSuccess) { (void)hipHostFree(stg.ptr); return fail(r, BPS_ERR_HIP, "bps_load_scene: %s", hipGetErrorString(e)); }
    }
    unsigned char* img = (unsigned char*)stg.ptr;
    std::memcpy(img + o_cverts, cs.verts.data(), cs.verts.size() * 4);
    std::memcpy(img + o_ctris, cs.tris.data(), cs.tris.size() * 4);
    std::memcpy(img + o_ids, cs.tri_id.data(), cs.tri_id.size() * 4);
    std::memcpy(img + o_verts, vertices, (size_t)V * 12);
    std::memcpy(img + o_idx, indices, (size_t)T * 12);
    if (colors) std::memcpy(img + o_col, colors, (size_t)V * 3);
    if (textured) {
        std::memcpy(img + o_uv, tex.uvs, (size_t)V * 8);
        // mip pyramid: every level halves both sides (not below 1); a texel is (a + b + c + d + 2) >> 2
        // of its 2x2 parents, parents clamped at the border
        uint8_t* lvl = img + o_tex;
        uint32_t pw = tex.w, ph = tex.h;
        for (size_t i = 0; i < (size_t)pw * ph; ++i) {
            lvl[4 * i + 0] = tex.texels[3 * i + 0];
            lvl[4 * i + 1] = tex.texels[3 * i + 1];
            lvl[4 * i + 2] = tex.texels[3 * i + 2];
            lvl[4 * i + 3] = 255;
        }
        for (uint32_t l = 1; l < tex_levels; ++l) {
            const uint8_t* prev = lvl;
            lvl += (size_t)pw * ph * 4;
            const uint32_t lw = pw > 1 ? pw / 2 : 1, lh = ph > 1 ? ph / 2 : 1;
            for (uint32_t y = 0; y < lh; ++y)
                for (uint32_t x = 0; x < lw; ++x) {
                    const uint32_t x0 = std::min(2 * x, pw - 1), x1 = std::min(2 * x + 1, pw - 1);
                    const uint32_t y0 = std::min(2 * y, ph - 1), y1 = std::min(2 * y + 1, ph - 1);
                    for (int ch = 0; ch < 4; ++ch) {
                        uint32_t sum = prev[4 * ((size_t)y0 * pw + x0) + ch] + prev[4 * ((size_t)y0 * pw + x1) + ch] +
                                       prev[4 * ((size_t)y1 * pw + x0) + ch] + prev[4 * ((size_t)y1 * pw + x1) + ch];
                        lvl[4 * ((size_t)y * lw + x) + ch] = (uint8_t)((sum + 2) >> 2);
                    }
                }
            pw = lw;
            ph = lh;
        }
    }
    {   // bounds as six planes so that 64 lanes read 64 consecutive clusters (or blocks of 64 clusters)
        float* cb = (float*)(img + o_cb);
        float* bb = (float*)(img + o_bb);
        std::memset(cb, 0, (size_t)6 * c_stride * 4);
        for (uint32_t c = 0; c < cs.count; ++c)
            for (int k = 0; k < 6; ++k) cb[(size_t)k * c_stride + c] = cs.bounds[(size_t)c * 6 + k];
        for (uint32_t b = 0; b < nblocks; ++b)
            for (int k = 0; k < 6; ++k) {
                float v = cs.bounds[(size_t)b * 64 * 6 + k];
                for (uint32_t c = b * 64; c < std::min(cs.count, b * 64 + 64); ++c)
                    v = k < 3 ? std::min(v, cs.bounds[(size_t)c * 6 + k]) : std::max(v, cs.bounds[(size_t)c * 6 + k]);
                bb[(size_t)k * nblocks + b] = v;
            }
    }

    // ---- table slot and device block (smallest free one that fits, else a new allocation)
    lock.lock();
    collect(r);
    int slot = -1;
    for (size_t i = 0; i < r->scenes.size(); ++i)
        if (!r->scenes[i].live && !slot_busy(r, (int)i)) { slot = (int)i; break; }
    if (slot < 0) {
        if ((int)r->scenes.size() >= kMaxScenes) {
            r->staging.push_back(stg);
            (void)hipEventRecord(stg.done, stream);
            return fail(r, BPS_ERR_OOM, "bps_load_scene: scene table full (%d)", kMaxScenes);
        }
        slot = (int)r->scenes.size();
        r->scenes.emplace_back();
        r->gens.push_back(0u);
    }
    Arena arena;
    int best = -1;
    for (size_t i = 0; i < r->arena_pool.size(); ++i)
        if (r->arena_pool[i].bytes >= dev_bytes && (best < 0 || r->arena_pool[i].bytes < r->arena_pool[best].bytes)) best = (int)i;
    if (best >= 0) {
        arena = r->arena_pool[best];
        r->arena_pool[best] = r->arena_pool.back();
        r->arena_pool.pop_back();
    } else {
        hipError_t e = hipMalloc(&arena.ptr, dev_bytes);
        if (e != hipSuccess) {
            r->staging.push_back(stg);
            (void)hipEventRecord(stg.done, stream);
            return fail(r, e == hipErrorOutOfMemory ? BPS_ERR_OOM : BPS_ERR_HIP, "bps_load_scene: hipMalloc(%zu): %s", dev_bytes,
                        hipGetErrorString(e));
        }
        arena.bytes = dev_bytes;
        ++r->arena_allocs;
    }
    unsigned char* d = (unsigned char*)arena.ptr;
    HostScene hs;
    hs.arena = arena;
    hs.bytes = dev_bytes;
    hs.has_colors = colors != nullptr || textured;
    hs.dev.cverts = (const float*)(d + o_cverts);
    hs.dev.ctris = (const uint32_t*)(d + o_ctris);
    hs.dev.ctri_id = (const uint32_t*)(d + o_ids);
    hs.dev.verts = (const float*)(d + o_verts);
    hs.dev.indices = (const uint32_t*)(d + o_idx);
    hs.dev.colors = colors ? (const uint8_t*)(d + o_col) : nullptr;
    hs.dev.uvs = textured ? (const float*)(d + o_uv) : nullptr;
    hs.dev.texels = textured ? (const uint32_t*)(d + o_tex) : nullptr;
    hs.dev.tex_w = textured ? tex.w : 0;
    hs.dev.tex_h = textured ? tex.h : 0;
    hs.dev.tex_levels = tex_levels;
    hs.dev.tri_rec = shaded ? (const float*)(d + o_trirec) : nullptr;
    hs.dev.cbounds = (const float*)(d + o_cb);
    hs.dev.bbounds = (const float*)(d + o_bb);
    hs.dev.n_clusters = cs.count;
    hs.dev.n_tris = T;
    hs.dev.n_verts = V;
    hs.dev.c_stride = c_stride;
    hs.dev.b_stride = nblocks;
    std::memcpy(img + o_rec, &hs.dev, sizeof(bps::SceneDev));

    auto undo = [&](hipError_t e, const char* what) {
        r->arena_pool.push_back(arena);
        r->staging.push_back(stg);
        (void)hipEventRecord(stg.done, stream);
        return fail(r, BPS_ERR_HIP, "bps_load_scene: %s: %s", what, hipGetErrorString(e));
    };
    hipError_t e = hipMemcpyAsync(d, img, copy_bytes, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return undo(e, "mesh copy");
    if (shaded) {
        bps::launch_build_shade_records(stream, hs.dev, (float*)(d + o_trirec));
        e = hipGetLastError();
        if (e != hipSuccess) return undo(e, "shading records");
    }
    e = hipMemcpyAsync(r->d_scenes + slot, img + o_rec, sizeof(bps::SceneDev), hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return undo(e, "scene table update");
    e = hipEventCreateWithFlags(&hs.ready, hipEventDisableTiming);
    if (e != hipSuccess) return undo(e, "event");
    (void)hipEventRecord(hs.ready, stream);
    (void)hipEventRecord(stg.done, stream);
    r->staging.push_back(stg);
    hs.live = true;
    r->scenes[slot] = hs;
    r->plan_ids.clear();
    *out_handle = make_handle(r, slot);
    return BPS_OK;
}

}  // namespace

bps_status bps_load_scene(bps_renderer* r, const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T,
                          const uint8_t* colors, bps_scene* out_handle) {
    if (!r) return BPS_ERR_INVALID_ARG;
    bps_status st = load_scene_on(r, vertices, V, indices, T, colors, TextureArg{}, r->load_stream, out_handle);
    if (st != BPS_OK) return st;
    BPS_HIP(r, hipStreamSynchronize(r->load_stream));
    std::lock_guard<std::mutex> lock(r->mu);
    const int slot = slot_of(r, *out_handle);
    if (slot < 0) return BPS_OK;      // (another thread has retired it already)
    HostScene& hs = r->scenes[slot];
    if (hs.ready) (void)hipEventDestroy(hs.ready);
    hs.ready = nullptr;
    return BPS_OK;
}

bps_status bps_load_scene_async(bps_renderer* r, const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T,
                                const uint8_t* colors, void* copy_stream, bps_scene* out_handle) {
    if (!r) return BPS_ERR_INVALID_ARG;
    return load_scene_on(r, vertices, V, indices, T, colors, TextureArg{}, (hipStream_t)copy_stream, out_handle);
}

bps_status bps_load_scene_textured(bps_renderer* r, const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T,
                                   const float* uvs, const uint8_t* texels, uint32_t tex_w, uint32_t tex_h,
                                   void* copy_stream, bps_scene* out_handle) {
    if (!r) return BPS_ERR_INVALID_ARG;
    if (!uvs || !texels) return fail(r, BPS_ERR_INVALID_ARG, "bps_load_scene_textured: null uvs or texels");
    TextureArg tex;
    tex.uvs = uvs;
    tex.texels = texels;
    tex.w = tex_w;
    tex.h = tex_h;
    hipStream_t stream = copy_stream ? (hipStream_t)copy_stream : r->load_stream;
    bps_status st = load_scene_on(r, vertices, V, indices, T, nullptr, tex, stream, out_handle);
    if (st != BPS_OK || copy_stream) return st;
    BPS_HIP(r, hipStreamSynchronize(r->load_stream));
    std::lock_guard<std::mutex> lock(r->mu);
    const int slot = slot_of(r, *out_handle);
    if (slot < 0) return BPS_OK;      // (another thread has retired it already)
    HostScene& hs = r->scenes[slot];
    if (hs.ready) (void)hipEventDestroy(hs.ready);
    hs.ready = nullptr;
    return BPS_OK;
}

bps_status bps_scene_ready(bps_renderer* r, bps_scene scene, int32_t* ready) {
    if (!r || !ready) return BPS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(r->mu);
    const int slot = slot_of(r, scene);
    if (slot < 0) return fail(r, BPS_ERR_BAD_HANDLE, "bps_scene_ready: scene %d is not loaded", scene);
    HostScene& hs = r->scenes[slot];
    if (hs.ready && hipEventQuery(hs.ready) == hipSuccess) {
        (void)hipEventDestroy(hs.ready);
        hs.ready = nullptr;
    }
    (void)hipGetLastError();
    *ready = hs.ready == nullptr ? 1 : 0;
    return BPS_OK;
}

bps_status bps_pack_clusters(const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T, uint32_t* count,
                             float* verts_out, uint32_t* tris_out, uint32_t* ids_out) {
    if (!vertices || !indices || !count || V == 0 || T == 0) return BPS_ERR_INVALID_ARG;
    for (size_t i = 0; i < 3 * (size_t)T; ++i)
        if (indices[i] >= V) return BPS_ERR_INVALID_ARG;
    bps::ClusterSet cs;
    try {
        cs = bps::build_clusters(vertices, V, indices, T);
    } catch (const std::bad_alloc&) {
        return BPS_ERR_OOM;
    }
    const uint32_t room = *count;
    *count = cs.count;
    if (!verts_out && !tris_out && !ids_out) return BPS_OK;
    if (room < cs.count) return BPS_ERR_INVALID_ARG;
    if (verts_out) std::memcpy(verts_out, cs.verts.data(), cs.verts.size() * sizeof(float));
    if (tris_out) std::memcpy(tris_out, cs.tris.data(), cs.tris.size() * sizeof(uint32_t));
    if (ids_out) std::memcpy(ids_out, cs.tri_id.data(), cs.tri_id.size() * sizeof(uint32_t));
    return BPS_OK;
}

bps_status bps_unload_scene(bps_renderer* r, bps_scene scene) {
    if (!r) return BPS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(r->mu);
    const int slot = slot_of(r, scene);
    if (slot < 0) return fail(r, BPS_ERR_BAD_HANDLE, "bps_unload_scene: scene %d is not loaded", scene);
    BPS_HIP(r, hipSetDevice(r->device));
    HostScene& hs = r->scenes[slot];
    // queued requests may still read the block and the table slot, and the scene's own upload may
    // still be writing it: park both until all of that is over (nothing here waits for the device)
    Retired x;
    x.arena = hs.arena;
    x.slot = slot;
    x.last_use = hs.last_use;
    x.upload = hs.ready;
    r->retired.push_back(x);
    hs = HostScene{};
    r->gens[slot] = (r->gens[slot] + 1u) & ((1u << (31 - kSlotBits)) - 1u);      // handles to the old scene stop matching
    r->plan_ids.clear();
    collect(r);
    return BPS_OK;
}

bps_status bps_render(bps_renderer* r, const bps_scene* scene_ids, const float* view_proj, uint32_t B, float* out_depth,
                      uint8_t* out_rgb, uint32_t* out_tri_id, void* stream_) {
    if (!r) return BPS_ERR_INVALID_ARG;
    if (B == 0) return BPS_OK;
    std::lock_guard<std::mutex> lock(r->mu);
    if (!scene_ids || !view_proj || !out_depth) return fail(r, BPS_ERR_INVALID_ARG, "bps_render: null argument");
    if (B > (uint32_t)r->cfg.max_batch)
        return fail(r, BPS_ERR_INVALID_ARG, "bps_render: B=%u exceeds max_batch=%d", B, r->cfg.max_batch);
    const bool rgbd = r->cfg.mode == BPS_MODE_RGBD;
    if (rgbd && !out_rgb) return fail(r, BPS_ERR_INVALID_ARG, "bps_render: out_rgb is required in RGB-D mode");
    hipStream_t stream = (hipStream_t)stream_;
    uint32_t min_clusters = 0xFFFFFFFFu;
    r->call_slots.resize(B);
    for (uint32_t b = 0; b < B; ++b) {
        const int s = slot_of(r, scene_ids[b]);
        if (s < 0) return fail(r, BPS_ERR_BAD_HANDLE, "bps_render: scene_ids[%u]=%d is not a loaded scene", b, scene_ids[b]);
        if (rgbd && !r->scenes[s].has_colors)
            return fail(r, BPS_ERR_INVALID_ARG, "bps_render: scene %d (scene_ids[%u]) was loaded without colours", scene_ids[b], b);
        min_clusters = std::min(min_clusters, r->scenes[s].dev.n_clusters);
        r->call_slots[b] = s;
    }
    scene_ids = r->call_slots.data();      // table slots from here on
    BPS_HIP(r, hipSetDevice(r->device));
    const uint64_t seq = ++r->seq;
    std::vector<hipEvent_t> uploads_pending;      // asynchronous scene uploads this request has to follow
    for (uint32_t b = 0; b < B; ++b) {
        HostScene& hs = r->scenes[scene_ids[b]];
        if (hs.last_use == seq) continue;     // already handled for this request
        hs.last_use = seq;
        if (hs.ready) {                       // asynchronous upload: order this request after the copy
            if (hipEventQuery(hs.ready) == hipSuccess) {
                (void)hipEventDestroy(hs.ready);
                hs.ready = nullptr;
            } else {
                (void)hipGetLastError();
                BPS_HIP(r, hipStreamWaitEvent(stream, hs.ready, 0));
                uploads_pending.push_back(hs.ready);
            }
        }
    }
    const int H = r->rh, W = r->rw;       // rendered size
    const size_t HW = (size_t)H * W;
    float* final_depth = out_depth;
    uint8_t* final_rgb = out_rgb;
    if (r->ss > 1) {
        if (out_tri_id) return fail(r, BPS_ERR_INVALID_ARG, "bps_render: triangle ids are not available with supersampling");
        if (!r->ss_depth) BPS_HIP(r, hipMalloc((void**)&r->ss_depth, (size_t)r->cfg.max_batch * HW * sizeof(float)));
        if (rgbd && !r->ss_rgb) BPS_HIP(r, hipMalloc((void**)&r->ss_rgb, (size_t)r->cfg.max_batch * HW * 3));
        out_depth = r->ss_depth;
        out_rgb = r->ss_rgb;
    }
    const int S = plan_splits(r, B, min_clusters);

    make_plan(r, scene_ids, B, S);
    const size_t n_items = r->plan_items.size();

    // ---- stage the request (work items + matrices unless they already live on the device)
    hipPointerAttribute_t attr;
    bool vp_on_device = false;
    if (hipPointerGetAttributes(&attr, view_proj) == hipSuccess) vp_on_device = attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged;
    (void)hipGetLastError();
    const size_t items_bytes = n_items * sizeof(bps::WorkItem);
    const size_t vp_bytes = (size_t)B * 16 * sizeof(float);
    const size_t ids_bytes = rgbd ? (size_t)B * sizeof(uint32_t) : 0;
    // costliest-first dispatch pays off once the launch no longer fits on the device in one go
    const bool planned = fp_cull_enabled(r) && n_items > (size_t)2 * r->num_cu && n_items <= bps::kMaxPlannedItems &&
                         !(r->cfg.flags & BPS_FLAG_NO_DISPATCH_ORDER);
    const size_t plan_bytes = planned ? n_items * (sizeof(bps::WorkItem) + sizeof(uint32_t)) + 16 : 0;
    const size_t need = items_bytes + ids_bytes + vp_bytes + plan_bytes;
    RingSlot& slot = r->ring[r->ring_next];
    r->ring_next = (r->ring_next + 1) % kRing;
    if (slot.pending) {
        BPS_HIP(r, hipEventSynchronize(slot.done));
        slot.pending = false;
    }
    if (slot.capacity < need) {
        if (slot.host) (void)hipHostFree(slot.host);
        if (slot.dev) (void)hipFree(slot.dev);
        slot.host = slot.dev = nullptr;
        slot.capacity = 0;
        size_t cap = std::max<size_t>(need, 1 << 16);
        BPS_HIP(r, hipHostMalloc((void**)&slot.host, cap, hipHostMallocDefault));
        BPS_HIP(r, hipMalloc((void**)&slot.dev, cap));
        slot.capacity = cap;
        slot.items_version = 0;
    }
    unsigned char* const payload = slot.dev;
    // The work items only change with the scene ids: each slot keeps the copy it has until then, so
    // a depth request whose matrices are on the device stages nothing at all.
    size_t copy_from = items_bytes, copy_to = items_bytes;
    if (slot.items_version != r->plan_version) {
        std::memcpy(slot.host, r->plan_items.data(), items_bytes);
        copy_from = 0;
    }
    if (rgbd) {
        std::memcpy(slot.host + items_bytes, scene_ids, ids_bytes);
        copy_to = items_bytes + ids_bytes;
    }
    if (!vp_on_device) {
        std::memcpy(slot.host + items_bytes + ids_bytes, view_proj, vp_bytes);
        copy_to = items_bytes + ids_bytes + vp_bytes;
    }
    // Staging and launch planning read nothing but the request.  When the request is complete at the
    // call (host matrices, or device matrices the caller vouches for), they run on the renderer's own
    // stream and may start while the caller's stream is still busy with earlier work: the planning
    // kernels then fill the compute units that the end of the previous request's launch leaves idle.
    const bool early = planned && (!vp_on_device || (r->cfg.flags & BPS_FLAG_INPUTS_READY));
    // (the stream is made on first use: the device has few hardware queues, and a stream nobody uses
    // could take the one that lets two caller streams run side by side)
    if (early && !r->plan_stream) BPS_HIP(r, hipStreamCreateWithFlags(&r->plan_stream, hipStreamNonBlocking));
    hipStream_t pstream = early ? r->plan_stream : stream;
    if (early)
        for (hipEvent_t e : uploads_pending) BPS_HIP(r, hipStreamWaitEvent(pstream, e, 0));
    if (copy_to > copy_from)
        BPS_HIP(r, hipMemcpyAsync(payload + copy_from, slot.host + copy_from, copy_to - copy_from, hipMemcpyHostToDevice, pstream));
    slot.items_version = r->plan_version;
    const bps::WorkItem* d_items = reinterpret_cast<const bps::WorkItem*>(payload);
    const uint32_t* d_env_scene = reinterpret_cast<const uint32_t*>(payload + items_bytes);
    const float* d_vp = vp_on_device ? view_proj : reinterpret_cast<const float*>(payload + items_bytes + ids_bytes);
    // planning area: the items in launch order (16-byte aligned), then cost and order words
    const size_t plan_at = (items_bytes + ids_bytes + vp_bytes + 15) & ~(size_t)15;
    bps::WorkItem* d_ordered = reinterpret_cast<bps::WorkItem*>(payload + plan_at);
    uint32_t* d_cost = reinterpret_cast<uint32_t*>(d_ordered + n_items);

    // ---- RGB-D: the colour pass needs the winning triangle ids even when the caller does not
    if (rgbd && !out_tri_id) {
        if (!r->ids) BPS_HIP(r, hipMalloc((void**)&r->ids, (size_t)r->cfg.max_batch * HW * sizeof(uint32_t)));
        out_tri_id = r->ids;
    }

    // ---- global visibility buffer, only when frames are split
    if (S > 1 && !r->gvis) {
        size_t n = (size_t)r->cfg.max_batch * HW;
        BPS_HIP(r, hipMalloc((void**)&r->gvis, n * sizeof(unsigned long long)));
        hipLaunchKernelGGL(bps::k_fill_keys, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, r->gvis, n);
        BPS_HIP(r, hipGetLastError());
    }

    // Requests on one stream run in order.  A request on another stream may overlap the previous one
    // unless both use one of the renderer's own buffers: then it waits for that one.
    // ---- RGB-D: queue of the pixels whose winning triangle crosses a clip plane, and its two counters
    if (rgbd && !r->shade_queue) {
        const size_t n = (size_t)bps::kShadeQueues * bps::shade_queue_cap((size_t)r->cfg.max_batch * HW);
        BPS_HIP(r, hipMalloc((void**)&r->shade_queue, (n + 2 * 32 * bps::kShadeQueues) * sizeof(uint32_t)));
        BPS_HIP(r, hipMemsetAsync(r->shade_queue + n, 0, 2 * 32 * bps::kShadeQueues * sizeof(uint32_t), stream));
    }
    const bool uses_shared = rgbd || S > 1 || r->ss > 1 || r->want_stats;
    if (uses_shared && r->shared_done && r->shared_stream != stream) BPS_HIP(r, hipStreamWaitEvent(stream, r->shared_done, 0));

    const bps::FrameParams fp = frame_params(r, S);

    unsigned long long* d_stats = nullptr;
    if (r->want_stats) {
        if (r->stats_cap < 16 * n_items) {
            if (r->d_stats) (void)hipFree(r->d_stats);
            r->d_stats = nullptr;
            r->stats_cap = 0;
            BPS_HIP(r, hipMalloc((void**)&r->d_stats, (16 * n_items) * sizeof(unsigned long long)));
            r->stats_cap = 16 * n_items;
        }
        hipLaunchKernelGGL(bps::k_zero_words, dim3((unsigned)((16 * n_items + 255) / 256)), dim3(256), 0, stream, r->d_stats,
                           16 * n_items);
        d_stats = r->d_stats;
    }
    if (planned) {
        bps::launch_plan(pstream, r->d_scenes, d_items, d_vp, fp, (uint32_t)n_items, d_cost, d_ordered);
        BPS_HIP(r, hipGetLastError());
        if (early) {
            BPS_HIP(r, hipEventRecord(slot.planned, pstream));
            BPS_HIP(r, hipStreamWaitEvent(stream, slot.planned, 0));
        }
    }
    hipEvent_t ev_stop = nullptr;      // profiling: the events bracket the raster kernel alone
    if (r->profiling && (r->profile_count++ % r->profile_every) == 0 && r->ev_used + 2 <= 2 * kMaxProfiled) {
        while (r->ev.size() < r->ev_used + 2) {
            hipEvent_t e;
            BPS_HIP(r, hipEventCreate(&e));
            r->ev.push_back(e);
        }
        BPS_HIP(r, hipEventRecord(r->ev[r->ev_used], stream));
        ev_stop = r->ev[r->ev_used + 1];
        r->ev_used += 2;
    }
    bps::launch_raster(r->threads, dim3((unsigned)n_items), r->lds, stream, r->d_scenes, planned ? d_ordered : d_items, d_vp, fp,
                       r->gvis, out_depth, out_tri_id, d_stats);
    BPS_HIP(r, hipGetLastError());
    if (ev_stop) BPS_HIP(r, hipEventRecord(ev_stop, stream));
    if (S > 1) {
        size_t n = (size_t)B * HW;
        hipLaunchKernelGGL(bps::k_resolve, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, r->gvis, n, fp.background,
                           out_depth, out_tri_id);
        BPS_HIP(r, hipGetLastError());
    }
    if (rgbd) {
        uint32_t* counters = r->shade_queue + (size_t)bps::kShadeQueues * bps::shade_queue_cap((size_t)r->cfg.max_batch * HW);
        bps::launch_shade(stream, r->d_scenes, d_env_scene, d_vp, fp, B, out_tri_id, out_rgb, r->shade_queue,
                          counters + 32 * bps::kShadeQueues * r->shade_parity,
                          counters + 32 * bps::kShadeQueues * (r->shade_parity ^ 1u));
        r->shade_parity ^= 1u;
        BPS_HIP(r, hipGetLastError());
    }
    if (r->ss > 1) {
        bps::launch_downsample(stream, out_depth, out_rgb, B, H, W, final_depth, final_rgb);
        BPS_HIP(r, hipGetLastError());
    }
    BPS_HIP(r, hipEventRecord(slot.done, stream));
    slot.pending = true;
    slot.seq = seq;
    if (uses_shared) {
        r->shared_done = slot.done;
        r->shared_stream = stream;
    }
    r->last_splits = (uint64_t)S;
    r->last_groups = (uint64_t)n_items;
    return BPS_OK;
}

bps_status bps_render_static(bps_renderer* r, const bps_scene* scene_ids, const float* view_proj, uint32_t B,
                             float* out_depth, uint32_t* out_tri_id, void* stream_) {
    if (!r) return BPS_ERR_INVALID_ARG;
    if (B == 0) return BPS_OK;
    std::lock_guard<std::mutex> lock(r->mu);
    if (!scene_ids || !view_proj || !out_depth) return fail(r, BPS_ERR_INVALID_ARG, "bps_render_static: null argument");
    if (B > (uint32_t)r->cfg.max_batch)
        return fail(r, BPS_ERR_INVALID_ARG, "bps_render_static: B=%u exceeds max_batch=%d", B, r->cfg.max_batch);
    if (r->cfg.mode != BPS_MODE_DEPTH || r->ss > 1 || r->want_stats || r->cfg.splits > 1)
        return fail(r, BPS_ERR_UNSUPPORTED,
                    "bps_render_static: depth renderers only, without supersampling, forced splits or diagnostics");
    const size_t n_items = (size_t)B * (size_t)r->tiles;
    if (n_items > kStaticMaxItems || B > 0xFFFFu)
        return fail(r, BPS_ERR_INVALID_ARG, "bps_render_static: %zu work-groups (B x tiles of the frame) exceed the static scratch (%u)",
                    n_items, kStaticMaxItems);
    if (!r->static_scratch) return fail(r, BPS_ERR_UNSUPPORTED, "bps_render_static: no static scratch on device %d", r->device);
    hipPointerAttribute_t attr;
    const bool vp_on_device = hipPointerGetAttributes(&attr, view_proj) == hipSuccess &&
                              (attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged);
    (void)hipGetLastError();
    if (!vp_on_device) return fail(r, BPS_ERR_INVALID_ARG, "bps_render_static: view_proj must be device memory");
    hipStream_t stream = (hipStream_t)stream_;
    r->call_slots.resize(B);
    for (uint32_t b = 0; b < B; ++b) {
        const int s = slot_of(r, scene_ids[b]);
        if (s < 0) return fail(r, BPS_ERR_BAD_HANDLE, "bps_render_static: scene_ids[%u]=%d is not a loaded scene", b, scene_ids[b]);
        r->call_slots[b] = s;
    }
    scene_ids = r->call_slots.data();      // table slots from here on
    BPS_HIP(r, hipSetDevice(r->device));
    const uint64_t seq = ++r->seq;
    for (uint32_t b = 0; b < B; ++b) {
        HostScene& hs = r->scenes[scene_ids[b]];
        if (hs.last_use == seq) continue;
        hs.last_use = seq;
        if (hs.ready) {                       // asynchronous upload: order this request after the copy
            if (hipEventQuery(hs.ready) == hipSuccess) {
                (void)hipEventDestroy(hs.ready);
                hs.ready = nullptr;
            } else {
                (void)hipGetLastError();
                BPS_HIP(r, hipStreamWaitEvent(stream, hs.ready, 0));
            }
        }
    }
    make_plan(r, scene_ids, B, 1);      // (host containers only; they keep their capacity between calls)
    // a ring slot is taken for its completion event only: scene retirement tracks requests through them
    RingSlot& slot = r->ring[r->ring_next];
    r->ring_next = (r->ring_next + 1) % kRing;
    if (slot.pending) {
        BPS_HIP(r, hipEventSynchronize(slot.done));
        slot.pending = false;
    }
    // layout of the static array: items as planned, items in launch order, cost words
    bps::WorkItem* d_items = reinterpret_cast<bps::WorkItem*>(r->static_scratch);
    bps::WorkItem* d_ordered = d_items + kStaticMaxItems;
    uint32_t* d_cost = reinterpret_cast<uint32_t*>(d_ordered + kStaticMaxItems);
    {   // the items reach the device as kernel arguments, unless the array still holds this very plan
        std::lock_guard<std::mutex> g(g_scratch_mu);
        if (g_scratch_owner[r->device] != r || g_scratch_plan[r->device] != r->plan_version) {
            bps::PackedItems packed;
            for (size_t first = 0; first < n_items; first += bps::kPackedItemsPerLaunch) {
                const uint32_t count = (uint32_t)std::min<size_t>(bps::kPackedItemsPerLaunch, n_items - first);
                for (uint32_t k = 0; k < count; ++k) {
                    const bps::WorkItem& it = r->plan_items[first + k];
                    packed.word[k] = it.env | (it.scene << 16) | (it.tile << 28);
                }
                bps::launch_unpack_items(stream, packed, (uint32_t)first, count, d_items);
                BPS_HIP(r, hipGetLastError());
            }
            g_scratch_owner[r->device] = r;
            g_scratch_plan[r->device] = r->plan_version;
        }
    }
    const bps::FrameParams fp = frame_params(r, 1);
    const bool planned = fp_cull_enabled(r) && n_items > (size_t)2 * r->num_cu && !(r->cfg.flags & BPS_FLAG_NO_DISPATCH_ORDER);
    if (planned) {
        bps::launch_plan(stream, r->d_scenes, d_items, view_proj, fp, (uint32_t)n_items, d_cost, d_ordered);
        BPS_HIP(r, hipGetLastError());
    }
    bps::launch_raster(r->threads, dim3((unsigned)n_items), r->lds, stream, r->d_scenes, planned ? d_ordered : d_items, view_proj,
                       fp, nullptr, out_depth, out_tri_id, nullptr);
    BPS_HIP(r, hipGetLastError());
    BPS_HIP(r, hipEventRecord(slot.done, stream));
    slot.pending = true;
    slot.seq = seq;
    r->last_splits = 1;
    r->last_groups = (uint64_t)n_items;
    return BPS_OK;
}

bps_status bps_set_profiling(bps_renderer* r, int32_t enable) {
    if (!r) return BPS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(r->mu);
    r->profiling = enable != 0;
    r->profile_every = enable > 1 ? (uint32_t)enable : 1u;
    r->profile_count = 0;
    r->ev_used = 0;
    return BPS_OK;
}

bps_status bps_last_kernel_ms(bps_renderer* r, float* ms) {
    if (!r || !ms) return BPS_ERR_INVALID_ARG;
    if (r->ev_used < 2) return fail(r, BPS_ERR_INVALID_ARG, "bps_last_kernel_ms: no profiled request yet");
    BPS_HIP(r, hipEventSynchronize(r->ev[r->ev_used - 1]));
    BPS_HIP(r, hipEventElapsedTime(ms, r->ev[r->ev_used - 2], r->ev[r->ev_used - 1]));
    return BPS_OK;
}

bps_status bps_kernel_ms_total(bps_renderer* r, uint32_t* launches, float* total_ms) {
    if (!r || !launches || !total_ms) return BPS_ERR_INVALID_ARG;
    float sum = 0.0f;
    for (size_t k = 0; k + 1 < r->ev_used; k += 2) {
        float ms = 0.0f;
        BPS_HIP(r, hipEventSynchronize(r->ev[k + 1]));
        BPS_HIP(r, hipEventElapsedTime(&ms, r->ev[k], r->ev[k + 1]));
        sum += ms;
    }
    *launches = (uint32_t)(r->ev_used / 2);
    *total_ms = sum;
    r->ev_used = 0;
    return BPS_OK;
}

bps_status bps_kernel_ms_each(bps_renderer* r, float* out, uint32_t capacity, uint32_t* written) {
    if (!r || !out || !written) return BPS_ERR_INVALID_ARG;
    uint32_t n = 0;
    for (size_t k = 0; k + 1 < r->ev_used && n < capacity; k += 2, ++n) {
        BPS_HIP(r, hipEventSynchronize(r->ev[k + 1]));
        BPS_HIP(r, hipEventElapsedTime(&out[n], r->ev[k], r->ev[k + 1]));
    }
    *written = n;
    r->ev_used = 0;
    return BPS_OK;
}

bps_status bps_set_diagnostics(bps_renderer* r, int32_t enable) {
    if (!r) return BPS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(r->mu);
    r->want_stats = enable != 0;
    r->stats_mode = enable > 1 ? (enable <= 4 ? enable - 1 : 1) : 0;
    return BPS_OK;
}

bps_status bps_read_diagnostics(bps_renderer* r, uint64_t* out, uint32_t capacity, uint32_t* written) {
    if (!r || !out || !written) return BPS_ERR_INVALID_ARG;
    if (!r->d_stats) return fail(r, BPS_ERR_INVALID_ARG, "bps_read_diagnostics: no request ran with diagnostics enabled");
    BPS_HIP(r, hipSetDevice(r->device));
    BPS_HIP(r, hipDeviceSynchronize());
    size_t n = std::min<size_t>(capacity, 16 * (size_t)r->last_groups);
    BPS_HIP(r, hipMemcpy(out, r->d_stats, n * sizeof(uint64_t), hipMemcpyDeviceToHost));
    *written = (uint32_t)n;
    return BPS_OK;
}

bps_status bps_query(bps_renderer* r, bps_scene scene, int32_t what, uint64_t* value) {
    if (!r || !value) return BPS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(r->mu);
    if (what >= 0 && what <= 3) {
        const int slot = slot_of(r, scene);
        if (slot < 0) return fail(r, BPS_ERR_BAD_HANDLE, "bps_query: scene %d is not loaded", scene);
        const HostScene& s = r->scenes[slot];
        *value = what == 0 ? s.dev.n_clusters : what == 1 ? s.dev.n_tris : what == 2 ? s.dev.n_verts : s.bytes;
        return BPS_OK;
    }
    switch (what) {
    case 4: *value = r->last_splits; return BPS_OK;
    case 5: *value = r->last_groups; return BPS_OK;
    case 6: *value = (uint64_t)r->threads; return BPS_OK;
    case 7: *value = (uint64_t)r->lds; return BPS_OK;
    case 8: *value = r->arena_allocs; return BPS_OK;
    case 9: *value = (uint64_t)r->arena_pool.size() + (uint64_t)r->retired.size(); return BPS_OK;
    default: return fail(r, BPS_ERR_INVALID_ARG, "bps_query: unknown item %d", what);
    }
}

}  // extern "C"
