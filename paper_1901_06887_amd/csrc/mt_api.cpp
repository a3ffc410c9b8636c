// Host side of the multi-tenant worker runtime: the C ABI of include/mt.h, the tenant
// registry (closed layer set, paper section 3.1), the packed weight arena in device memory
// (models stay resident on the accelerator, section 3.3) and the fixed launch sequence of
// mt_run (segmentation, gather, one grouped launch per layer index, head).
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <string>
#include <vector>

#include "mt_internal.h"
#include "../../include/mt_debug.h"

using namespace mt;

// Scratch of mt_run_static: batch descriptors, both activation buffers and logits of one run.  The
// array lives in device memory of every GPU the library runs on until the process ends.  On the
// host its name is only a handle: the device address is looked up once per context
// (hipGetSymbolAddress in mt_create, with the context's device current) and kept in the context.
static __device__ __align__(256) unsigned char scratch[MT_STATIC_SCRATCH_BYTES];


namespace {

constexpr uint32_t kMaxTenants = 2048;
constexpr uint32_t kSegSlots = MT_SEG_SLOTS;   // pinned segment tables: runs of several submissions in flight at once
constexpr uint32_t kMaxRunSlots = 4;      // runs in flight at once (each with its own device scratch); <= kSegSlots
constexpr uint64_t kArenaAlign = 256;
// profiling slots: batcher, gather, head, then gemm and gap of every layer index
constexpr uint32_t kProfBatcher = 0, kProfGather = 1, kProfHead = 2, kProfFc = 3, kProfConv = 3 + MT_MAX_LAYERS,
                   kProfGap = 3 + 2 * MT_MAX_LAYERS, kProfBig = 3 + 3 * MT_MAX_LAYERS, kProfGatherImg = 3 + 4 * MT_MAX_LAYERS,
                   kProfImageOps = 4 + 4 * MT_MAX_LAYERS;
constexpr uint32_t kProfSlots = 4 + 5 * MT_MAX_LAYERS;

inline uint32_t round_up(uint32_t v, uint32_t a) { return (v + a - 1) / a * a; }
inline uint64_t round_up64(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

struct HostLayer {
    mt_layer_spec spec;
    LayerDev dev;               // w_off / b_off: absolute arena offsets while the model is resident
    uint64_t w_bytes, b_bytes;
    uint64_t w_rel, b_rel;      // the same offsets relative to the model's arena block
};

struct HostTenant {
    bool registered = false;
    uint32_t n_layers = 0;
    HostLayer layers[MT_MAX_LAYERS];
    TenantDev dev{};
    uint64_t arena_off = 0, arena_len = 0;
    uint32_t act_buffers = 2;   // activation buffers a run needs for this model (two for a chain)
    // Model cache (cfg.cache): the packed weights stay in pinned host memory (`stage`: the arena
    // image followed by the device table rows of this tenant) and the arena holds the models used
    // most recently.  Outside cache mode every registered model is resident and stage is null.
    bool resident = false;
    uint64_t last_use = 0;
    uint8_t* stage = nullptr;
};

struct FreeBlock { uint64_t off, len; };

// Device scratch of one run in flight: batch descriptors, activation buffers, logits.  A run owns
// one slot from its batcher to its last kernel; the weights and model tables are shared.
struct RunSlot {
    int32_t* d_row_tenant = nullptr; uint32_t* d_row_rank = nullptr; uint32_t* d_hist_g = nullptr;
    const void** d_row_src = nullptr; int32_t* d_pos_of = nullptr; int32_t* d_perm = nullptr;
    uint32_t* d_M = nullptr; uint32_t* d_off = nullptr; uint32_t* d_tile_base = nullptr;
    void* d_act[kActBuffers] = {}; float* d_logits = nullptr;   // (only as many activation buffers as the registered models need)
    hipEvent_t done = nullptr;      // recorded behind the slot's last run
    hipStream_t stream = nullptr;   // ... which was enqueued here
    uint64_t last_run = 0;          // ... and was the context's run number this
    bool used = false;
};

}  // namespace

struct mt_ctx {
    mt_config cfg{};
    bool host_only = false;
    uint32_t elem_size = 2;
    uint32_t S = 0;        // elements between consecutive requests in an activation buffer
    uint32_t C_pad = 0;    // floats between consecutive rows of the internal logits buffer
    std::vector<HostTenant> tenants;
    std::vector<FreeBlock> free_list;
    uint64_t arena_used = 0;
    uint32_t n_registered = 0;

    // per layer index, over registered tenants: bounds that size the grouped launches
    uint32_t n_layer_slots = 0;
    uint32_t max_in_len = 0;
    // [kind][layer]: kind 0 = FC tiles, 1 = conv tiles, 2 = big FC tiles
    uint32_t max_rpr[kListKinds][MT_MAX_LAYERS]{}, max_nt[kListKinds][MT_MAX_LAYERS]{}, has_gap[MT_MAX_LAYERS]{};
    // pool_fused[l]: layer index l + 1 is a global average pool for every registered model that is that deep, and
    // each of their convolutions at l can pool by itself: the convolution launch writes the pooled activation
    // and nothing runs at index l + 1 (all or nothing: the activation buffers alternate per layer index)
    bool pool_fused[MT_MAX_LAYERS]{};
    double sum_macs = 0.0;                           // multiply-accumulates of one request, summed over the registered tenants
    uint32_t max_conv_cb[MT_MAX_LAYERS]{};
    uint32_t conv_img_lds[MT_MAX_LAYERS]{};          // every conv of a layer index can keep its tiles' input in LDS: the largest frame in bytes, else 0
    int conv_img_two[MT_MAX_LAYERS]{};               // ... and their pixels are one 16-byte chunk: 1, none is: 0 (-1: no convolution seen yet)
    uint32_t no_conv_img = 0;                        // tuning: never use that kernel
    bool conv_uniform[MT_MAX_LAYERS]{};              // every conv of a layer index has input channels in multiples of a k step, and a window of at most 64 taps
    bool conv_quad[MT_MAX_LAYERS]{};                 // every conv of a layer index has input channels in multiples of four 16-byte chunks           // widest conv tile (32-channel blocks, at most 4) of a layer index
    uint64_t sum_nt[kListKinds][MT_MAX_LAYERS]{};
    uint32_t max_fc_per64[MT_MAX_LAYERS]{};   // streaming FC tiles per 64 rows of one tenant, maximum over the registered models
    uint64_t sum_nt_sk[MT_MAX_LAYERS]{};      // the same two figures for the K-split tile shape
    uint32_t max_fc_per64_sk[MT_MAX_LAYERS]{};
    uint32_t max_big_blocks[MT_MAX_LAYERS]{};  // most column blocks of a registered FC layer whose rows past the big tiles take K-split tiles
    uint32_t fc_split_k = 0;   // tuning: every run uses FC tiles of one column block with K split four ways
    uint32_t no_auto_split_k = 0;   // tuning: small runs keep the ordinary tile shape
    uint32_t no_fused_gather = 0;  // tuning/testing: always stage FC inputs with the gather kernel
    bool fc_first_chunked = true;  // every registered FC-first model's input is a whole number of 16-byte chunks
    bool any_conv_first = false, any_fc_first = false;
    uint32_t list_mask[MT_MAX_LAYERS / kLayerGroup] = {};   // per group of layer indices, bit kind*kLayerGroup + l%kLayerGroup: some registered model has that kind at layer l
    uint32_t has_image_ops[MT_MAX_LAYERS]{};   // some registered model has a max-pool or an addition at this layer index
    uint32_t image_op_fill[MT_MAX_LAYERS]{};   // ... and the longest output row (elements) among them
    uint32_t max_image_pixels = 0;             // most pixels in a submitted image (models whose first layer is a convolution)
    uint32_t act_buffers = 2;      // activation buffers every run slot holds (grows when a model with skip connections needs more)
    uint32_t max_reg_classes = 0, min_reg_classes = 0;
    uint32_t no_fused_head = 0;    // tuning/testing: always run the separate head kernel
    uint32_t no_fused_pool = 0;    // tuning/testing: always run the separate pooling kernel
    uint32_t no_fused_add = 0;     // tuning/testing: residual additions always run as launches of their own
    uint32_t big_walk = 1;         // big FC tiles: one workgroup per CU walks several tiles (tuning/testing: MT_BIG_WALK=0 gives every tile a workgroup of its own)
    uint32_t n_cus = 256;          // compute units of the device, rounded down to a multiple of 8
    uint32_t min_fc_k[MT_MAX_LAYERS]{};        // shortest padded fan-in among the registered FC layers of a layer index
    uint32_t no_conv_uniform = 0;  // tuning/testing: convolution gathers always walk the window lane by lane
    uint32_t no_conv_loaders = 0;  // tuning/testing: convolution tiles never get waves of their own for the loads
    uint32_t min_conv_k[MT_MAX_LAYERS]{};      // shortest reduction among the registered convolutions of a layer index
    uint32_t big_min_tiles = kBigMinTiles;   // testing: MT_BIG_MIN_TILES=1 sends every qualifying tenant-layer to big tiles
    uint32_t P_cap = 0;        // packed rows incl. per-tenant padding to 32

    // device state.  The per-run pointers below (d_row_tenant .. d_logits) are those of the run
    // slot bound last (bind_slot): the slot of the run being enqueued, then of the last run.
    std::vector<RunSlot> slots;
    RunSlot static_slot;               // the slot of mt_run_static: its buffers are carved out of static_scratch per run
    uint8_t* static_scratch = nullptr; // device address of `scratch` on this context's GPU
    uint8_t* d_arena = nullptr;
    TenantDev* d_tenants = nullptr;
    LayerDev* d_layers = nullptr;
    uint64_t* d_served = nullptr;      // [max_tenants][2]: requests served, runs with at least one request (accounting)
    uint32_t* d_facts = nullptr;       // [max_tenants][MT_MAX_LAYERS][2]: the batcher's view of the layers (BatchArgs::facts)
    int32_t* d_row_tenant = nullptr;
    uint32_t* d_row_rank = nullptr;
    uint32_t* d_hist_g = nullptr;      // [kHistEntries] per-workgroup tenant histograms of the ranking kernel
    const void** d_row_src = nullptr;
    int32_t* d_pos_of = nullptr;
    int32_t* d_perm = nullptr;
    uint32_t* d_M = nullptr;
    uint32_t* d_off = nullptr;
    void* d_zeros = nullptr;           // 256 bytes of zeros: where masked operand loads point instead of branching
    uint32_t* d_tile_base = nullptr;   // [kListKinds][MT_MAX_LAYERS][T+1]: FC, conv and big-FC arrays, then one word: the big-tile layer mask
    void* d_act[kActBuffers] = {};
    float* d_logits = nullptr;
    Segment* h_segs[kSegSlots] = {};    // pinned, device-visible
    Segment* d_segs[kSegSlots] = {};    // device addresses of the same memory
    hipEvent_t seg_event[kSegSlots] = {};
    bool seg_busy[kSegSlots] = {};
    uint64_t run_count = 0;
    hipStream_t last_stream = nullptr;

    // model cache
    bool cache = false;
    uint64_t use_clock = 0;                 // stamps HostTenant::last_use
    hipEvent_t cache_event = nullptr;       // recorded behind the last asynchronous residency change
    hipStream_t cache_stream = nullptr;
    bool cache_pending = false;
    uint64_t n_uploads = 0, upload_bytes = 0, n_evictions = 0;

    // pending submissions
    std::vector<Segment> pending;
    uint32_t pending_rows = 0;

    uint32_t last_run_rows = 0, last_run_launches = 0;
    std::string err;

    // optional per-kernel timing: event 2*i / 2*i+1 bracket launch slot i
    bool profiling = false;
    std::vector<hipEvent_t> prof_events;
    bool prof_used[kProfSlots] = {};
    bool prof_valid = false;
    uint32_t prof_last = 0;
};

namespace {

mt_status fail(mt_ctx* c, mt_status st, const char* fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
        c->err = buf;
    }
    return st;
}

void bind_slot(mt_ctx* c, const RunSlot& r)
{
    c->d_row_tenant = r.d_row_tenant; c->d_row_rank = r.d_row_rank; c->d_hist_g = r.d_hist_g; c->d_row_src = r.d_row_src;
    c->d_pos_of = r.d_pos_of; c->d_perm = r.d_perm; c->d_M = r.d_M; c->d_off = r.d_off; c->d_tile_base = r.d_tile_base;
    for (int i = 0; i < kActBuffers; ++i) c->d_act[i] = r.d_act[i];
    c->d_logits = r.d_logits;
}

#define HIP_TRY(c, expr)                                                                    \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail((c), e_ == hipErrorOutOfMemory ? MT_ENOMEM : MT_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// ---- arena: first-fit free list, blocks merged on release -----------------------------
bool arena_alloc(mt_ctx* c, uint64_t len, uint64_t* off)
{
    len = round_up64(len, kArenaAlign);
    for (size_t i = 0; i < c->free_list.size(); ++i) {
        FreeBlock& b = c->free_list[i];
        if (b.len >= len) {
            *off = b.off;
            b.off += len; b.len -= len;
            if (b.len == 0) c->free_list.erase(c->free_list.begin() + (long)i);
            c->arena_used += len;
            return true;
        }
    }
    return false;
}

void arena_free(mt_ctx* c, uint64_t off, uint64_t len)
{
    len = round_up64(len, kArenaAlign);
    FreeBlock nb{off, len};
    auto it = std::lower_bound(c->free_list.begin(), c->free_list.end(), nb,
                               [](const FreeBlock& a, const FreeBlock& b) { return a.off < b.off; });
    it = c->free_list.insert(it, nb);
    if (it + 1 != c->free_list.end() && it->off + it->len == (it + 1)->off) { it->len += (it + 1)->len; c->free_list.erase(it + 1); }
    if (it != c->free_list.begin() && (it - 1)->off + (it - 1)->len == it->off) { (it - 1)->len += it->len; c->free_list.erase(it); }
    c->arena_used -= len;
}

// how an FC layer's column blocks are grouped into tiles (must match the device code)
uint32_t fc_groups(uint32_t n_pad, uint32_t split_k)
{
    const uint32_t nblk = n_pad / kBrickRows;
    const uint32_t split = split_k ? 1u : (nblk >= 3 ? 4u : nblk);
    return (nblk + split - 1) / split;
}
// ... and the rows of such a tile: 64 where the four waves stand side by side, else 32
uint32_t fc_tile_rows(uint32_t n_pad, uint32_t split_k)
{
    return (!split_k && n_pad / kBrickRows >= 3) ? kTileRows : kTileRows / 2;
}

// Bytes of LDS that the input rows of one row tile take (conv_img_kernel's frame): per sub-image the input rows of
// its output rows and one more above and below, a pixel slot left and right, pixels 16 bytes apart from cin
// elements (a padded three-channel pixel of 16 bytes stands alone).
uint64_t row_tile_frame_bytes(const LayerDev& L, uint32_t es, RowTiling r)
{
    const bool chunk_pixel = L.cin * es == 16;
    const uint32_t n_ih = (r.n_oh - 1) * L.stride + 3;
    return (uint64_t)r.ni * n_ih * (L.in_w + 2) * (L.cin * es + (chunk_pixel ? 0 : 16));
}

// Row tiling of a 3x3 convolution (0: none): the most output rows per tile, or the most whole small images (a power
// of two), whose input rows fit the frame.  Tiles of fewer than 128 pixels leave MFMA columns idle; the gathering
// kernels they replace move every input byte nine times through the texture path at a quarter of the rate of a
// contiguous load.
uint32_t choose_row_tiling(const LayerDev& L, uint32_t es)
{
    // (stride 2: a tile's frame is four times its output rows, its workgroups sit alone on their CUs with the
    // zeroing, the copy and the K loop in a row; measured slower than the gathers on every such layer of r18 and c4)
    if (L.stride != 1) return 0;
    const uint64_t budget = kConvFrameMaxBytes;
    const uint32_t kb = 32 / es, rpr = L.rows_per_req;
    if (L.ksize != 3 || L.pad != 1 || L.out_w == 0 || L.out_w > (uint32_t)kConvTileRows) return 0;
    if (L.cin % kb != 0 && L.cin * es != 16) return 0;
    const uint32_t H = rpr / L.out_w;
    for (uint32_t ni = 8; ni >= 2; ni >>= 1) {               // whole images side by side
        const RowTiling r{H, ni, 1};
        if (rpr * ni <= (uint32_t)kConvTileRows && row_tile_frame_bytes(L, es, r) <= budget) return pack_row_tiling(r);
    }
    for (uint32_t n_oh = std::min<uint32_t>(H, (uint32_t)kConvTileRows / L.out_w); n_oh >= 1; --n_oh) {
        const RowTiling r{n_oh, 1, (H + n_oh - 1) / n_oh};
        if (r.tpi < 65536 && row_tile_frame_bytes(L, es, r) <= budget) return pack_row_tiling(r);
    }
    return 0;
}

// The batcher's two words per layer of one tenant (see BatchArgs::facts).
void fill_facts(const mt_ctx* c, const HostTenant& ht, uint32_t (*w)[2])
{
    for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) w[l][0] = w[l][1] = 0;
    for (uint32_t l = 0; l < ht.n_layers; ++l) {
        const LayerDev& L = ht.layers[l].dev;
        if (L.kind == MT_FC) {
            w[l][0] = fc_groups(L.N_pad, c->fc_split_k) | (fc_tile_rows(L.N_pad, c->fc_split_k) == kTileRows ? 0u : 1u << 30);
            w[l][1] = L.N_pad;
        } else if (L.kind == MT_CONV2D) {
            w[l][0] = (L.N + kTileCols - 1) / kTileCols | 1u << 31;
            w[l][1] = conv_tile_rows(L.rows_per_req, L.row_tiles);
        }
    }
}

// What a tenant's device state is uploaded from, in one host block: the arena image
// (arena_len bytes), then its rows of the three device tables.
struct StageTail {
    LayerDev rows[MT_MAX_LAYERS];
    TenantDev td;
    uint32_t facts[MT_MAX_LAYERS][2];
};
size_t stage_tail_offset(uint64_t arena_len) { return (size_t)round_up64(arena_len, 256); }
size_t stage_bytes(uint64_t arena_len) { return stage_tail_offset(arena_len) + sizeof(StageTail); }

// A tenant's rows of the three device tables travel inside kernel arguments: the runtime copies
// those when the launch is enqueued, so the host may change its copy (a later placement of the same
// model at another arena offset) while this one is still queued behind earlier work.  An asynchronous
// copy from the host block would read it only when it executes.  Kernel arguments are limited to a
// few kilobytes, so the layer rows go in pieces of kLayerGroup layers; the tenant row goes with the
// last piece, after a fence: a tenant that the batcher sees has its layer rows in place.
struct RowsPiece {
    LayerDev rows[kLayerGroup];
    uint32_t facts[kLayerGroup][2];
    TenantDev td;
};
static_assert(sizeof(RowsPiece) <= 2048, "a piece of a tenant's table rows must fit kernel arguments");
__global__ void install_rows_kernel(RowsPiece piece, LayerDev* rows, uint32_t* facts, TenantDev* td)
{
    const uint32_t* src_rows = (const uint32_t*)piece.rows;
    for (uint32_t i = threadIdx.x; i < sizeof(piece.rows) / 4; i += blockDim.x) ((uint32_t*)rows)[i] = src_rows[i];
    const uint32_t* src_facts = &piece.facts[0][0];
    for (uint32_t i = threadIdx.x; i < sizeof(piece.facts) / 4; i += blockDim.x) facts[i] = src_facts[i];
    if (!td) return;
    __threadfence();
    __syncthreads();
    const uint32_t* src_td = (const uint32_t*)&piece.td;
    for (uint32_t i = threadIdx.x; i < sizeof(piece.td) / 4; i += blockDim.x) ((uint32_t*)td)[i] = src_td[i];
}

hipError_t install_rows(mt_ctx* c, uint32_t tenant, const StageTail& tail, hipStream_t s);

// Point the tenant's layer descriptors at arena block `off` and refresh the table rows in its stage.
void place_tenant(const mt_ctx* c, HostTenant& ht, uint64_t off, uint8_t* stage)
{
    ht.arena_off = off;
    StageTail* tail = (StageTail*)(stage + stage_tail_offset(ht.arena_len));
    *tail = StageTail{};
    for (uint32_t l = 0; l < ht.n_layers; ++l) {
        ht.layers[l].dev.w_off = off + ht.layers[l].w_rel;
        ht.layers[l].dev.b_off = off + ht.layers[l].b_rel;
        tail->rows[l] = ht.layers[l].dev;
    }
    tail->td = ht.dev; tail->td.registered = 1;
    fill_facts(c, ht, tail->facts);
}

hipError_t install_rows(mt_ctx* c, uint32_t tenant, const StageTail& tail, hipStream_t s)
{
    // a tenant that disappears (n_layers 0) loses its tenant row first, in the first piece
    const uint32_t n_pieces = tail.td.registered ? (tail.td.n_layers + kLayerGroup - 1) / kLayerGroup : MT_MAX_LAYERS / kLayerGroup;
    for (uint32_t g = 0; g < n_pieces; ++g) {
        RowsPiece piece;
        std::memcpy(piece.rows, tail.rows + g * kLayerGroup, sizeof piece.rows);
        std::memcpy(piece.facts, tail.facts + g * kLayerGroup, sizeof piece.facts);
        piece.td = tail.td;
        const bool with_td = tail.td.registered ? g + 1 == n_pieces : g == 0;
        hipLaunchKernelGGL(install_rows_kernel, dim3(1), dim3(256), 0, s, piece, c->d_layers + (size_t)tenant * MT_MAX_LAYERS + g * kLayerGroup,
                           c->d_facts + ((size_t)tenant * MT_MAX_LAYERS + g * kLayerGroup) * 2, with_td ? c->d_tenants + tenant : nullptr);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Copy a placed tenant's weights and table rows to the device: on `s` without waiting (the arena
// image in the stage must be pinned and is never changed again; the table rows are taken from the
// stage now, see install_rows_kernel), or synchronously.
hipError_t upload_tenant(mt_ctx* c, uint32_t tenant, const HostTenant& ht, const uint8_t* stage, hipStream_t s, bool async)
{
    const StageTail* tail = (const StageTail*)(stage + stage_tail_offset(ht.arena_len));
    hipError_t e = async ? hipMemcpyAsync(c->d_arena + ht.arena_off, stage, (size_t)ht.arena_len, hipMemcpyHostToDevice, s)
                         : hipMemcpy(c->d_arena + ht.arena_off, stage, (size_t)ht.arena_len, hipMemcpyHostToDevice);
    if (e != hipSuccess) return e;
    e = install_rows(c, tenant, *tail, async ? s : nullptr);          // behind the weights on the same stream
    if (e != hipSuccess) return e;
    if (!async) { e = hipStreamSynchronize(nullptr); if (e != hipSuccess) return e; }
    c->n_uploads++; c->upload_bytes += ht.arena_len;
    return hipSuccess;
}

// Take a tenant's model off the device: the batcher no longer sees it, its arena block is free.
hipError_t hide_tenant(mt_ctx* c, uint32_t tenant, hipStream_t s, bool async)
{
    const hipError_t e = install_rows(c, tenant, StageTail{}, async ? s : nullptr);
    if (e != hipSuccess || async) return e;
    return hipStreamSynchronize(nullptr);
}

// Find `len` bytes of arena.  In cache mode, models used least recently (and before `protect`)
// give way until the block fits; their stages stay in host memory.
bool make_room(mt_ctx* c, uint64_t len, uint64_t protect, hipStream_t s, bool async, uint64_t* off, hipError_t* err)
{
    *err = hipSuccess;
    while (!arena_alloc(c, len, off)) {
        if (!c->cache) return false;
        int victim = -1;
        for (uint32_t t = 0; t < c->cfg.max_tenants; ++t) {
            const HostTenant& h = c->tenants[t];
            if (h.registered && h.resident && h.last_use < protect && (victim < 0 || h.last_use < c->tenants[victim].last_use)) victim = (int)t;
        }
        if (victim < 0) return false;
        HostTenant& v = c->tenants[victim];
        if (!c->host_only) { *err = hide_tenant(c, (uint32_t)victim, s, async); if (*err != hipSuccess) return false; }
        arena_free(c, v.arena_off, v.arena_len);
        v.resident = false;
        c->n_evictions++;
    }
    return true;
}

void recompute_pool_fusion(mt_ctx* c)
{
    for (uint32_t l = 0; l + 1 < MT_MAX_LAYERS; ++l) {
        bool any = false, all = true;
        for (const HostTenant& t : c->tenants) {
            if (!t.registered || t.n_layers <= l + 1) continue;
            any = true;
            all = all && t.layers[l + 1].dev.kind == MT_GAP && t.layers[l].dev.pool_fill != 0;
        }
        c->pool_fused[l] = any && all && !c->no_fused_pool;
    }
}

void recompute_bounds(mt_ctx* c)
{
    c->n_layer_slots = 0;
    c->max_in_len = 0; c->max_image_pixels = 0;
    c->fc_first_chunked = true; c->any_conv_first = c->any_fc_first = false;
    for (uint32_t& m : c->list_mask) m = 0;
    c->max_reg_classes = 0; c->min_reg_classes = 0xffffffffu; c->sum_macs = 0.0;
    for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
        c->has_gap[l] = 0; c->has_image_ops[l] = 0; c->image_op_fill[l] = 0; c->min_conv_k[l] = 0xffffffffu; c->min_fc_k[l] = 0xffffffffu; c->max_conv_cb[l] = 0; c->conv_quad[l] = true; c->conv_uniform[l] = true; c->pool_fused[l] = false; c->conv_img_lds[l] = 1; c->conv_img_two[l] = -1;
        for (int k = 0; k < kListKinds; ++k) { c->max_rpr[k][l] = c->max_nt[k][l] = 0; c->sum_nt[k][l] = 0; }
        c->max_fc_per64[l] = 0; c->max_fc_per64_sk[l] = 0; c->sum_nt_sk[l] = 0; c->max_big_blocks[l] = 0;
    }
    for (const HostTenant& t : c->tenants) {
        if (!t.registered) continue;
        c->n_layer_slots = std::max(c->n_layer_slots, t.n_layers);
        c->max_in_len = std::max(c->max_in_len, t.dev.in_len);
        c->max_reg_classes = std::max(c->max_reg_classes, t.dev.n_classes);
        c->min_reg_classes = std::min(c->min_reg_classes, t.dev.n_classes);
        if (t.dev.in_layout == kLayoutBricks) {
            c->any_fc_first = true;
            if ((t.dev.in_len * c->elem_size) % 16) c->fc_first_chunked = false;
        } else {
            c->any_conv_first = true;
            c->max_image_pixels = std::max(c->max_image_pixels, t.dev.in_len / (t.dev.in_cin ? t.dev.in_cin : (uint32_t)kChanPad));
        }
        for (uint32_t l = 0; l < t.n_layers; ++l) {
            const LayerDev& L = t.layers[l].dev;
            if (L.kind == kKindNone) continue;
            if (L.kind == MT_GAP) { c->has_gap[l] = 1; continue; }
            if (L.kind == MT_MAXPOOL || L.kind == MT_ADD) { c->has_image_ops[l] = 1; c->image_op_fill[l] = std::max(c->image_op_fill[l], L.out_fill); continue; }
            const int k = L.kind == MT_FC ? 0 : 1;
            c->sum_macs += (double)L.k_valid * L.N * L.rows_per_req;
            c->list_mask[l / kLayerGroup] |= 1u << (k * kLayerGroup + l % kLayerGroup);
            const uint32_t nt = k == 0 ? fc_groups(L.N_pad, c->fc_split_k) : (L.N + kTileCols - 1) / kTileCols;
            c->max_rpr[k][l] = std::max(c->max_rpr[k][l], k == 1 ? conv_tile_rows(L.rows_per_req, L.row_tiles) : L.rows_per_req);
            c->max_nt[k][l] = std::max(c->max_nt[k][l], nt);
            c->sum_nt[k][l] += nt;
            if (k == 0) {
                c->min_fc_k[l] = std::min(c->min_fc_k[l], L.K);
                c->max_fc_per64[l] = std::max(c->max_fc_per64[l], nt * (kTileRows / fc_tile_rows(L.N_pad, c->fc_split_k)));
                const uint32_t nt_sk = fc_groups(L.N_pad, 1);
                c->sum_nt_sk[l] += nt_sk;
                c->max_fc_per64_sk[l] = std::max(c->max_fc_per64_sk[l], nt_sk * (kTileRows / fc_tile_rows(L.N_pad, 1)));
            }
            if (k == 1) {
                c->min_conv_k[l] = std::min(c->min_conv_k[l], L.k_valid);
                c->max_conv_cb[l] = std::max(c->max_conv_cb[l], std::min<uint32_t>(L.N_pad / kBrickRows, kTileCols / kBrickRows));
                if (L.cin % (4 * (16 / c->elem_size))) c->conv_quad[l] = false;
                if (L.cin % (2 * (16 / c->elem_size)) || L.ksize * L.ksize > 64) c->conv_uniform[l] = false;
                // frame of one tile of the LDS-resident-input kernel (conv_img_kernel), which serves the layer index
                // when every tenant's layer is row-tiled
                const bool chunk_pixel = L.cin * c->elem_size == 16;            // a pixel is one 16-byte chunk: two taps per k step, no padding
                const uint64_t frame = L.row_tiles ? row_tile_frame_bytes(L, c->elem_size, unpack_row_tiling(L.row_tiles)) : 0;
                if (c->conv_img_two[l] < 0) c->conv_img_two[l] = chunk_pixel;
                if (frame == 0 || c->conv_img_lds[l] == 0 || c->conv_img_two[l] != (int)chunk_pixel) c->conv_img_lds[l] = 0;
                else c->conv_img_lds[l] = std::max<uint32_t>(c->conv_img_lds[l], (uint32_t)frame);
            }
            if (k == 0 && L.N_pad >= (uint32_t)kBigMinCols && l < (uint32_t)kBigMaxLayer) {      // may be served with big tiles when it gets enough rows
                c->list_mask[l / kLayerGroup] |= 1u << (2 * kLayerGroup + l % kLayerGroup);
                c->max_nt[2][l] = std::max(c->max_nt[2][l], (L.N_pad + kBigTile - 1) / kBigTile);
                if (big_remainder_split_k(L.N_pad)) c->max_big_blocks[l] = std::max(c->max_big_blocks[l], L.N_pad / kBrickRows);
            }
        }
    }
}

// Upper bound of the number of tiles of one list over any split of R rows among tenants.
uint64_t tile_bound(const mt_ctx* c, int kind, uint32_t l, uint64_t R, bool split_k = false, bool big_enabled = false)
{
    if (c->max_nt[kind][l] == 0) return 0;
    // streaming tiles of a run with big tiles: the tenants that big tiles serve (at most R / kBigMinRows of them) leave
    // at most kBigRemRows rows each, in narrow layers tiled 32 rows and one column block at a time
    if (kind == 0 && big_enabled && !split_k)
        return tile_bound(c, 0, l, R) + (R / kBigMinRows) * (kBigRemRows / kBrickRows) * c->max_big_blocks[l];
    if (kind == 2)      // big FC tiles: only tenants with >= kBigMinRows rows; sum ceil(M_t/256) <= R/256 + R/kBigMinRows
        return R < (uint64_t)kBigMinBatch ? 0 : (uint64_t)c->max_nt[2][l] * (R / kBigTile + R / kBigMinRows);
    // sum over tenants of ceil(M_t / rows_t) * groups_t <= R * max(groups_t / rows_t) + sum(groups_t)
    if (kind == 0 && split_k) return ((uint64_t)c->max_fc_per64_sk[l] * R + kTileRows - 1) / kTileRows + c->sum_nt_sk[l];
    if (kind == 0) return ((uint64_t)c->max_fc_per64[l] * R + kTileRows - 1) / kTileRows + c->sum_nt[0][l];
    return (uint64_t)c->max_nt[kind][l] * (R * c->max_rpr[kind][l] / kConvTileRows) + c->sum_nt[kind][l];
}

// Tile shape of the FC layers of a run over R rows.  When no layer index can have more than
// kSplitKMaxTiles ordinary tiles the launches fill a fraction of the chip and their duration is one
// wave's walk through K (on the fp32 mix of four small models: 13-16 us per layer, most of it the
// fp32 MFMAs of a 256- or 512-step K loop in a single wave).  Such runs take tiles of one column
// block whose four waves split K (and 32 rows): four times the workgroups, a quarter of the walk.
constexpr uint64_t kSplitKMaxTiles = 128;
bool run_split_k(const mt_ctx* c, uint64_t R)
{
    if (c->fc_split_k) return true;
    if (c->no_auto_split_k) return false;
    // at most min(R, registered models) tenants have rows, each with one ragged row tile per column group
    const uint64_t active = std::min<uint64_t>(R, c->n_registered);
    uint64_t most = 0;
    for (uint32_t l = 0; l < c->n_layer_slots; ++l)
        most = std::max(most, ((uint64_t)c->max_fc_per64[l] * R + kTileRows - 1) / kTileRows + active * c->max_nt[0][l]);
    return most > 0 && most <= kSplitKMaxTiles;
}

// Most classes a last layer may have for its FC tiles to finish their rows themselves (softmax,
// argmax, outputs) in a run: one column block (32), or a whole tile of four (128) where the run's
// tiles are not single column blocks; 0: the head kernel does every row.
uint32_t fused_head_classes(const mt_ctx* c, bool split_k)
{
    if (c->no_fused_head) return 0;
    return split_k ? (uint32_t)kBrickRows : (uint32_t)kTileCols;
}

// ---- validation of a layer chain; fills dev layouts (without arena offsets) -------------
mt_status plan_model(mt_ctx* c, const mt_layer_spec* specs, uint32_t n_layers, HostTenant* out)
{
    if (n_layers == 0 || n_layers > MT_MAX_LAYERS)
        return fail(c, MT_EUNSUPPORTED, "a model needs 1..%d layers, got %u", MT_MAX_LAYERS, n_layers);
    const uint32_t es = c->elem_size;
    out->n_layers = n_layers;
    out->dev = TenantDev{};
    // Values: 0 is the request, l + 1 the output of layer l.  A layer reads the value before it unless
    // its spec names another one (skip connections); shape[] is what every value looks like.
    struct Shape { uint32_t h, w, ch, len; bool image; };
    Shape shape[MT_MAX_LAYERS + 1] = {};
    uint32_t src_of[MT_MAX_LAYERS] = {}, src2_of[MT_MAX_LAYERS] = {}, last_use[MT_MAX_LAYERS + 1] = {};
    for (uint32_t l = 0; l < n_layers; ++l) {
        const mt_layer_spec& s = specs[l];
        HostLayer& hl = out->layers[l];
        hl.spec = s;
        LayerDev d{};
        d.kind = s.kind; d.act = s.act; d.is_last = (l == n_layers - 1);
        d.stride = 1; d.out_w = 1; d.rows_per_req = 1;
        if (s.act > MT_ACT_GELU) return fail(c, MT_EUNSUPPORTED, "layer %u: activation %u is not in the supported set", l, s.act);
        if (d.is_last && s.act != MT_ACT_NONE) return fail(c, MT_EUNSUPPORTED, "layer %u: the last layer yields logits and takes no activation", l);
        if (s.src > l || s.src2 > l) return fail(c, MT_EUNSUPPORTED, "layer %u: a layer can only read outputs of earlier layers", l);
        if (s.src2 != 0 && s.kind != MT_ADD) return fail(c, MT_EUNSUPPORTED, "layer %u: only an addition takes a second source", l);
        const uint32_t src = s.src ? s.src : l;              // value read: the named one, else the one before this layer
        src_of[l] = src; last_use[src] = l;
        const Shape in = shape[src];                         // (undefined for the request: the first layer defines it)
        const bool first = l == 0;
        const bool image_kind = s.kind == MT_CONV2D || s.kind == MT_GAP || s.kind == MT_MAXPOOL || s.kind == MT_ADD;
        if (image_kind) {
            if (s.in_features == 0 || s.in_h == 0 || s.in_w == 0) return fail(c, MT_EINVAL, "layer %u: zero-sized image", l);
            if ((uint64_t)s.in_h * s.in_w * s.in_features > 0x7fffffffu) return fail(c, MT_EUNSUPPORTED, "layer %u: image too large", l);
            if (!first && (!in.image || in.h != s.in_h || in.w != s.in_w || in.ch != s.in_features))
                return fail(c, MT_EUNSUPPORTED, "layer %u takes a %ux%ux%u image but its source yields %s of %u values", l, s.in_h, s.in_w, s.in_features,
                            in.image ? "another image" : "a vector", in.len);
            if (d.is_last) return fail(c, MT_EUNSUPPORTED, "layer %u: the last layer must be fully connected", l);
        }
        Shape o{};
        if (s.kind == MT_FC) {
            if (s.in_features == 0 || s.out_features == 0) return fail(c, MT_EINVAL, "layer %u: zero-sized FC", l);
            if (!first && in.image)
                return fail(c, MT_EUNSUPPORTED, "layer %u: an FC layer cannot read an image directly; pool first", l);
            if (!first && in.len != s.in_features) return fail(c, MT_EUNSUPPORTED, "layer %u takes %u values but its source yields %u", l, s.in_features, in.len);
            d.K = round_up(s.in_features, kWidthAlign); d.k_valid = s.in_features; d.N = s.out_features;
            d.N_pad = round_up(s.out_features, d.is_last ? kBrickRows : kWidthAlign);
            d.out_len = s.out_features;
            hl.w_bytes = (uint64_t)d.N_pad * d.K * es; hl.b_bytes = (uint64_t)d.N_pad * 4;
            o = Shape{1, 1, s.out_features, s.out_features, false};
        } else if (s.kind == MT_CONV2D) {
            if (s.kh != s.kw || (s.kh != 1 && s.kh != 3 && s.kh != 7) || s.pad != (s.kh - 1) / 2 || (s.stride != 1 && s.stride != 2))
                return fail(c, MT_EUNSUPPORTED, "layer %u: convolutions are 1x1, 3x3 or 7x7 with pad (k - 1) / 2 and stride 1 or 2", l);
            if (s.out_features == 0) return fail(c, MT_EINVAL, "layer %u: zero-sized conv", l);
            if (s.out_features % kChanPad) return fail(c, MT_EUNSUPPORTED, "layer %u: conv output channels must be a multiple of %d", l, kChanPad);
            if (!first && s.in_features % kChanPad) return fail(c, MT_EUNSUPPORTED, "layer %u: conv input channels must be a multiple of %d past the first layer", l, kChanPad);
            const uint32_t oh = (s.in_h + 2 * s.pad - s.kh) / s.stride + 1, ow = (s.in_w + 2 * s.pad - s.kw) / s.stride + 1;
            d.cin = round_up(s.in_features, kChanPad);
            d.in_h = s.in_h; d.in_w = s.in_w; d.stride = s.stride; d.out_w = ow; d.ksize = s.kh; d.pad = s.pad;
            d.rows_per_req = oh * ow;
            d.K = round_up(s.kh * s.kw * d.cin, kWidthAlign); d.k_valid = s.kh * s.kw * d.cin; d.N = s.out_features; d.N_pad = round_up(s.out_features, kBrickRows);
            d.out_len = oh * ow * s.out_features;
            hl.w_bytes = (uint64_t)d.N_pad * d.K * es; hl.b_bytes = (uint64_t)d.N_pad * 4;
            o = Shape{oh, ow, s.out_features, d.out_len, true};
        } else if (s.kind == MT_GAP) {
            if (s.out_features != s.in_features || s.act != MT_ACT_NONE) return fail(c, MT_EUNSUPPORTED, "layer %u: pooling keeps the channel count and has no activation", l);
            if (first) return fail(c, MT_EUNSUPPORTED, "layer %u: pooling cannot be the first layer", l);
            d.cin = s.in_features; d.in_h = s.in_h; d.in_w = s.in_w; d.N = s.in_features; d.N_pad = s.in_features;
            d.out_len = s.in_features;
            hl.w_bytes = hl.b_bytes = 0;
            o = Shape{1, 1, s.in_features, s.in_features, false};
        } else if (s.kind == MT_MAXPOOL) {
            if (s.kh != s.kw || (s.kh != 2 && s.kh != 3) || s.pad > 1 || s.pad >= s.kh || (s.stride != 1 && s.stride != 2))
                return fail(c, MT_EUNSUPPORTED, "layer %u: max-pooling takes 2x2 or 3x3 windows, pad 0 or 1, stride 1 or 2", l);
            if (s.out_features != s.in_features || s.act != MT_ACT_NONE) return fail(c, MT_EUNSUPPORTED, "layer %u: pooling keeps the channel count and has no activation", l);
            if (first) return fail(c, MT_EUNSUPPORTED, "layer %u: pooling cannot be the first layer", l);
            if (s.in_h + 2 * s.pad < s.kh || s.in_w + 2 * s.pad < s.kw) return fail(c, MT_EUNSUPPORTED, "layer %u: the window exceeds the image", l);
            const uint32_t oh = (s.in_h + 2 * s.pad - s.kh) / s.stride + 1, ow = (s.in_w + 2 * s.pad - s.kw) / s.stride + 1;
            d.cin = s.in_features; d.in_h = s.in_h; d.in_w = s.in_w; d.stride = s.stride; d.out_w = ow; d.ksize = s.kh; d.pad = s.pad;
            d.rows_per_req = oh * ow; d.N = s.in_features; d.N_pad = s.in_features;
            d.out_len = oh * ow * s.in_features;
            hl.w_bytes = hl.b_bytes = 0;
            o = Shape{oh, ow, s.in_features, d.out_len, true};
        } else if (s.kind == MT_ADD) {
            if (first || s.src2 == 0) return fail(c, MT_EUNSUPPORTED, "layer %u: an addition names its second source and cannot be the first layer", l);
            if (s.out_features != s.in_features) return fail(c, MT_EUNSUPPORTED, "layer %u: an addition keeps the channel count", l);
            const Shape in2 = shape[s.src2];
            if (!in2.image || in2.h != s.in_h || in2.w != s.in_w || in2.ch != s.in_features)
                return fail(c, MT_EUNSUPPORTED, "layer %u: the second source is not a %ux%ux%u image", l, s.in_h, s.in_w, s.in_features);
            src2_of[l] = s.src2; last_use[s.src2] = l;
            d.cin = s.in_features; d.in_h = s.in_h; d.in_w = s.in_w; d.out_w = s.in_w; d.rows_per_req = s.in_h * s.in_w;
            d.N = s.in_features; d.N_pad = s.in_features;
            d.out_len = s.in_h * s.in_w * s.in_features;
            hl.w_bytes = hl.b_bytes = 0;
            o = Shape{s.in_h, s.in_w, s.in_features, d.out_len, true};
        } else {
            return fail(c, MT_EUNSUPPORTED, "layer %u: kind %u is not in the supported set", l, s.kind);
        }
        if (s.kind != MT_FC && s.in_features % kChanPad && !(first && s.kind == MT_CONV2D))
            return fail(c, MT_EUNSUPPORTED, "layer %u: image channels must be a multiple of %d", l, kChanPad);
        shape[l + 1] = o;
        d.out_fill = round_up(d.out_len, kWidthAlign);
        if (first) {
            const uint32_t in_len = s.kind == MT_FC ? s.in_features : s.in_h * s.in_w * s.in_features;
            out->dev.in_len = in_len;
            uint32_t staged = in_len;
            if (s.kind == MT_CONV2D && d.cin != s.in_features) {
                out->dev.in_cin = s.in_features; out->dev.in_cin_pad = d.cin;
                staged = s.in_h * s.in_w * d.cin;
            }
            out->dev.in_fill = round_up(staged, kWidthAlign);
            out->dev.in_layout = s.kind == MT_FC ? kLayoutBricks : kLayoutRows;
            if (out->dev.in_fill > c->S) return fail(c, MT_EUNSUPPORTED, "input of %u values exceeds max_width", in_len);
        }
        if (!d.is_last && d.out_fill > c->S) return fail(c, MT_EUNSUPPORTED, "layer %u output of %u values exceeds max_width", l, d.out_len);
        if (s.kind == MT_FC && d.K > c->S) return fail(c, MT_EUNSUPPORTED, "layer %u fan-in %u exceeds max_width", l, s.in_features);
        if (d.is_last && d.out_len > c->cfg.max_classes) return fail(c, MT_EUNSUPPORTED, "%u classes exceed max_classes", d.out_len);
        hl.dev = d;
    }
    out->dev.n_layers = n_layers;
    out->dev.n_classes = shape[n_layers].len;

    // A convolution whose output goes to a global average pool and nowhere else can pool by itself
    // when every image lies inside one wave's pixel blocks; its input then has to outlive the pooling
    // layer's index, because the pooled activation is written where that layer would have written it.
    for (uint32_t l = 1; l < n_layers; ++l) {
        if (out->layers[l].dev.kind != MT_GAP || src_of[l] != l || out->layers[l - 1].dev.kind != MT_CONV2D) continue;
        LayerDev& conv = out->layers[l - 1].dev;
        last_use[src_of[l - 1]] = std::max(last_use[src_of[l - 1]], l);
        if (conv.N % kWidthAlign == 0 && (conv.rows_per_req == kBrickRows || conv.rows_per_req == 2 * kBrickRows) && last_use[l] == l)
            conv.pool_fill = round_up(out->layers[l].dev.N, kWidthAlign);
    }
    // A convolution whose output goes to a residual addition right behind it and nowhere else adds the
    // other operand itself (rounding its own output first, as the addition would have read it) and writes
    // what the addition would have written; the addition's index is then empty for this tenant.
    bool fused_add[MT_MAX_LAYERS] = {};
    for (uint32_t l = 1; l < n_layers && !c->no_fused_add; ++l) {
        const LayerDev& add = out->layers[l].dev;
        LayerDev& conv = out->layers[l - 1].dev;
        if (add.kind != MT_ADD || conv.kind != MT_CONV2D || conv.pool_fill || last_use[l] != l) continue;
        if (src_of[l] != l && src2_of[l] != l) continue;                            // neither operand is that convolution's output
        const uint32_t other = src_of[l] == l ? src2_of[l] : src_of[l];
        if (other == l) continue;                                                   // x + x
        fused_add[l] = true;
        conv.fuse_add = 1 + add.act;
        src2_of[l - 1] = other;                                                     // the convolution reads it now
    }
    // Activation buffers: the request sits in buffer 0; a layer writes the lowest-numbered buffer that
    // holds no value still to be read at or after its index (its own inputs included).  A plain chain
    // alternates between two buffers.
    uint32_t buf_of[MT_MAX_LAYERS + 1] = {};
    out->act_buffers = 1;
    for (uint32_t l = 0; l < n_layers; ++l) {
        LayerDev& d = out->layers[l].dev;
        d.in_buf = buf_of[src_of[l]];
        d.in2_buf = (d.kind == MT_ADD || d.fuse_add) ? buf_of[src2_of[l]] : 0;
        if (d.is_last) break;                                 // logits have a buffer of their own
        if (fused_add[l]) {                                   // the sum is where the convolution before wrote it
            buf_of[l + 1] = buf_of[l]; d.out_buf = buf_of[l]; d.kind = kKindNone;
            continue;
        }
        uint32_t pick = kActBuffers;
        for (uint32_t b = 0; b < (uint32_t)kActBuffers && pick == (uint32_t)kActBuffers; ++b) {
            bool busy = false;
            for (uint32_t v = 0; v <= l; ++v) busy = busy || (buf_of[v] == b && last_use[v] >= l);
            if (!busy) pick = b;
        }
        if (pick == (uint32_t)kActBuffers)
            return fail(c, MT_EUNSUPPORTED, "layer %u: more than %d layer outputs are alive at once", l, kActBuffers);
        buf_of[l + 1] = pick; d.out_buf = pick;
        out->act_buffers = std::max(out->act_buffers, pick + 1);
    }
    for (uint32_t l = 0; l + 1 < n_layers; ++l)
        if (out->layers[l].dev.pool_fill) out->layers[l].dev.pool_buf = out->layers[l + 1].dev.out_buf;
    for (uint32_t l = 0; l < n_layers && !c->no_conv_img; ++l) {
        LayerDev& d = out->layers[l].dev;
        if (d.kind == MT_CONV2D && !d.pool_fill) d.row_tiles = choose_row_tiling(d, es);
    }
    return MT_OK;
}

// Arena image of one layer: bricks[n_block][k_block][lane][EPC] with lane = row + 32*half (zero
// rows and columns as padding), the order in which a wavefront consumes MFMA operands.  The
// reduction index k is the fan-in for FC; for conv the filters [Co][Ci][kh][kw] are read as
// k = (kh*ksize + kw) * ci_padded + ci, so that a GEMM k index walks the NHWC input contiguously.
template <typename T>
void pack_weights(const HostLayer& hl, const void* w_src, uint8_t* dst)
{
    const LayerDev& d = hl.dev;
    const T* src = (const T*)w_src;
    T* out = (T*)dst;
    std::memset(dst, 0, hl.w_bytes);
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t nKB = d.K / KB;
    auto put = [&](uint32_t n, uint32_t k, T v) {
        const uint32_t nb = n / kBrickRows, i = n % kBrickRows, kb = k / KB, h = (k % KB) / EPC, e = k % EPC;
        out[(((size_t)nb * nKB + kb) * 64 + i + 32 * h) * EPC + e] = v;
    };
    if (d.kind == MT_FC) {
        const uint32_t K = hl.spec.in_features;
        for (uint32_t n = 0; n < d.N; ++n)
            for (uint32_t k = 0; k < K; ++k) put(n, k, src[(size_t)n * K + k]);
    } else {
        const uint32_t Ci = hl.spec.in_features, ks = d.ksize;
        for (uint32_t co = 0; co < d.N; ++co)
            for (uint32_t ci = 0; ci < Ci; ++ci)
                for (uint32_t kh = 0; kh < ks; ++kh)
                    for (uint32_t kw = 0; kw < ks; ++kw)
                        put(co, (kh * ks + kw) * d.cin + ci, src[(((size_t)co * Ci + ci) * ks + kh) * ks + kw]);
    }
}

// ---- batch normalisation folded into the convolution in front of it ---------------------------
// Nearest-even rounding of a double to bfloat16 (bit pattern), done on the bits of the double so
// that the value is rounded once: sign, 8 exponent bits, 7 fraction bits; results below 2^-126
// are subnormal (spacing 2^-133), results beyond the largest finite value become infinity.
uint16_t bf16_bits_from_double(double x)
{
    uint64_t u; std::memcpy(&u, &x, 8);
    const uint16_t sign = (uint16_t)((u >> 63) << 15);
    const int64_t e = (int64_t)((u >> 52) & 0x7ff) - 1023;
    const uint64_t frac = u & ((1ull << 52) - 1);
    if (((u >> 52) & 0x7ff) == 0x7ff) return (uint16_t)(sign | 0x7f80 | (frac ? 0x40 : 0));       // infinity / NaN
    if (((u >> 52) & 0x7ff) == 0 || e < -140) return sign;                                        // zero, or far below half the smallest subnormal
    const uint64_t mant = (1ull << 52) | frac;                       // value = mant * 2^(e - 52)
    // keep 7 fraction bits of a normal result; a result below 2^-126 keeps fewer: its last place is 2^-133
    const int shift = e >= -126 ? 45 : (int)(45 + (-126 - e));
    uint64_t kept = mant >> shift;
    const uint64_t rem = mant & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (kept & 1))) ++kept;
    if (e >= -126) {
        int64_t be = e + 127;                                        // biased exponent; kept holds the hidden bit (128..256)
        if (kept == 256) { kept = 128; ++be; }
        if (be >= 255) return (uint16_t)(sign | 0x7f80);
        return (uint16_t)(sign | (uint16_t)(be << 7) | (uint16_t)(kept - 128));
    }
    return (uint16_t)(sign | (uint16_t)kept);                        // subnormal; kept == 128 is the smallest normal number
}

// W' = round(W * s), b' = float((b - mean) * s + beta) with s = gamma / sqrt(var + eps), per output
// channel, in double precision, each rounded once (no fused multiply-add: the products are rounded
// to double before the sums).  `w` holds the layer's filters [Co][per] in the context's element
// type and is folded in place; `b` its fp32 bias [Co].
#pragma clang fp contract(off)
void fold_batchnorm(uint32_t elem_size, void* w, float* b, uint32_t Co, size_t per, const float* bn, double eps)
{
    const float *gamma = bn, *beta = bn + Co, *mean = bn + 2 * (size_t)Co, *var = bn + 3 * (size_t)Co;
    for (uint32_t c = 0; c < Co; ++c) {
        const double s = (double)gamma[c] / std::sqrt((double)var[c] + eps);
        if (elem_size == 2) {
            uint16_t* row = (uint16_t*)w + c * per;
            for (size_t i = 0; i < per; ++i) {
                const uint32_t wide = (uint32_t)row[i] << 16;
                float f; std::memcpy(&f, &wide, 4);
                const double prod = (double)f * s;
                row[i] = bf16_bits_from_double(prod);
            }
        } else {
            float* row = (float*)w + c * per;
            for (size_t i = 0; i < per; ++i) { const double prod = (double)row[i] * s; row[i] = (float)prod; }
        }
        const double shifted = ((double)b[c] - (double)mean[c]) * s;
        const double sum = shifted + (double)beta[c];
        b[c] = (float)sum;
    }
}

// Offsets of a planned model's layers inside its arena block; returns the block's length.
uint64_t layout_model(HostTenant* ht)
{
    uint64_t total = 0;
    for (uint32_t l = 0; l < ht->n_layers; ++l) {
        HostLayer& hl = ht->layers[l];
        hl.w_rel = total; total += round_up64(hl.w_bytes, kArenaAlign);
        hl.b_rel = total; total += round_up64(hl.b_bytes, kArenaAlign);
    }
    if (total == 0) total = kArenaAlign;
    ht->arena_len = total;
    return total;
}

}  // namespace

extern "C" {

const char* mt_version(void) { return "mt 0.1 gfx950"; }

const char* mt_last_error(const mt_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

mt_status mt_create(mt_ctx** out, const mt_config* cfg)
{
    if (!out || !cfg) return MT_EINVAL;
    *out = nullptr;
    if (cfg->max_tenants == 0 || cfg->max_tenants > kMaxTenants || cfg->max_requests == 0 || cfg->max_width == 0 ||
        cfg->max_classes == 0 || cfg->arena_bytes == 0 || cfg->dtype > MT_BF16 || cfg->run_slots > kMaxRunSlots)
        return MT_EINVAL;
    if ((uint64_t)cfg->max_requests * 4096 > (1ull << 31)) return MT_EINVAL;   // row indices and GEMM row counts stay in 32 bits
    mt_ctx* c = new (std::nothrow) mt_ctx;
    if (!c) return MT_ENOMEM;
    c->cfg = *cfg;
    c->host_only = cfg->device < 0;
    c->elem_size = cfg->dtype == MT_BF16 ? 2 : 4;
    c->S = round_up(cfg->max_width, kWidthAlign);
    c->C_pad = round_up(cfg->max_classes, 4);
    c->P_cap = round_up(cfg->max_requests, kBrickRows) + kBrickRows * std::min(cfg->max_tenants, cfg->max_requests);
    if (const char* e = getenv("MT_FC_SPLIT_K")) c->fc_split_k = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_AUTO_SPLIT_K")) c->no_auto_split_k = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_FUSED_GATHER")) c->no_fused_gather = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_FUSED_HEAD")) c->no_fused_head = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_FUSED_POOL")) c->no_fused_pool = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_CONV_IMG")) c->no_conv_img = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_FUSED_ADD")) c->no_fused_add = atoi(e) != 0;
    if (const char* e = getenv("MT_BIG_WALK")) c->big_walk = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_CONV_LOADERS")) c->no_conv_loaders = atoi(e) != 0;
    if (const char* e = getenv("MT_NO_CONV_UNIFORM")) c->no_conv_uniform = atoi(e) != 0;
    if (const char* e = getenv("MT_BIG_MIN_TILES")) c->big_min_tiles = (uint32_t)std::max(1, atoi(e));
    c->cache = cfg->cache != 0;
    c->tenants.resize(cfg->max_tenants);
    c->cfg.arena_bytes = cfg->arena_bytes / kArenaAlign * kArenaAlign;
    c->free_list.push_back(FreeBlock{0, c->cfg.arena_bytes});
    *out = c;
    if (c->host_only) return MT_OK;

    auto bail = [&](mt_status st) { mt_destroy(c); *out = nullptr; return st; };
#define CREATE_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { fprintf(stderr, "mt_create: %s: %s\n", #expr, hipGetErrorString(e_)); return bail(e_ == hipErrorOutOfMemory ? MT_ENOMEM : MT_EDEVICE); } } while (0)
    CREATE_TRY(hipSetDevice(cfg->device));
    {
        int cus = 0;
        CREATE_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device));
        c->n_cus = (uint32_t)std::max(cus, 8) / 8 * 8;
    }
    CREATE_TRY(prepare_conv(cfg->dtype));
    const uint64_t R = cfg->max_requests, T = cfg->max_tenants;
    CREATE_TRY(hipMalloc((void**)&c->d_arena, c->cfg.arena_bytes));
    CREATE_TRY(hipMalloc((void**)&c->d_tenants, T * sizeof(TenantDev)));
    CREATE_TRY(hipMemset(c->d_tenants, 0, T * sizeof(TenantDev)));
    CREATE_TRY(hipMalloc((void**)&c->d_layers, T * MT_MAX_LAYERS * sizeof(LayerDev)));
    CREATE_TRY(hipMemset(c->d_layers, 0, T * MT_MAX_LAYERS * sizeof(LayerDev)));
    CREATE_TRY(hipMalloc((void**)&c->d_facts, 2 * MT_MAX_LAYERS * T * 4));
    CREATE_TRY(hipMemset(c->d_facts, 0, 2 * MT_MAX_LAYERS * T * 4));
    CREATE_TRY(hipMalloc((void**)&c->d_served, T * 16));
    CREATE_TRY(hipMemset(c->d_served, 0, T * 16));
    CREATE_TRY(hipMalloc(&c->d_zeros, 256));
    CREATE_TRY(hipMemset(c->d_zeros, 0, 256));
    c->slots.resize(std::max<uint32_t>(1, cfg->run_slots));
    for (RunSlot& r : c->slots) {          // (a failed allocation leaves the rest null; mt_destroy frees what exists)
        CREATE_TRY(hipMalloc((void**)&r.d_row_tenant, R * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_row_rank, R * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_hist_g, kHistEntries * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_row_src, R * sizeof(void*)));
        CREATE_TRY(hipMalloc((void**)&r.d_pos_of, R * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_perm, (uint64_t)c->P_cap * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_M, T * 4));
        CREATE_TRY(hipMemset(r.d_M, 0, T * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_off, (T + 1) * 4));
        CREATE_TRY(hipMalloc((void**)&r.d_tile_base, (kListKinds * MT_MAX_LAYERS * (T + 1) + 1) * 4));
        CREATE_TRY(hipMemset(r.d_tile_base, 0, (kListKinds * MT_MAX_LAYERS * (T + 1) + 1) * 4));
        for (uint32_t i = 0; i < c->act_buffers; ++i) {
            CREATE_TRY(hipMalloc(&r.d_act[i], (uint64_t)c->P_cap * c->S * c->elem_size));
        }
        CREATE_TRY(hipMalloc((void**)&r.d_logits, (uint64_t)c->P_cap * c->C_pad * 4));
        CREATE_TRY(hipEventCreateWithFlags(&r.done, hipEventDisableTiming));
    }
    bind_slot(c, c->slots[0]);
    CREATE_TRY(hipGetSymbolAddress((void**)&c->static_scratch, HIP_SYMBOL(scratch)));      // this device's copy of the array
    CREATE_TRY(hipEventCreateWithFlags(&c->static_slot.done, hipEventDisableTiming));
    if (c->cache) {
        CREATE_TRY(hipEventCreateWithFlags(&c->cache_event, hipEventDisableTiming));
    }
    for (uint32_t i = 0; i < kSegSlots; ++i) {
        CREATE_TRY(hipHostMalloc((void**)&c->h_segs[i], R * sizeof(Segment), hipHostMallocMapped));
        CREATE_TRY(hipHostGetDevicePointer((void**)&c->d_segs[i], c->h_segs[i], 0));
        CREATE_TRY(hipEventCreateWithFlags(&c->seg_event[i], hipEventDisableTiming));
    }
#undef CREATE_TRY
    return MT_OK;
}

mt_status mt_destroy(mt_ctx* c)
{
    if (!c) return MT_EINVAL;
    if (!c->host_only) {
        (void)hipSetDevice(c->cfg.device);
        (void)hipDeviceSynchronize();
        void* bufs[] = {c->d_arena, c->d_tenants, c->d_layers, c->d_facts, c->d_served, c->d_zeros};
        for (void* p : bufs) if (p) (void)hipFree(p);
        for (RunSlot& r : c->slots) {
            void* rb[] = {r.d_row_tenant, r.d_row_rank, r.d_hist_g, (void*)r.d_row_src, r.d_pos_of, r.d_perm, r.d_M, r.d_off, r.d_tile_base,
                          r.d_act[0], r.d_act[1], r.d_act[2], r.d_act[3], r.d_logits};
            static_assert(kActBuffers == 4, "the list above names every activation buffer");
            for (void* p : rb) if (p) (void)hipFree(p);
            if (r.done) (void)hipEventDestroy(r.done);
        }
        if (c->static_slot.done) (void)hipEventDestroy(c->static_slot.done);
        for (uint32_t i = 0; i < kSegSlots; ++i) {
            if (c->h_segs[i]) (void)hipHostFree(c->h_segs[i]);
            if (c->seg_event[i]) (void)hipEventDestroy(c->seg_event[i]);
        }
        for (hipEvent_t e : c->prof_events) if (e) (void)hipEventDestroy(e);
        for (HostTenant& t : c->tenants) if (t.stage) (void)hipHostFree(t.stage);
        if (c->cache_event) (void)hipEventDestroy(c->cache_event);
    }
    delete c;
    return MT_OK;
}

mt_status mt_model_footprint_get(const mt_layer_spec* specs, uint32_t n_layers, uint32_t dtype, mt_model_footprint* out)
{
    if (!specs || !out || dtype > MT_BF16) return MT_EINVAL;
    *out = mt_model_footprint{};
    mt_ctx probe;                                   // a context without limits: the plan only depends on the element size
    probe.elem_size = dtype == MT_BF16 ? 2 : 4;
    probe.S = 0xffffffc0u;
    probe.cfg.max_classes = 0xffffffffu;
    HostTenant ht;
    const mt_status st = plan_model(&probe, specs, n_layers, &ht);
    if (st != MT_OK) return st;
    out->arena_bytes = layout_model(&ht);
    out->n_classes = ht.dev.n_classes;
    out->in_len = ht.dev.in_len;
    uint32_t width = ht.dev.in_fill;                // what plan_model holds against max_width
    for (uint32_t l = 0; l < n_layers; ++l) {
        const LayerDev& d = ht.layers[l].dev;
        if (!d.is_last) width = std::max(width, d.out_fill);
        if (d.kind == MT_FC) width = std::max(width, d.K);
    }
    out->min_width = width;
    return MT_OK;
}

mt_status mt_register_model(mt_ctx* c, uint32_t tenant, const mt_layer_spec* specs, uint32_t n_layers,
                            const void* const* weights, const void* const* biases)
{
    return mt_register_model_bn(c, tenant, specs, n_layers, weights, biases, nullptr, 0.0f);
}

mt_status mt_register_model_bn(mt_ctx* c, uint32_t tenant, const mt_layer_spec* specs, uint32_t n_layers,
                               const void* const* weights, const void* const* biases, const float* const* bn, float bn_eps)
{
    if (!c) return MT_EINVAL;
    if (!specs || !weights) return fail(c, MT_EINVAL, "null specs or weights");
    if (tenant >= c->cfg.max_tenants) return fail(c, MT_EINVAL, "tenant %u is outside 0..%u", tenant, c->cfg.max_tenants - 1);
    if (c->tenants[tenant].registered) return fail(c, MT_EEXIST, "tenant %u already has a model", tenant);
    HostTenant ht;
    mt_status st = plan_model(c, specs, n_layers, &ht);
    if (st != MT_OK) return st;
    for (uint32_t l = 0; l < n_layers; ++l) {
        const bool has_params = ht.layers[l].dev.kind == MT_FC || ht.layers[l].dev.kind == MT_CONV2D;
        if (has_params && !weights[l]) return fail(c, MT_EINVAL, "layer %u: null weights", l);
        if (bn && bn[l]) {
            if (ht.layers[l].dev.kind != MT_CONV2D) return fail(c, MT_EUNSUPPORTED, "layer %u: only a convolution can be followed by a batch normalisation", l);
            for (uint32_t ch = 0; ch < ht.layers[l].dev.N; ++ch)
                if (!((double)bn[l][3 * (size_t)ht.layers[l].dev.N + ch] + (double)bn_eps > 0.0))
                    return fail(c, MT_EINVAL, "layer %u: variance + eps of channel %u is not positive", l, ch);
        }
    }

    const uint64_t total = layout_model(&ht);
    if (total > c->cfg.arena_bytes)
        return fail(c, MT_ENOMEM, "model needs %llu bytes, the weight arena has %llu", (unsigned long long)total, (unsigned long long)c->cfg.arena_bytes);

    // the stage: pinned and kept in cache mode (models are reloaded from it), else a temporary
    std::vector<uint8_t> temp;
    uint8_t* stage = nullptr;
    if (!c->host_only) {
        HIP_TRY(c, hipSetDevice(c->cfg.device));
        if (c->cache) {
            if (hipHostMalloc((void**)&stage, stage_bytes(total), hipHostMallocDefault) != hipSuccess)
                return fail(c, MT_ENOMEM, "no pinned host memory for the %llu bytes of tenant %u", (unsigned long long)total, tenant);
            std::memset(stage, 0, stage_bytes(total));
        } else {
            temp.assign(stage_bytes(total), 0);
            stage = temp.data();
        }
        for (uint32_t l = 0; l < n_layers; ++l) {
            const HostLayer& hl = ht.layers[l];
            if (hl.dev.kind != MT_FC && hl.dev.kind != MT_CONV2D) continue;
            uint8_t* w_dst = stage + hl.w_rel;
            if (biases && biases[l]) std::memcpy(stage + hl.b_rel, biases[l], (size_t)hl.dev.N * 4);
            const void* w_src = weights[l];
            std::vector<uint8_t> folded;
            if (bn && bn[l]) {          // fold the normalisation into a copy of the filters and into the staged bias
                const size_t per = (size_t)hl.spec.in_features * hl.dev.ksize * hl.dev.ksize;
                folded.assign((const uint8_t*)weights[l], (const uint8_t*)weights[l] + (size_t)hl.dev.N * per * c->elem_size);
                fold_batchnorm(c->elem_size, folded.data(), (float*)(stage + hl.b_rel), hl.dev.N, per, bn[l], (double)bn_eps);
                w_src = folded.data();
            }
            if (c->elem_size == 2) pack_weights<uint16_t>(hl, w_src, w_dst); else pack_weights<float>(hl, w_src, w_dst);
        }
    }
    auto drop_stage = [&]() { if (c->cache && stage) (void)hipHostFree(stage); };

    // a model with skip connections may need a third or fourth activation buffer in every run slot
    if (!c->host_only && ht.act_buffers > c->act_buffers) {
        const size_t act_bytes = (size_t)c->P_cap * c->S * c->elem_size;
        for (RunSlot& r : c->slots)
            for (uint32_t i = c->act_buffers; i < ht.act_buffers; ++i)
                if (!r.d_act[i] && hipMalloc(&r.d_act[i], act_bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    drop_stage();
                    return fail(c, MT_ENOMEM, "no device memory for activation buffer %u of %zu bytes", i, act_bytes);
                }
        c->act_buffers = ht.act_buffers;
        for (RunSlot& r : c->slots) if (r.d_act[0] == c->d_act[0]) bind_slot(c, r);
    }

    // Registration is synchronous.  In cache mode every run in flight ends first: models may have to
    // give way, and a block that an earlier eviction freed may still be read by a run enqueued before it.
    uint64_t off = 0;
    hipError_t e = hipSuccess;
    const uint64_t stamp = ++c->use_clock;
    if (c->cache && !c->host_only) {
        const hipError_t es = hipDeviceSynchronize();
        if (es != hipSuccess) { drop_stage(); return fail(c, MT_EDEVICE, "device synchronisation failed: %s", hipGetErrorString(es)); }
    }
    if (!make_room(c, total, stamp, nullptr, false, &off, &e)) {
        drop_stage();
        if (e != hipSuccess) return fail(c, MT_EDEVICE, "eviction failed: %s", hipGetErrorString(e));
        return fail(c, MT_ENOMEM, "weight arena exhausted: model needs %llu bytes, %llu of %llu in use",
                    (unsigned long long)total, (unsigned long long)c->arena_used, (unsigned long long)c->cfg.arena_bytes);
    }
    ht.arena_off = off;
    for (uint32_t l = 0; l < n_layers; ++l) { ht.layers[l].dev.w_off = off + ht.layers[l].w_rel; ht.layers[l].dev.b_off = off + ht.layers[l].b_rel; }
    if (!c->host_only) {
        place_tenant(c, ht, off, stage);
        e = upload_tenant(c, tenant, ht, stage, nullptr, false);
        if (e != hipSuccess) {
            arena_free(c, off, total);
            drop_stage();
            return fail(c, MT_EDEVICE, "upload of tenant %u failed: %s", tenant, hipGetErrorString(e));
        }
    }
    ht.registered = true; ht.dev.registered = 1; ht.resident = true; ht.last_use = stamp;
    ht.stage = c->cache ? stage : nullptr;
    c->tenants[tenant] = ht;
    c->n_registered++;
    recompute_bounds(c);
    recompute_pool_fusion(c);
    return MT_OK;
}

mt_status mt_prefetch(mt_ctx* c, const uint32_t* tenants, uint32_t n, void* hip_stream)
{
    if (!c || (!tenants && n)) return MT_EINVAL;
    for (uint32_t i = 0; i < n; ++i)
        if (tenants[i] >= c->cfg.max_tenants || !c->tenants[tenants[i]].registered)
            return fail(c, MT_ENOTFOUND, "tenant %u has no model", tenants[i]);
    const uint64_t stamp = ++c->use_clock;          // everything named here is used "now": none of it gives way to the rest
    bool missing = false;
    for (uint32_t i = 0; i < n; ++i) { c->tenants[tenants[i]].last_use = stamp; missing |= !c->tenants[tenants[i]].resident; }
    if (!missing) return MT_OK;                     // (always the case outside cache mode)
    hipStream_t s = (hipStream_t)hip_stream;
    if (!c->host_only) {
        HIP_TRY(c, hipSetDevice(c->cfg.device));
        // runs in flight keep their weights and tables: the changes below queue up behind them
        for (RunSlot& r : c->slots)
            if (r.used) HIP_TRY(c, hipStreamWaitEvent(s, r.done, 0));
        if (c->static_slot.used) HIP_TRY(c, hipStreamWaitEvent(s, c->static_slot.done, 0));
        if (c->cache_pending && c->cache_stream != s) HIP_TRY(c, hipStreamWaitEvent(s, c->cache_event, 0));
    }
    mt_status result = MT_OK;
    for (uint32_t i = 0; i < n && result == MT_OK; ++i) {
        HostTenant& ht = c->tenants[tenants[i]];
        if (ht.resident) continue;
        uint64_t off = 0;
        hipError_t e = hipSuccess;
        if (!make_room(c, ht.arena_len, stamp, s, true, &off, &e)) {
            result = e != hipSuccess ? fail(c, MT_EDEVICE, "eviction failed: %s", hipGetErrorString(e))
                                     : fail(c, MT_ENOMEM, "the models named do not fit the weight arena together (%llu of %llu bytes in use, tenant %u needs %llu)",
                                            (unsigned long long)c->arena_used, (unsigned long long)c->cfg.arena_bytes, tenants[i], (unsigned long long)ht.arena_len);
            break;
        }
        if (!c->host_only) {
            place_tenant(c, ht, off, ht.stage);
            e = upload_tenant(c, tenants[i], ht, ht.stage, s, true);
            if (e != hipSuccess) {
                arena_free(c, off, ht.arena_len);
                result = fail(c, MT_EDEVICE, "upload of tenant %u failed: %s", tenants[i], hipGetErrorString(e));
                break;
            }
        } else {
            ht.arena_off = off;
        }
        ht.resident = true;
    }
    if (!c->host_only) {                            // also after a failure: part of the changes may be enqueued
        const hipError_t e = hipEventRecord(c->cache_event, s);
        if (e != hipSuccess && result == MT_OK) result = fail(c, MT_EDEVICE, "hipEventRecord failed: %s", hipGetErrorString(e));
        c->cache_pending = true; c->cache_stream = s;
    }
    return result;
}

mt_status mt_unregister_model(mt_ctx* c, uint32_t tenant)
{
    if (!c) return MT_EINVAL;
    if (tenant >= c->cfg.max_tenants || !c->tenants[tenant].registered) return fail(c, MT_ENOTFOUND, "tenant %u has no model", tenant);
    for (const Segment& s : c->pending)
        if (!s.ids && s.tenant == (int32_t)tenant) return fail(c, MT_ESTATE, "tenant %u has pending requests", tenant);
    if (!c->host_only) {
        HIP_TRY(c, hipSetDevice(c->cfg.device));
        HIP_TRY(c, hipDeviceSynchronize());
        HIP_TRY(c, hide_tenant(c, tenant, nullptr, false));
        if (c->tenants[tenant].stage) (void)hipHostFree(c->tenants[tenant].stage);
    }
    if (c->tenants[tenant].resident) arena_free(c, c->tenants[tenant].arena_off, c->tenants[tenant].arena_len);
    c->tenants[tenant] = HostTenant{};
    c->n_registered--;
    recompute_bounds(c);
    recompute_pool_fusion(c);
    return MT_OK;
}

static mt_status push_segment(mt_ctx* c, const Segment& s, uint32_t* first_index)
{
    if ((uint64_t)c->pending_rows + s.n_rows > c->cfg.max_requests)
        return fail(c, MT_EFULL, "%u rows pending, %u more exceed max_requests %u", c->pending_rows, s.n_rows, c->cfg.max_requests);
    Segment seg = s;
    seg.row_begin = c->pending_rows;
    if (first_index) *first_index = c->pending_rows;
    // consecutive submissions of one tenant from one contiguous buffer collapse into one run
    if (!c->pending.empty()) {
        Segment& b = c->pending.back();
        if (!b.ids && !seg.ids && b.tenant == seg.tenant && b.row_stride == seg.row_stride &&
            (const uint8_t*)b.src + (size_t)b.n_rows * b.row_stride * c->elem_size == (const uint8_t*)seg.src) {
            b.n_rows += seg.n_rows; c->pending_rows += seg.n_rows;
            return MT_OK;
        }
    }
    c->pending.push_back(seg);
    c->pending_rows += seg.n_rows;
    return MT_OK;
}

mt_status mt_submit(mt_ctx* c, uint32_t tenant, const void* inputs, uint32_t n_rows, uint32_t* first_index)
{
    if (!c) return MT_EINVAL;
    if (!inputs || n_rows == 0) return fail(c, MT_EINVAL, "null inputs or zero rows");
    if (tenant >= c->cfg.max_tenants || !c->tenants[tenant].registered) return fail(c, MT_ENOTFOUND, "tenant %u has no model", tenant);
    Segment s{};
    s.ids = nullptr; s.src = inputs; s.n_rows = n_rows; s.row_stride = c->tenants[tenant].dev.in_len; s.tenant = (int32_t)tenant;
    return push_segment(c, s, first_index);
}

mt_status mt_submit_batch(mt_ctx* c, const int32_t* tenant_ids, const void* inputs, uint32_t n_rows, uint32_t row_stride,
                          uint32_t* first_index)
{
    if (!c) return MT_EINVAL;
    if (!tenant_ids || !inputs || n_rows == 0 || row_stride == 0) return fail(c, MT_EINVAL, "null buffers, zero rows or zero stride");
    if (row_stride < c->max_in_len)
        return fail(c, MT_EINVAL, "row_stride %u is shorter than the longest registered input (%u)", row_stride, c->max_in_len);
    Segment s{};
    s.ids = tenant_ids; s.src = inputs; s.n_rows = n_rows; s.row_stride = row_stride; s.tenant = -1;
    return push_segment(c, s, first_index);
}

namespace {

__global__ void fill_zero_kernel(uint32_t* p, uint32_t n)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

// Packed rows a run of R rows can occupy: every tenant with traffic pads its segment to a multiple of 32.
constexpr uint32_t kBigWalkMinK = 256;     // the walking big-tile kernel needs seven stages of 32 (bf16) or 16 (fp32) per tile
constexpr uint32_t kConvLongK = 1024;      // reductions from here on are worth loader waves when a launch has at most one tile per CU

// Workgroups that share one packed row in the per-row kernels: `per_wg` units of work each, at most 64.
static uint32_t row_slices(uint64_t units, uint32_t per_wg)
{
    return (uint32_t)std::min<uint64_t>(std::max<uint64_t>((units + per_wg - 1) / per_wg, 1), 64);
}

uint32_t packed_rows_bound(const mt_ctx* c, uint32_t R)
{
    return (uint32_t)std::min<uint64_t>(c->P_cap, (uint64_t)round_up(R, kBrickRows) + (uint64_t)kBrickRows * std::min(R, c->n_registered));
}

// Carve the buffers of a run of R rows out of the static scratch array.  Returns the bytes needed;
// the slot's pointers are set only when they fit.  The batch descriptors come first, in one block
// that is cleared before the run (descr_words 32-bit words from rs->d_M).
uint64_t carve_static_slot(const mt_ctx* c, uint32_t R, RunSlot* rs, uint32_t* descr_words)
{
    const uint64_t T = c->cfg.max_tenants, P = packed_rows_bound(c, R);
    uint64_t at = 0;
    auto take = [&](uint64_t bytes) { const uint64_t o = at; at += round_up64(bytes, 256); return o; };
    const uint64_t o_M = take(T * 4), o_off = take((T + 1) * 4), o_tb = take((kListKinds * MT_MAX_LAYERS * (T + 1) + 1) * 4);
    const uint64_t descr_end = at;
    const uint64_t o_rt = take((uint64_t)R * 4), o_rr = take((uint64_t)R * 4), o_h = take((uint64_t)kHistEntries * 4);
    const uint64_t o_src = take((uint64_t)R * sizeof(void*)), o_pos = take((uint64_t)R * 4), o_perm = take(P * 4);
    uint64_t o_act[kActBuffers] = {};
    for (uint32_t i = 0; i < c->act_buffers; ++i) o_act[i] = take(P * c->S * c->elem_size);
    const uint64_t o_lg = take(P * c->C_pad * 4);
    if (at <= MT_STATIC_SCRATCH_BYTES) {
        uint8_t* b = c->static_scratch;
        rs->d_M = (uint32_t*)(b + o_M); rs->d_off = (uint32_t*)(b + o_off); rs->d_tile_base = (uint32_t*)(b + o_tb);
        rs->d_row_tenant = (int32_t*)(b + o_rt); rs->d_row_rank = (uint32_t*)(b + o_rr); rs->d_hist_g = (uint32_t*)(b + o_h);
        rs->d_row_src = (const void**)(b + o_src); rs->d_pos_of = (int32_t*)(b + o_pos); rs->d_perm = (int32_t*)(b + o_perm);
        for (uint32_t i = 0; i < (uint32_t)kActBuffers; ++i) rs->d_act[i] = i < c->act_buffers ? b + o_act[i] : nullptr;
        rs->d_logits = (float*)(b + o_lg);
        *descr_words = (uint32_t)(descr_end / 4);
    }
    return at;
}

mt_status run_impl(mt_ctx* c, void* hip_stream, const mt_outputs* out, uint32_t* n_rows, bool use_static);

}  // namespace

mt_status mt_run(mt_ctx* c, void* hip_stream, const mt_outputs* out, uint32_t* n_rows)
{
    return run_impl(c, hip_stream, out, n_rows, false);
}

mt_status mt_run_static(mt_ctx* c, void* hip_stream, const mt_outputs* out, uint32_t* n_rows)
{
    return run_impl(c, hip_stream, out, n_rows, true);
}

namespace {

mt_status run_impl(mt_ctx* c, void* hip_stream, const mt_outputs* out, uint32_t* n_rows, bool use_static)
{
    if (!c) return MT_EINVAL;
    if (n_rows) *n_rows = 0;
    if (c->host_only) return fail(c, MT_ESTATE, "host-only context cannot run");
    const uint32_t R = c->pending_rows;
    if (R == 0) { c->last_run_rows = 0; c->last_run_launches = 0; return MT_OK; }
    if (!out || !out->labels) return fail(c, MT_EINVAL, "null outputs");
    if (out->capacity < R) return fail(c, MT_EINVAL, "outputs hold %u rows, %u pending", out->capacity, R);
    if ((out->probs || out->logits) && out->row_stride < c->cfg.max_classes)
        return fail(c, MT_EINVAL, "row_stride %u is below max_classes %u", out->row_stride, c->cfg.max_classes);
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(c, hipSetDevice(c->cfg.device));

    // Model cache: the tenants of per-tenant submissions are made resident here (the host knows
    // them); tenants that appear only in device-resident id arrays must have been prefetched.
    // A residency change enqueued on another stream comes first.
    if (c->cache) {
        std::vector<uint32_t> named;
        for (const Segment& sg : c->pending)
            if (!sg.ids && (named.empty() || named.back() != (uint32_t)sg.tenant)) named.push_back((uint32_t)sg.tenant);
        std::sort(named.begin(), named.end());
        named.erase(std::unique(named.begin(), named.end()), named.end());
        if (!named.empty()) { const mt_status st = mt_prefetch(c, named.data(), (uint32_t)named.size(), hip_stream); if (st != MT_OK) return st; }
        if (c->cache_pending && c->cache_stream != s) HIP_TRY(c, hipStreamWaitEvent(s, c->cache_event, 0));
    }
    // the run's slot of device scratch; a stream other than the one that used it last waits for that run
    // (the slot this stream used last, so that runs on one stream keep their buffers and never wait
    // across streams; else a slot nobody has used; else the one used longest ago)
    RunSlot* pick = nullptr;
    uint32_t static_descr_words = 0;
    if (use_static) {
        // the run's buffers come out of the static array, sized for this run; nothing is allocated
        const uint64_t need = carve_static_slot(c, R, &c->static_slot, &static_descr_words);
        if (need > MT_STATIC_SCRATCH_BYTES)
            return fail(c, MT_EINVAL, "a run of %u rows needs %llu bytes of scratch in this context, the static array holds %u",
                        R, (unsigned long long)need, (unsigned)MT_STATIC_SCRATCH_BYTES);
        pick = &c->static_slot;
    }
    if (!pick) for (RunSlot& r : c->slots) if (r.used && r.stream == s) { pick = &r; break; }
    if (!pick) for (RunSlot& r : c->slots) if (!r.used) { pick = &r; break; }
    if (!pick) { pick = &c->slots[0]; for (RunSlot& r : c->slots) if (r.last_run < pick->last_run) pick = &r; }
    RunSlot& rs = *pick;
    // A run of one submission carries its segment in the kernel arguments; only runs of several
    // submissions put the table into one of the pinned slots, which stays busy until the run is over.
    // The host never waits for one: when the GPU is still reading all of them the call is refused.
    const uint32_t n_segs = (uint32_t)c->pending.size();
    uint32_t slot = 0;
    if (n_segs > 1) {
        bool found = false;
        for (uint32_t i = 0; i < kSegSlots && !found; ++i) {
            const uint32_t cand = (uint32_t)((c->run_count + i) % kSegSlots);
            if (c->seg_busy[cand]) {
                const hipError_t q = hipEventQuery(c->seg_event[cand]);
                if (q == hipErrorNotReady) continue;
                if (q != hipSuccess) return fail(c, MT_EDEVICE, "hipEventQuery: %s", hipGetErrorString(q));
                c->seg_busy[cand] = false;
            }
            slot = cand; found = true;
        }
        if (!found) return fail(c, MT_EFULL, "%u runs of several submissions are still in flight; call again later", kSegSlots);
        std::memcpy(c->h_segs[slot], c->pending.data(), c->pending.size() * sizeof(Segment));
    }
    if (rs.used && rs.stream != s) HIP_TRY(c, hipStreamWaitEvent(s, rs.done, 0));
    bind_slot(c, rs);
    const uint32_t T = c->cfg.max_tenants;
    uint32_t launches = 0;

    // Big tiles are for runs that are compute bound as a whole: enough rows, and more flops per
    // byte of registered weights than the chip's ridge point.  Weight-streaming mixes keep every
    // tenant in the streaming kernel (no second launch per layer, layer 0 reads submitted rows).
    const double run_flops = 2.0 * R * (c->n_registered ? c->sum_macs / c->n_registered : 0.0);
    const bool big_enabled = R >= (uint32_t)kBigMinBatch && run_flops >= kRidgeFlopsPerByte * (double)c->arena_used;
    const bool split_k = run_split_k(c, R);
    BatchArgs b{};
    b.segs = c->d_segs[slot]; b.n_segs = n_segs; b.R = R; b.T = T; b.n_layer_slots = c->n_layer_slots;
    b.first = c->pending[0]; b.row_src = c->d_row_src; b.elem_size = c->elem_size;
    b.tenants = c->d_tenants; b.facts = c->d_facts; b.served = (unsigned long long*)c->d_served;
    {   // large batches are ranked by a kernel of their own, where its per-workgroup histograms fit the batcher's LDS
        uint32_t Tp = 64;
        while (Tp < T) Tp <<= 1;
        const uint32_t groups = (R + kRankRows - 1) / kRankRows;
        const bool spread = R >= (uint32_t)kRankMinRows && T <= (uint32_t)kRankMaxTenants && (uint64_t)groups * Tp <= (uint64_t)kHistEntries;
        b.n_rank_groups = spread ? groups : 0; b.hist_g = c->d_hist_g;
    }
    b.row_tenant = c->d_row_tenant; b.row_rank = c->d_row_rank; b.pos_of = c->d_pos_of; b.perm = c->d_perm;
    b.M = c->d_M; b.off = c->d_off; b.tile_base = c->d_tile_base; b.big_layers = c->d_tile_base + (size_t)kListKinds * MT_MAX_LAYERS * (T + 1); b.fc_split_k = split_k;
    for (uint32_t g = 0; g < MT_MAX_LAYERS / kLayerGroup; ++g)
        b.list_mask[g] = big_enabled ? c->list_mask[g] : c->list_mask[g] & ((1u << (2 * kLayerGroup)) - 1);   // no big-tile lists to build
    b.big_enabled = big_enabled; b.big_min_tiles = c->big_min_tiles;
    const OutPtrs outp{out->labels, out->probs, out->logits, out->n_classes, out->row_stride};
    b.out = outp;
    // A last layer of at most 32 classes is one column block: its FC tiles finish their rows
    // themselves.
    // ... and one of at most 128 classes is one tile of four column blocks, unless this run's tiles
    // are single column blocks (the K-split shape of small runs).
    const uint32_t fuse_head_max = fused_head_classes(c, split_k);
    const bool fuse_head = fuse_head_max > 0 && c->min_reg_classes <= fuse_head_max;
    const uint32_t head_min_classes = fuse_head ? fuse_head_max + 1 : 0;
    const bool out_vec_ok = out->row_stride % 4 == 0 && ((uintptr_t)out->probs & 15) == 0 && ((uintptr_t)out->logits & 15) == 0;
    if (c->profiling) for (uint32_t i = 0; i < kProfSlots; ++i) c->prof_used[i] = false;
    // From here on a failure may leave part of the run enqueued: the launches sit in a body of their
    // own, and the bookkeeping behind it (events, slot, pending list) is closed whatever it returns.
    auto enqueue = [&]() -> mt_status {
#define TIMED(slot, call)                                                                   \
    do {                                                                                    \
        if (c->profiling) HIP_TRY(c, hipEventRecord(c->prof_events[2 * (slot)], s));        \
        HIP_TRY(c, call); ++launches;                                                       \
        if (c->profiling) { HIP_TRY(c, hipEventRecord(c->prof_events[2 * (slot) + 1], s)); c->prof_used[slot] = true; c->prof_last = (slot); } \
    } while (0)
    if (use_static) {
        // the array keeps what the last run on this GPU left: the descriptors start from zero (a fill
        // kernel, not a memset node, so that the sequence can be captured into a graph)
        hipLaunchKernelGGL(fill_zero_kernel, dim3((static_descr_words + 255) / 256), dim3(256), 0, s, rs.d_M, static_descr_words);
        HIP_TRY(c, hipGetLastError()); ++launches;
    }
    TIMED(kProfBatcher, launch_batcher(b, s));
    if (b.n_rank_groups) launches += 2;

    // The FC kernel of layer 0 reads the submitted rows itself when every row is 16-byte aligned
    // and a whole number of 16-byte chunks long; otherwise (and for CNN models, whose images are
    // channel-padded) a gather pass stages the inputs first.
    // The big-tile kernel reads bricks only (it was measured slower when it gathers rows itself,
    // since every row is then fetched in 16-byte pieces by each of a layer's column tiles):
    // whenever a tenant could reach it at layer 0, stage.
    const bool big_possible = big_enabled && c->max_nt[2][0] > 0 && tile_bound(c, 2, 0, R) >= c->big_min_tiles;
    bool fuse_gather = c->any_fc_first && c->fc_first_chunked && !c->no_fused_gather && !big_possible;
    for (const Segment& sg : c->pending)
        if (((uintptr_t)sg.src & 15) || ((uint64_t)sg.row_stride * c->elem_size) % 16) fuse_gather = false;
    // packed rows: every tenant with traffic pads its segment to a multiple of 32
    const uint32_t P = packed_rows_bound(c, R);
    {
        GatherArgs g{};
        g.row_src = c->d_row_src; g.P = P; g.tenants = c->d_tenants; g.layers = c->d_layers; g.row_tenant = c->d_row_tenant;
        g.perm = c->d_perm; g.off = c->d_off; g.T = T; g.act = c->d_act[0]; g.S = c->S; g.elem_size = c->elem_size; g.zeros = c->d_zeros;
        // workgroups per block of 32 rows: each takes ~64 KiB of it, so that long rows have enough loads in flight
        const uint32_t gs = row_slices((uint64_t)c->max_in_len * c->elem_size * kBrickRows, 65536);      // c5: 146 -> 133 us with four
        if (c->any_fc_first && !fuse_gather) TIMED(kProfGather, launch_gather(g, gs, s));
        // workgroups per image row: each takes ~2048 pixels (eight per thread), so that a few large images fill the chip too
        if (c->any_conv_first) TIMED(kProfGatherImg, launch_gather_image(g, row_slices(c->max_image_pixels, 2048), s));
    }

    ActBufs bufs{};                        // every layer names the buffers it reads and writes (LayerDev::in_buf ...)
    for (int i = 0; i < kActBuffers; ++i) bufs.p[i] = c->d_act[i];
    for (uint32_t l = 0; l < c->n_layer_slots; ++l) {
        // a pooling index that the convolutions before it have already served: nothing runs, the
        // pooled activation is where the pooling layer would have written it
        if (l > 0 && c->pool_fused[l - 1]) continue;
        for (int kind = 0; kind < kListKinds; ++kind) {
            const uint64_t grid = tile_bound(c, kind, l, R, split_k, big_enabled);
            if (grid == 0 || (kind == 2 && (!big_enabled || grid < c->big_min_tiles))) continue;   // no big tiles possible: the batcher made none
            GemmArgs ga{};
            ga.tile_base = c->d_tile_base + ((size_t)kind * MT_MAX_LAYERS + l) * (T + 1);
            ga.T = T; ga.layer = l; ga.fc_split_k = split_k; ga.big_layers = b.big_layers;
            ga.gather = (kind == 0 && l == 0 && fuse_gather); ga.perm = c->d_perm; ga.row_src = c->d_row_src;
            ga.fuse_head = fuse_head; ga.fuse_head_max = fuse_head_max; ga.out_vec_ok = out_vec_ok; ga.out = outp; ga.pool = kind == 1 && c->pool_fused[l];
            ga.layers = c->d_layers; ga.off = c->d_off; ga.M = c->d_M; ga.act = bufs; ga.arena = c->d_arena;
            ga.logits = c->d_logits; ga.S = c->S; ga.C_pad = c->C_pad; ga.zeros = c->d_zeros;
            if (grid > 0x7ffffff0u)          // cannot happen within the limits mt_create accepts; never launch fewer workgroups than tiles
                return fail(c, MT_EUNSUPPORTED, "layer %u: %llu tiles exceed one launch", l, (unsigned long long)grid);
            const uint32_t g32 = (uint32_t)grid;
            if (kind == 0) TIMED(kProfFc + l, launch_fc(ga, c->cfg.dtype, g32, s));
            else if (kind == 1) TIMED(kProfConv + l, launch_conv(ga, c->cfg.dtype, c->max_conv_cb[l], c->conv_quad[l],
                                                                    (c->conv_img_lds[l] > 1 && !c->pool_fused[l] && !c->no_conv_img) ? c->conv_img_lds[l] : 0, c->conv_img_two[l] == 1,
                                                                    !c->no_conv_loaders && c->min_conv_k[l] >= kConvLongK,
                                                                    c->conv_uniform[l] && !c->no_conv_uniform && (uint64_t)c->cfg.max_requests * c->S * c->elem_size < (1ull << 31), g32, s));
            else TIMED(kProfBig + l, launch_fc_big(ga, c->cfg.dtype, g32, (c->big_walk && c->min_fc_k[l] >= kBigWalkMinK) ? c->n_cus : 0, s));
        }
        if (c->has_gap[l]) {
            GapArgs pa{};
            pa.layer = l; pa.P = P; pa.layers = c->d_layers; pa.tenants = c->d_tenants; pa.row_tenant = c->d_row_tenant;
            pa.perm = c->d_perm; pa.off = c->d_off; pa.T = T; pa.act = bufs; pa.S = c->S;
            pa.elem_size = c->elem_size;
            TIMED(kProfGap + l, launch_gap(pa, s));
        }
        if (c->has_image_ops[l]) {         // max-pooling and residual additions of this layer index
            GapArgs pa{};
            pa.layer = l; pa.P = P; pa.layers = c->d_layers; pa.tenants = c->d_tenants; pa.row_tenant = c->d_row_tenant;
            pa.perm = c->d_perm; pa.off = c->d_off; pa.T = T; pa.act = bufs; pa.S = c->S;
            pa.elem_size = c->elem_size;
            TIMED(kProfImageOps + l, launch_image_ops(pa, row_slices(c->image_op_fill[l] * c->elem_size / 16, 2048), s));   // eight 16-byte chunks per thread
        }
    }

    if (!fuse_head || c->max_reg_classes > fuse_head_max) {
        HeadArgs h{};
        h.R = R; h.tenants = c->d_tenants; h.row_tenant = c->d_row_tenant; h.pos_of = c->d_pos_of; h.logits = c->d_logits;
        h.C_pad = c->C_pad; h.out = outp; h.min_classes = head_min_classes;
        h.vec_ok = out_vec_ok;
        TIMED(kProfHead, launch_head(h, s));
    }
#undef TIMED
    return MT_OK;
    };
    mt_status st = enqueue();
    if (st != MT_OK && launches == 0) return st;         // nothing was enqueued: the pending list is kept
    c->prof_valid = c->profiling && st == MT_OK;
    if (n_segs > 1) {
        const hipError_t e = hipEventRecord(c->seg_event[slot], s);
        if (e != hipSuccess && st == MT_OK) st = fail(c, MT_EDEVICE, "hipEventRecord: %s", hipGetErrorString(e));
        c->seg_busy[slot] = true;
    }
    {
        const hipError_t e = hipEventRecord(rs.done, s);
        if (e != hipSuccess && st == MT_OK) st = fail(c, MT_EDEVICE, "hipEventRecord: %s", hipGetErrorString(e));
    }
    rs.used = true; rs.stream = s; rs.last_run = c->run_count;
    c->run_count++;
    c->last_stream = s;
    c->pending.clear();
    c->pending_rows = 0;
    c->last_run_rows = st == MT_OK ? R : 0; c->last_run_launches = launches;
    if (n_rows && st == MT_OK) *n_rows = R;
    return st;
}

}  // namespace

mt_status mt_last_counts(mt_ctx* c, uint32_t* counts)
{
    if (!c || !counts) return MT_EINVAL;
    if (c->host_only) return fail(c, MT_ESTATE, "host-only context");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipStreamSynchronize(c->last_stream));
    HIP_TRY(c, hipMemcpy(counts, c->d_M, (size_t)c->cfg.max_tenants * 4, hipMemcpyDeviceToHost));
    return MT_OK;
}

// ---- accounting and cost prediction (paper section 3.2) -------------------------------------
namespace {

// Algorithmic cost of one request of a model, from its description alone.
void request_cost(const mt_ctx* c, const HostTenant& ht, uint64_t* flops, uint64_t* weight_bytes, uint64_t* io_bytes)
{
    const uint64_t es = c->elem_size;
    *flops = *weight_bytes = *io_bytes = 0;
    for (uint32_t l = 0; l < ht.n_layers; ++l) {
        const mt_layer_spec& s = ht.layers[l].spec;
        const LayerDev& d = ht.layers[l].dev;
        uint64_t in_len = 0;
        if (s.kind == MT_FC) {
            *flops += 2ull * s.in_features * s.out_features;
            *weight_bytes += (uint64_t)s.in_features * s.out_features * es + (uint64_t)s.out_features * 4;
            in_len = s.in_features;
        } else if (s.kind == MT_CONV2D) {
            *flops += 2ull * d.rows_per_req * s.kh * s.kw * s.in_features * s.out_features;
            *weight_bytes += (uint64_t)s.kh * s.kw * s.in_features * s.out_features * es + (uint64_t)s.out_features * 4;
            in_len = (uint64_t)s.in_h * s.in_w * s.in_features;
        } else {
            in_len = (uint64_t)s.in_h * s.in_w * s.in_features;
        }
        if (l == 0) *io_bytes += in_len * es;
        if (l + 1 < ht.n_layers) *io_bytes += 2ull * d.out_len * es;
        else *io_bytes += 2ull * d.out_len * 4 + 4;
    }
}

// Per-kernel time model, microseconds and megabytes; constants fitted on one MI355X (the
// measurements are in the design notes).  A streaming FC launch costs a fixed part, its bytes
// from HBM (weights of the active tenants) and the bytes its tiles re-read through L2 (weight
// panels re-read by further row tiles, activation rows re-read by every column group; three
// times that when layer 0 gathers the submitted rows in 16-byte pieces); it cannot be shorter
// than the chain of dependent loads through K of one tile.
// Weights that fit the 256 MB memory-side cache and are read by every run stream faster than
// weights that come from HBM every time (steady serving of the same tenants is assumed).
constexpr double kUsLaunchGap = 4.0;
constexpr double kUsFcFixed = 3.7, kUsPerMbCached = 0.132, kUsPerMbHbm = 0.18, kCachedMb = 240.0;
constexpr double kUsPerMbL2 = 0.056, kUsFcChainFixed = 4.0, kUsPerKStep = 0.12;
constexpr double kUsBigFixed = 4.0, kUsBigTileFixed = 7.0, kUsBigTilePer4096 = 116.0;
constexpr double kUsConvFixed = 5.0, kConvMbPerUs = 4.0, kConvMflopPerUs = 0.5e3;      // 4.0 TB/s, 0.5 PFLOP/s
constexpr double kUsConvFramePerKStep = 0.13, kConvFrameMflopPerUs = 0.6e3;   // the same for layer indices served from LDS frames: filter bricks are the only loads in the K loop
constexpr double kUsConvPerKStep = 0.21;     // a convolution tile's walk through K, per k-step of 32 bytes per pixel: a launch lasts at least as long as its longest tile
constexpr double kUsSmallFixed = 3.0, kCopyMbPerUs = 3.7, kHeadMbPerUs = 5.7, kUsHeadPerRow = 0.0008;
constexpr double kComputeUnits = 256.0;
constexpr double kUploadBytesPerMs = 55e6, kUsUploadFixed = 20.0;     // pinned host memory to HBM over the host link: 55 GB/s measured

}  // namespace

mt_status mt_tenant_account_get(mt_ctx* c, uint32_t tenant, mt_tenant_account* out)
{
    if (!c || !out) return MT_EINVAL;
    if (tenant >= c->cfg.max_tenants) return fail(c, MT_EINVAL, "tenant %u is outside 0..%u", tenant, c->cfg.max_tenants - 1);
    if (!c->tenants[tenant].registered) return fail(c, MT_ENOTFOUND, "tenant %u has no model", tenant);
    *out = mt_tenant_account{};
    request_cost(c, c->tenants[tenant], &out->flops_per_request, &out->weight_bytes, &out->io_bytes_per_request);
    out->resident = c->tenants[tenant].resident;
    out->arena_bytes = c->tenants[tenant].arena_len;
    if (!c->host_only) {
        uint64_t counters[2] = {0, 0};
        HIP_TRY(c, hipSetDevice(c->cfg.device));
        HIP_TRY(c, hipDeviceSynchronize());
        HIP_TRY(c, hipMemcpy(counters, c->d_served + 2 * (size_t)tenant, sizeof counters, hipMemcpyDeviceToHost));
        out->requests = counters[0]; out->runs = counters[1];
    }
    return MT_OK;
}

mt_status mt_estimate_run(mt_ctx* c, const uint32_t* counts, mt_run_estimate* out)
{
    if (!c || !counts || !out) return MT_EINVAL;
    *out = mt_run_estimate{};
    const uint32_t T = c->cfg.max_tenants;
    const double es = c->elem_size, MB = 1e6;
    uint64_t R = 0;
    for (uint32_t t = 0; t < T; ++t) {
        if (!counts[t]) continue;
        if (!c->tenants[t].registered) return fail(c, MT_ENOTFOUND, "tenant %u has no model", t);
        R += counts[t];
        uint64_t f, wb, io;
        request_cost(c, c->tenants[t], &f, &wb, &io);
        out->flops += (double)f * counts[t];
        out->hbm_bytes += (double)wb + (double)io * counts[t];
    }
    if (R > c->cfg.max_requests) return fail(c, MT_EINVAL, "%llu rows exceed max_requests %u", (unsigned long long)R, c->cfg.max_requests);
    out->rows = (uint32_t)R;
    if (R == 0) return MT_OK;

    // the same decisions as mt_run and the batcher take
    const double run_flops = 2.0 * R * (c->n_registered ? c->sum_macs / c->n_registered : 0.0);
    const bool big_enabled = R >= (uint64_t)kBigMinBatch && run_flops >= kRidgeFlopsPerByte * (double)c->arena_used;
    const bool big_possible = big_enabled && c->max_nt[2][0] > 0 && tile_bound(c, 2, 0, R) >= c->big_min_tiles;
    const bool fuse_gather = c->any_fc_first && c->fc_first_chunked && !c->no_fused_gather && !big_possible;
    const bool split_k = run_split_k(c, R);
    const uint32_t fuse_head_max = fused_head_classes(c, split_k);
    const bool fuse_head = fuse_head_max > 0 && c->min_reg_classes <= fuse_head_max;
    uint32_t Tp = 64;
    while (Tp < T) Tp <<= 1;
    const uint64_t groups_r = (R + kRankRows - 1) / kRankRows;
    const bool spread = R >= (uint64_t)kRankMinRows && T <= (uint32_t)kRankMaxTenants && groups_r * Tp <= (uint64_t)kHistEntries;

    double weights_mb = 0.0;                 // weights this run reads, all layers
    for (uint32_t t = 0; t < T; ++t) {
        if (!counts[t]) continue;
        uint64_t f, wb, io;
        request_cost(c, c->tenants[t], &f, &wb, &io);
        weights_mb += wb / MB;
    }
    const double us_per_mb = weights_mb <= kCachedMb ? kUsPerMbCached : kUsPerMbHbm;
    double us = 0.0;
    uint32_t launches = 0;
    auto launch = [&](double t) { us += t + (launches ? kUsLaunchGap : 0.0); ++launches; };
    if (spread) { launch(20.0 + 0.15 * R / 1024.0); launches += 2; }       // ranking, scan, placement
    else launch(7.0 + 1.1 * R / 1024.0);                                   // kernel trace: 7.0 us at 64 rows, 9.2 at 2048, 11.3 at 4096

    double fc_in_mb = 0.0, img_in_mb = 0.0, img_out_mb = 0.0;
    for (uint32_t t = 0; t < T; ++t) {
        if (!counts[t]) continue;
        const HostTenant& ht = c->tenants[t];
        if (ht.dev.in_layout == kLayoutBricks) fc_in_mb += counts[t] * (double)ht.dev.in_len * es / MB;
        else { img_in_mb += counts[t] * (double)ht.dev.in_len * es / MB; img_out_mb += counts[t] * (double)ht.dev.in_fill * es / MB; }
    }
    if (c->any_fc_first && !fuse_gather) launch(kUsSmallFixed + 2.0 * fc_in_mb / kCopyMbPerUs);
    if (c->any_conv_first) launch(kUsSmallFixed + (img_in_mb + img_out_mb) / kCopyMbPerUs);

    for (uint32_t l = 0; l < c->n_layer_slots; ++l) {
        if (l > 0 && c->pool_fused[l - 1]) continue;           // pooled by the convolutions of the index before
        // which tenants take big tiles at this layer index (the batcher's rule)
        uint64_t big_tiles = 0;
        if (big_enabled && c->max_nt[2][l] > 0)
            for (uint32_t t = 0; t < T; ++t) {
                if (!counts[t] || l >= c->tenants[t].n_layers) continue;
                const LayerDev& d = c->tenants[t].layers[l].dev;
                if (d.kind == MT_FC && fc_is_big(counts[t], d.N_pad))
                    big_tiles += (uint64_t)((big_rows(counts[t]) + kBigTile - 1) / kBigTile) * ((d.N_pad + kBigTile - 1) / kBigTile);
            }
        const bool big_layer = big_tiles >= c->big_min_tiles;
        double w_mb = 0.0, l2_mb = 0.0, chain = 0.0, big_us = 0.0, conv_mb = 0.0, conv_mflop = 0.0, gap_mb = 0.0, ops_mb = 0.0;
        double big_rounds_k = 0.0, conv_chain = 0.0;
        const bool conv_frames = c->conv_img_lds[l] > 1 && !c->pool_fused[l] && !c->no_conv_img;     // the launch decision of run_impl
        for (uint32_t t = 0; t < T; ++t) {
            if (!counts[t] || l >= c->tenants[t].n_layers) continue;
            const LayerDev& d = c->tenants[t].layers[l].dev;
            const double M = counts[t];
            if (d.kind == MT_FC) {
                const bool big = big_layer && fc_is_big(counts[t], d.N_pad);
                const uint32_t Mb = big ? big_rows(counts[t]) : 0, Ms = counts[t] - Mb;
                if (big) big_rounds_k += (double)((Mb + kBigTile - 1) / kBigTile) * ((d.N_pad + kBigTile - 1) / kBigTile) * d.K;
                if (Ms) {
                    const uint32_t groups = fc_groups(d.N_pad, split_k), trows = fc_tile_rows(d.N_pad, split_k);
                    const double panel_mb = (double)d.N_pad * d.K * es / MB / groups;
                    const double row_tiles = (Ms + trows - 1) / trows;
                    const double act_mb = (double)Ms * d.K * es / MB;
                    w_mb += panel_mb * groups;
                    l2_mb += panel_mb * groups * (row_tiles - 1) + act_mb * groups * ((l == 0 && fuse_gather) ? 3.0 : 1.0);
                    const uint32_t nblk = d.N_pad / kBrickRows, split = split_k ? 1u : (nblk >= 3 ? 4u : nblk);
                    const double k_steps = d.K * es / 32.0 / (4 / split);       // bricks one wave walks (the waves split K when split < 4)
                    chain = std::max(chain, kUsFcChainFixed + kUsPerKStep * k_steps);
                }
            } else if (d.kind == MT_CONV2D) {
                const double out_elems = (c->pool_fused[l] ? d.N : d.out_len) + (d.fuse_add ? d.out_len : 0);      // pooled on the way out; the other operand of an addition done here
                conv_mb += (M * ((double)d.in_h * d.in_w * d.cin + out_elems) * es + (double)d.N_pad * d.K * es) / MB;
                conv_mflop += 2.0 * M * d.rows_per_req * d.k_valid * d.N / 1e6;
                conv_chain = std::max(conv_chain, (conv_frames ? kUsConvFramePerKStep : kUsConvPerKStep) * d.k_valid * es / 32.0);
            } else if (d.kind == MT_GAP) {
                gap_mb += M * ((double)d.in_h * d.in_w * d.cin + d.out_len) * es / MB;
            } else if (d.kind == MT_MAXPOOL || d.kind == MT_ADD) {    // an addition has two inputs
                ops_mb += M * ((double)d.in_h * d.in_w * d.cin * (d.kind == MT_ADD ? 2.0 : 1.0) + d.out_len) * es / MB;
            }
        }
        if (c->max_nt[0][l] > 0) launch(std::max(chain, kUsFcFixed + us_per_mb * w_mb + kUsPerMbL2 * l2_mb));
        if (c->max_nt[1][l] > 0) launch(kUsConvFixed + std::max(conv_chain, std::max(conv_mb / kConvMbPerUs, conv_mflop / (conv_frames ? kConvFrameMflopPerUs : kConvMflopPerUs))));
        if (big_enabled && c->max_nt[2][l] > 0 && tile_bound(c, 2, l, R) >= c->big_min_tiles) {
            // tiles share the chip in rounds of one per compute unit; a tile's time grows with K
            if (big_layer) big_us = std::ceil(big_tiles / kComputeUnits) * kUsBigTileFixed + big_rounds_k / kComputeUnits / 4096.0 * kUsBigTilePer4096;
            launch(kUsBigFixed + big_us);
        }
        if (c->has_gap[l]) launch(kUsSmallFixed + gap_mb / kCopyMbPerUs);
        if (c->has_image_ops[l]) launch(kUsSmallFixed + ops_mb / kCopyMbPerUs);
    }
    if (!fuse_head || c->max_reg_classes > fuse_head_max)
        launch(kUsSmallFixed + std::max(3.0 * R * c->C_pad * 4.0 / MB / kHeadMbPerUs, kUsHeadPerRow * R));
    out->launches = launches;
    out->device_ms = us * 1e-3;
    // models that are not resident have to cross the host link first: their footprint is fixed, so
    // that time is as predictable as the run itself (section 3.3)
    for (uint32_t t = 0; t < T; ++t)
        if (counts[t] && !c->tenants[t].resident) out->upload_bytes += (double)c->tenants[t].arena_len;
    out->upload_ms = out->upload_bytes ? kUsUploadFixed * 1e-3 + out->upload_bytes / kUploadBytesPerMs : 0.0;
    return MT_OK;
}

mt_status mt_admit(mt_ctx* c, const uint32_t* pending, double budget_ms, uint32_t* admitted, mt_run_estimate* est)
{
    if (!c || !pending || !admitted) return MT_EINVAL;
    if (!(budget_ms > 0.0)) return fail(c, MT_EINVAL, "the budget must be positive");
    const uint32_t T = c->cfg.max_tenants;
    uint32_t top = 0;
    for (uint32_t t = 0; t < T; ++t) {
        if (pending[t] && !c->tenants[t].registered) return fail(c, MT_ENOTFOUND, "tenant %u has no model", t);
        top = std::max(top, pending[t]);
    }
    std::vector<uint32_t> trial(T);
    mt_run_estimate e{};
    auto fits = [&](uint32_t level) {
        uint64_t rows = 0;
        for (uint32_t t = 0; t < T; ++t) { trial[t] = std::min(pending[t], level); rows += trial[t]; }
        if (rows > c->cfg.max_requests) return false;
        if (mt_estimate_run(c, trial.data(), &e) != MT_OK) return false;
        return e.device_ms + e.upload_ms <= budget_ms;
    };
    // the predicted time grows with the level (up to small steps where a larger batch changes
    // the launch plan), so the highest level that fits is found by bisection and then verified
    uint32_t lo = 0, hi = top;                  // invariant: level lo fits (0 always does)
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (fits(mid)) lo = mid; else hi = mid - 1;
    }
    while (lo > 0 && !fits(lo)) --lo;
    fits(lo);
    for (uint32_t t = 0; t < T; ++t) admitted[t] = trial[t];
    if (est) *est = e;
    return MT_OK;
}

mt_status mt_set_profiling(mt_ctx* c, int enable)
{
    if (!c) return MT_EINVAL;
    if (c->host_only) return fail(c, MT_ESTATE, "host-only context");
    if (enable && c->prof_events.empty()) {
        HIP_TRY(c, hipSetDevice(c->cfg.device));
        c->prof_events.resize(2 * kProfSlots);
        for (hipEvent_t& e : c->prof_events) HIP_TRY(c, hipEventCreate(&e));
    }
    c->profiling = enable != 0;
    if (!enable) c->prof_valid = false;
    return MT_OK;
}

mt_status mt_get_profile(mt_ctx* c, mt_profile* out)
{
    if (!c || !out) return MT_EINVAL;
    std::memset(out, 0, sizeof *out);
    if (!c->prof_valid) return fail(c, MT_ESTATE, "no profiled run to read");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipStreamSynchronize(c->last_stream));
    auto ms = [&](uint32_t slot, float* dst) -> hipError_t {
        *dst = 0.0f;
        if (!c->prof_used[slot]) return hipSuccess;
        return hipEventElapsedTime(dst, c->prof_events[2 * slot], c->prof_events[2 * slot + 1]);
    };
    HIP_TRY(c, ms(kProfBatcher, &out->batcher_ms));
    HIP_TRY(c, ms(kProfGather, &out->gather_ms));
    { float img = 0.0f; HIP_TRY(c, ms(kProfGatherImg, &img)); out->gather_ms += img; }
    HIP_TRY(c, ms(kProfHead, &out->head_ms));
    for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
        HIP_TRY(c, ms(kProfFc + l, &out->fc_ms[l]));
        HIP_TRY(c, ms(kProfConv + l, &out->conv_ms[l]));
        HIP_TRY(c, ms(kProfBig + l, &out->fc_big_ms[l]));
        HIP_TRY(c, ms(kProfGap + l, &out->gap_ms[l]));
        HIP_TRY(c, ms(kProfImageOps + l, &out->ops_ms[l]));
    }
    HIP_TRY(c, hipEventElapsedTime(&out->total_ms, c->prof_events[2 * kProfBatcher], c->prof_events[2 * c->prof_last + 1]));
    return MT_OK;
}

mt_status mt_debug_copy(void* dst, const void* src, uint64_t bytes, void* stream)
{
    if (!dst || !src || bytes % 16) return MT_EINVAL;
    return launch_copy(dst, src, bytes, (hipStream_t)stream) == hipSuccess ? MT_OK : MT_EDEVICE;
}

mt_status mt_debug_mfma_rate(void* stream, double* tflops)
{
    if (!tflops) return MT_EINVAL;
    *tflops = 0.0;
    constexpr uint32_t kGrid = 2048, kIters = 500;          // 2048 workgroups of 8 waves x 500 x 64 MFMAs: ~10 ms
    hipStream_t s = (hipStream_t)stream;
    float* buf = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = 0.0f;
    hipError_t e = hipMalloc((void**)&buf, (size_t)kGrid * 512 * 4);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = launch_mfma_rate(buf, kIters / 10, kGrid, s);      // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_mfma_rate(buf, kIters, kGrid, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (e != hipSuccess || ms <= 0.0f) return MT_EDEVICE;
    *tflops = (double)kGrid * 8 * kIters * 64 * 32768.0 / (ms * 1e-3) / 1e12;
    return MT_OK;
}

uint32_t mt_debug_big_tile_rows(uint32_t rows, uint32_t out_features)
{
    return fc_is_big(rows, round_up(out_features, (uint32_t)kBrickRows)) ? big_rows(rows) : 0;
}

uint32_t mt_debug_big_tile_walk(uint32_t in_features)
{
    return round_up(in_features, (uint32_t)kWidthAlign) >= kBigWalkMinK ? 1 : 0;
}

int mt_debug_conv_row_tiling(uint32_t in_h, uint32_t in_w, uint32_t in_channels, uint32_t ksize, uint32_t stride, uint32_t elem_size,
                             uint32_t* rows_per_tile, uint32_t* images_per_tile, uint32_t* tiles_per_image, uint64_t* frame_bytes)
{
    RowTiling r{0, 0, 0};
    uint64_t frame = 0;
    if (ksize >= 1 && (ksize & 1) && (stride == 1 || stride == 2) && (elem_size == 2 || elem_size == 4) && in_h && in_w && in_channels) {
        LayerDev d{};
        const uint32_t pad = (ksize - 1) / 2;
        const uint32_t oh = (in_h + 2 * pad - ksize) / stride + 1, ow = (in_w + 2 * pad - ksize) / stride + 1;
        d.kind = MT_CONV2D; d.cin = round_up(in_channels, (uint32_t)kChanPad); d.in_h = in_h; d.in_w = in_w; d.stride = stride;
        d.out_w = ow; d.ksize = ksize; d.pad = pad; d.rows_per_req = oh * ow;
        const uint32_t packed = choose_row_tiling(d, elem_size);
        if (packed) { r = unpack_row_tiling(packed); frame = row_tile_frame_bytes(d, elem_size, r); }
    }
    if (rows_per_tile) *rows_per_tile = r.n_oh;
    if (images_per_tile) *images_per_tile = r.ni;
    if (tiles_per_image) *tiles_per_image = r.tpi;
    if (frame_bytes) *frame_bytes = frame;
    return r.n_oh != 0;
}

mt_status mt_debug_poison(mt_ctx* c)
{
    if (!c) return MT_EINVAL;
    if (c->host_only) return fail(c, MT_ESTATE, "host-only context");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipDeviceSynchronize());
    const size_t act_bytes = (size_t)c->P_cap * c->S * c->elem_size;
    for (RunSlot& r : c->slots) {
        for (uint32_t i = 0; i < c->act_buffers; ++i) HIP_TRY(c, hipMemset(r.d_act[i], 0xFF, act_bytes));
        HIP_TRY(c, hipMemset(r.d_logits, 0xFF, (size_t)c->P_cap * c->C_pad * 4));
    }
    HIP_TRY(c, hipDeviceSynchronize());
    return MT_OK;
}

mt_status mt_cache_stats_get(const mt_ctx* c, mt_cache_stats* out)
{
    if (!c || !out) return MT_EINVAL;
    *out = mt_cache_stats{};
    for (const HostTenant& t : c->tenants) if (t.registered && t.resident) out->resident_models++;
    out->uploads = c->n_uploads; out->upload_bytes = c->upload_bytes; out->evictions = c->n_evictions;
    return MT_OK;
}

mt_status mt_get_stats(const mt_ctx* c, mt_stats* out)
{
    if (!c || !out) return MT_EINVAL;
    out->n_tenants = c->n_registered;
    out->arena_used = c->arena_used;
    out->arena_bytes = c->cfg.arena_bytes;
    out->last_run_rows = c->last_run_rows;
    out->last_run_launches = c->last_run_launches;
    return MT_OK;
}

}  // extern "C"
