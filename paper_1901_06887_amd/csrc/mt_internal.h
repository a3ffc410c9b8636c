// Internal declarations shared by the host runtime (mt_api.cpp) and the device code
// (the .hip files, through mt_device.h).  Not part of the public ABI.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#include "../../include/mt.h"

namespace mt {

// ---- geometry ---------------------------------------------------------------------------
// "Brick": the unit of the fully-connected data layout.  A brick is one MFMA operand of a
// whole wavefront, stored contiguously: 32 rows x KB reduction elements as 64 lanes x 16
// bytes, lane = row + 32*half, each lane holding EPC = 16/sizeof(T) consecutive k (KB =
// 2*EPC: 16 for bf16, 8 for fp32).  A matrix [rows][K] is stored as
// bricks[row_block][k_block][lane][EPC].  Weights are packed this way at registration and
// fully-connected activations are produced this way by the gather, the pooling kernel and
// the FC epilogue, so the hot loop issues nothing but 1 KiB contiguous wavefront loads that
// land directly in MFMA operand order.
constexpr int kBrickRows = 32;
constexpr int kBrickBytes = 1024;
constexpr int kTileRows = 64;       // rows (2 row blocks) of a grouped-GEMM workgroup tile: 128-row tiles leave room for only 8 weight
                                    // bricks in flight per wave, which made them the slowest tiles of a launch
constexpr int kTileCols = 128;      // columns (4 column blocks) of a workgroup tile
constexpr int kConvTileRows = 128;  // GEMM rows (output pixels) of a conv workgroup tile: one 32-row block per wave (512 measured slower)
// A tenant-layer with at least kBigMinRows requests and kBigMinCols (padded) outputs is
// compute bound; it is cut into kBigTile x kBigTile tiles and served by the big-tile FC kernel.
constexpr int kBigTile = 256;
constexpr int kBigMinRows = 2048;
// ... except a last row tile of at most kBigRemRows rows: alone on a compute unit it would take a
// whole tile's time (and, at the end of a launch, hold the chip for a round of its own), so
// those rows go to the streaming kernel, which reads the tenant's weights once more instead.
constexpr int kBigRemRows = 128;
constexpr int kBigMinCols = 192;
constexpr int kBigMinTiles = 512;   // a layer index is served with big tiles only when it has at least two per compute unit
constexpr double kRidgeFlopsPerByte = 312.0;   // dense bf16 MFMA peak over HBM bandwidth (2.5 PFLOP/s / 8 TB/s)
constexpr int kBigMinBatch = 8192;  // runs with fewer rows are latency/HBM bound as a whole: no big tiles
inline __host__ __device__ bool fc_is_big(uint32_t rows, uint32_t n_pad) { return rows >= (uint32_t)kBigMinRows && n_pad >= (uint32_t)kBigMinCols; }
// Rows of a big tenant-layer that the big tiles serve: all of them, unless the last row tile
// would hold at most kBigRemRows rows; those rows are left to the streaming kernel.
inline __host__ __device__ uint32_t big_rows(uint32_t rows)
{
    const uint32_t rem = rows % kBigTile;
    return rem && rem <= (uint32_t)kBigRemRows ? rows - rem : rows;
}
// The rows that big tiles leave to the streaming kernel (at most kBigRemRows per tenant) meet the whole of the
// layer's weights.  Where the layer has many column groups those tiles fill the chip and are bound by the weight
// stream, which ordinary 64-row tiles read the fewest times.  A narrow layer (the 1000 classes of the last one:
// 8 column groups, a few dozen tiles) leaves most of the chip idle while each tile walks all of K: there the rows
// are tiled 32 at a time and one column block wide with K split among the waves, as in runs of few tiles
// (c5's last layer: 35 -> 19 us; the hidden layers would go from 39 to 44 us, their weights read once more).
constexpr int kBigRemSplitMaxCols = 1024;
inline __host__ __device__ bool big_remainder_split_k(uint32_t n_pad) { return n_pad <= (uint32_t)kBigRemSplitMaxCols; }
constexpr int kRankRows = 1024;     // rows per workgroup of the ranking kernel
constexpr int kRankMinRows = 8192;  // smaller batches are ranked by the batcher's single workgroup (one launch less)
constexpr int kRankMaxTenants = 512;
constexpr int kHistEntries = 8192;  // histogram words the batcher holds in LDS (waves or ranking workgroups x padded tenants)
constexpr int kListKinds = 3;       // tile lists per layer index: FC (streaming), conv, FC (big tiles)
constexpr int kActBuffers = 4;      // most activation buffers of a run: layer outputs that may be alive at once
constexpr int kLayerGroup = 8;      // the batcher builds the tile lists of this many layer indices per pass
constexpr int kBigMaxLayer = 32;    // layer indices from here on never take big tiles (their decisions travel in one 32-bit mask)
constexpr int kRowBytes = 128;      // conv path: bytes of K one pipeline step consumes per row
constexpr int kChanPad = 8;         // conv input channels are padded to a multiple of this
constexpr int kWidthAlign = 64;     // K and activation widths are zero-padded to a multiple of this

// How a convolution layer is cut into tiles of whole output rows: a tile holds `ni` sub-images, each `n_oh` output
// rows of one image (ni > 1: whole images of at most 128 / ni pixels, n_oh = the image's height); an image takes
// `tpi` tiles.  Pixel slot p of a tile (0..127): sub-image p / (128 / ni), pixel p % (128 / ni) of its n_oh rows.
struct RowTiling { uint32_t n_oh, ni, tpi; };
inline __host__ __device__ uint32_t pack_row_tiling(RowTiling r) { return r.n_oh | r.ni << 8 | r.tpi << 16; }
inline __host__ __device__ RowTiling unpack_row_tiling(uint32_t p) { return RowTiling{p & 0xffu, (p >> 8) & 0xffu, p >> 16}; }
// GEMM rows per request by which the tile lists count a convolution layer's tiles (128 per tile): the layer's
// output pixels, or, with row tiling, 128 per tile of an image (tiles may be partly empty), 128 / ni for small images.
inline __host__ __device__ uint32_t conv_tile_rows(uint32_t rows_per_req, uint32_t row_tiles)
{
    if (!row_tiles) return rows_per_req;
    const RowTiling r = unpack_row_tiling(row_tiles);
    return r.ni > 1 ? (uint32_t)kConvTileRows / r.ni : r.tpi * (uint32_t)kConvTileRows;
}
constexpr uint32_t kConvFrameMaxBytes = 96 * 1024;   // most LDS that the input rows of one such tile may take

enum : uint32_t { kLayoutRows = 0, kLayoutBricks = 1 };
constexpr uint32_t kKindNone = 0xffu;     // a layer index at which this tenant has nothing to run (its work was taken over by the layer before)

// One layer of one tenant, as the kernels see it (lives in device memory).
struct LayerDev {
    uint32_t kind, act;
    uint32_t K;          // reduction length as stored (padded to kWidthAlign), elements
    uint32_t k_valid;    // FC: true fan-in; CONV: 9 * cin (the rest of K is zero padding)
    uint32_t N;          // output features (FC) / output channels (CONV)
    uint32_t N_pad;      // FC: weight rows as stored (multiple of 32; of 64 for hidden layers)
    uint32_t in_h, in_w; // CONV / GAP input geometry
    uint32_t cin;        // CONV: padded input channels (multiple of kChanPad); GAP: channels
    uint32_t stride;     // CONV
    uint32_t out_w;      // CONV output width
    uint32_t rows_per_req;  // GEMM rows one request contributes: 1 (FC) or out_h*out_w (CONV)
    uint32_t out_len;    // elements one request's output occupies
    uint32_t out_fill;   // out_len rounded up to kWidthAlign (zero-filled tail)
    uint32_t is_last;    // outputs are the logits
    uint32_t pool_fill;  // CONV whose next layer is a global average pool that the convolution can do itself (whole images
                         // per wave: 32 or 64 output pixels per image, channels a multiple of 64): the pool's out_fill, else 0
    uint32_t ksize;      // CONV / MAXPOOL: window (ksize x ksize)
    uint32_t pad;        // CONV / MAXPOOL
    // which of the run's activation buffers the layer reads (in2_buf: the second operand of ADD) and writes;
    // pool_buf: where a convolution that pools by itself writes (the out_buf of the pooling layer behind it)
    uint32_t in_buf, in2_buf, out_buf, pool_buf;
    // CONV whose output goes to a residual addition and nowhere else: the convolution adds the other operand
    // (buffer in2_buf, same pixel and channel) to its rounded output itself and applies the addition's
    // activation; 1 + that activation, else 0.  The addition's own row then has kind kKindNone.
    uint32_t fuse_add;
    // CONV whose tiles can be whole output rows of one image, or whole small images, with the input rows they need
    // held in LDS (RowTiling, packed; 0: its tiles are runs of 128 pixels).  The tile lists count such a layer's
    // tiles by conv_tile_rows() whichever kernel serves the layer index.
    uint32_t row_tiles;
    uint64_t w_off;      // byte offset of the packed weights in the arena
    uint64_t b_off;      // byte offset of the fp32 bias in the arena (N_pad entries for FC)
};

struct TenantDev {
    uint32_t registered;
    uint32_t n_layers;
    uint32_t in_len;     // elements of one request's input as submitted
    uint32_t n_classes;
    uint32_t in_cin;     // first layer CONV with channel padding: submitted channels, else 0
    uint32_t in_cin_pad; // ... and the padded count
    uint32_t in_fill;    // elements of the staged input row incl. zero tail
    uint32_t in_layout;  // kLayoutBricks if the first layer is FC, else kLayoutRows
};

// One run of submitted rows (lives in pinned host memory, read by the batcher kernel).
struct Segment {
    const int32_t* ids;   // device, per-row tenant ids, or nullptr
    const void* src;      // device, first input row
    uint32_t row_begin;   // submission index of the first row
    uint32_t n_rows;
    uint32_t row_stride;  // elements between rows
    int32_t tenant;       // used when ids == nullptr
};

// Where predictions go (caller's buffers, submission order).
struct OutPtrs {
    int32_t* labels; float* probs; float* logits; int32_t* n_classes; uint32_t row_stride;
};

// Grouped work of one layer index is described by one array per kind (FC, conv):
// tile_base[t] = number of workgroup tiles of all tenants before t, tile_base[T] = total.
// A workgroup finds its tenant by searching that array and derives its tile from the rest:
//   FC:   tiles of a tenant are numbered column-group-major, 64-row tile minor; a column
//         group is `split` column blocks of 32 (4, 2 or 1) that the four waves cover side
//         by side, the remaining factor 4/split splitting K between the waves.
//   CONV: kConvTileRows x kTileCols output tiles of the implicit GEMM, column-major likewise.
struct BatchArgs {
    const Segment* segs; uint32_t n_segs; uint32_t R; uint32_t T; uint32_t n_layer_slots;
    Segment first;         // copy of segs[0]: the common one-segment run never reads host memory
    uint32_t elem_size;
    uint32_t fc_split_k;   // 1: FC tiles take one column block each and split K four ways
    uint32_t big_enabled;  // 0: no tenant-layer is given big tiles in this run (small batches)
    uint32_t big_min_tiles; // a layer index uses big tiles only when its qualifying tenants make at least this many
    const TenantDev* tenants;
    // What the tile lists need to know of every tenant-layer: two words per layer, 64 bytes per
    // tenant, facts[tenant][layer][2].  Word 0: column groups of the layer's tiles (0: no tiles:
    // pooling, or no such layer), bit 31: convolution, bit 30: FC tiles of 32 rows instead of 64.
    // Word 1: GEMM rows per request (convolution) or padded outputs (FC).
    const uint32_t* facts;
    unsigned long long* served;   // [T][2]: requests served and runs with requests, per tenant, over all runs (atomic adds: runs may overlap)
    int32_t* row_tenant;   // [R] tenant of each submitted row, -1 if rejected
    uint32_t* row_rank;    // [R] scratch
    // Large batches are ranked by a kernel of their own, kRankRows rows per workgroup, before the
    // batcher proper: n_rank_groups workgroups (0: the batcher ranks the rows itself), each leaving
    // the rank of a row among its workgroup's rows of the same tenant in row_rank and its tenant
    // histogram in hist_g[group][Tp] (Tp: the tenant count padded to a power of two, at least 64).
    // The batcher turns hist_g into prefixes over the groups, and a third kernel places the rows.
    uint32_t n_rank_groups; uint32_t* hist_g;
    const void** row_src;  // [R] device address of each submitted row's input
    int32_t* pos_of;       // [R] packed position of each submitted row, -1 if rejected
    int32_t* perm;         // [P] packed position -> submission index, -1 for padding rows
    uint32_t* M;           // [T]
    uint32_t* off;         // [T+1] packed position of each tenant's first row (multiple of 32)
    uint32_t* tile_base;   // [kListKinds][MT_MAX_LAYERS][T+1]: FC, conv, big-FC arrays
    uint32_t* big_layers;  // [1] out: bit l set if layer index l is served with big tiles where a tenant qualifies
    uint32_t list_mask[MT_MAX_LAYERS / kLayerGroup];   // per group of layer indices: bit kind*kLayerGroup + l%kLayerGroup set if any registered model can have such tiles at layer l
    OutPtrs out;           // rejected rows are answered here (label -1, zero rows)
};

// The run's activation buffers; a layer names the ones it reads and writes (LayerDev::in_buf ...).
struct ActBufs { void* p[kActBuffers]; };

struct GatherArgs {
    const void* const* row_src; uint32_t P;      // P = upper bound of packed rows (multiple of 32)
    const TenantDev* tenants; const LayerDev* layers; const int32_t* row_tenant; const int32_t* perm;
    const uint32_t* off; uint32_t T;
    void* act; uint32_t S; uint32_t elem_size;
    const void* zeros;     // >= 16 readable zero bytes
};

struct GemmArgs {
    const uint32_t* tile_base; uint32_t T; uint32_t layer; uint32_t fc_split_k;
    const uint32_t* big_layers;   // the batcher's decision per layer index (see BatchArgs)
    uint32_t big_vgrid;           // big-tile launch whose workgroups walk several tiles: the grid of one tile per workgroup that they walk
    uint32_t pool;                // conv launch: the layers with pool_fill write the pooled activation instead of their own
    uint32_t img_lds;             // conv launch with LDS-resident input: bytes of dynamic LDS (the largest frame)
    // FC layer 0 can read the submitted rows itself (16-byte aligned rows whose length is a
    // whole number of 16-byte chunks), which saves the staging pass:
    uint32_t gather; const int32_t* perm; const void* const* row_src;
    // a last layer whose classes all lie inside one tile finishes its rows itself (softmax, argmax,
    // outputs): at most fuse_head_max classes (32: one column block; 128: a whole tile of four, not
    // in runs whose tiles are single column blocks); out_vec_ok: output rows take 16-byte stores
    uint32_t fuse_head; uint32_t fuse_head_max; uint32_t out_vec_ok; OutPtrs out;
    const LayerDev* layers; const uint32_t* off; const uint32_t* M;
    ActBufs act; const uint8_t* arena;
    float* logits; uint32_t S; uint32_t C_pad;
    const void* zeros;     // >= 16 readable zero bytes
};

struct GapArgs {
    uint32_t layer; uint32_t P; const LayerDev* layers; const TenantDev* tenants;
    const int32_t* row_tenant; const int32_t* perm; const uint32_t* off; uint32_t T;
    ActBufs act; uint32_t S; uint32_t elem_size;
};

struct HeadArgs {
    uint32_t R; const TenantDev* tenants; const int32_t* row_tenant; const int32_t* pos_of;
    const float* logits; uint32_t C_pad;
    OutPtrs out;
    uint32_t min_classes;   // rows of models with fewer classes were finished by the FC kernel
    uint32_t vec_ok;        // output rows can be written 16 bytes at a time (aligned buffers, row stride a multiple of 4)
};

// Launchers (defined next to their kernels).  All enqueue on `s` and return the launch status.
hipError_t launch_batcher(const BatchArgs& a, hipStream_t s);   // three launches when a.n_rank_groups > 0
hipError_t launch_gather(const GatherArgs& a, uint32_t slices, hipStream_t s);   // `slices` workgroups share a block of 32 rows
hipError_t launch_gather_image(const GatherArgs& a, uint32_t slices, hipStream_t s);   // `slices` workgroups share a row
hipError_t launch_fc(const GemmArgs& a, uint32_t dtype, uint32_t grid, hipStream_t s);
hipError_t launch_fc_big(const GemmArgs& a, uint32_t dtype, uint32_t grid, uint32_t walk_grid, hipStream_t s);   // walk_grid > 0: that many workgroups walk the tiles (a multiple of 8)
hipError_t launch_copy(void* dst, const void* src, uint64_t bytes, hipStream_t s);
hipError_t launch_mfma_rate(float* out, uint32_t iters, uint32_t grid, hipStream_t s);   // out: grid * 512 floats
hipError_t prepare_conv(uint32_t dtype);   // once per device, before the first launch_conv: lets the frame kernels ask for more than 64 KiB of LDS
// max_cb: the widest tile of this layer index over the registered tenants, in 32-channel blocks (1..4)
// quad: every tenant's input channels at this layer index are a multiple of four 16-byte chunks
hipError_t launch_conv(const GemmArgs& a, uint32_t dtype, uint32_t max_cb, bool quad, uint32_t img_lds_bytes, bool img_two, bool long_k, bool uniform_walk, uint32_t grid, hipStream_t s);
hipError_t launch_gap(const GapArgs& a, hipStream_t s);
hipError_t launch_image_ops(const GapArgs& a, uint32_t slices, hipStream_t s);   // max-pool and residual add of one layer index
hipError_t launch_head(const HeadArgs& a, hipStream_t s);

}  // namespace mt
