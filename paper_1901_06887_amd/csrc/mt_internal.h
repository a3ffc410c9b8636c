// Internal declarations shared by the host runtime (mt_api.cpp) and the device code
// (mt_kernels.hip).  Not part of the public ABI.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#include "../../include/mt.h"

namespace mt {

// ---- tile geometry of the grouped GEMM (all sizes in elements unless noted) ----
constexpr int kBM = 128;            // rows of a workgroup tile
constexpr int kBN = 128;            // columns of a workgroup tile
constexpr int kRowBytes = 128;      // bytes of K one pipeline step consumes per row
constexpr int kChanPad = 8;         // conv input channels are padded to a multiple of this
constexpr int kWidthAlign = 64;     // activation rows are zero-filled up to a multiple of this

// One layer of one tenant, as the kernels see it (lives in device memory).
struct LayerDev {
    uint32_t kind, act;
    uint32_t K;          // reduction length actually stored per weight row (padded, elements)
    uint32_t N;          // output features (FC) / output channels (CONV)
    uint32_t in_h, in_w; // CONV / GAP input geometry
    uint32_t cin;        // CONV: padded input channels (multiple of kChanPad); GAP: channels
    uint32_t stride;     // CONV
    uint32_t out_w;      // CONV output width
    uint32_t rows_per_req;  // GEMM rows one request contributes: 1 (FC) or out_h*out_w (CONV)
    uint32_t out_len;    // elements one request's output occupies
    uint32_t out_fill;   // out_len rounded up to kWidthAlign (zero-filled tail)
    uint32_t is_last;    // outputs are the logits
    uint32_t pad0;
    uint64_t w_off;      // byte offset of the packed weights in the arena
    uint64_t b_off;      // byte offset of the fp32 bias in the arena
};

struct TenantDev {
    uint32_t registered;
    uint32_t n_layers;
    uint32_t in_len;     // elements of one request's input as submitted
    uint32_t n_classes;
    uint32_t in_cin;     // first layer CONV with channel padding: submitted channels, else 0
    uint32_t in_cin_pad; // ... and the padded count
    uint32_t in_fill;    // elements of the staged input row incl. zero tail
    uint32_t pad0;
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

// One unit of grouped-GEMM work.
struct Tile {
    uint32_t tenant;
    uint32_t m0;      // first GEMM row inside the tenant's segment
    uint32_t rows;    // valid rows (<= kBM)
    uint32_t n0;      // first output column
};

struct BatchArgs {
    const Segment* segs; uint32_t n_segs; uint32_t R; uint32_t T; uint32_t n_layer_slots;
    Segment first;         // copy of segs[0]: the common one-segment run never reads host memory
    const void** row_src;  // [R] device address of each submitted row's input
    uint32_t elem_size;
    const TenantDev* tenants; const LayerDev* layers;
    int32_t* row_tenant;   // [R] tenant of each submitted row, -1 if rejected
    uint32_t* row_rank;    // [R] scratch
    int32_t* pos_of;       // [R] packed position of each submitted row, -1 if rejected
    uint32_t* perm;        // [R] packed position -> submission index
    uint32_t* M;           // [T]
    uint32_t* off;         // [T+1]
    Tile* tiles; uint32_t tile_cap;   // n_layer_slots lists of tile_cap entries
    uint32_t* n_tiles;     // [n_layer_slots]
    uint32_t* overflow;    // set to 1 if a tile list would not fit (never expected)
};

struct GatherArgs {
    const void* const* row_src; uint32_t R;
    const TenantDev* tenants; const int32_t* row_tenant; const uint32_t* perm; const uint32_t* off; uint32_t T;
    void* act; uint32_t S; uint32_t elem_size;
};

struct GemmArgs {
    const Tile* tiles; const uint32_t* n_tiles; uint32_t layer;
    const LayerDev* layers; const uint32_t* off;
    const void* act_in; void* act_out; const uint8_t* arena;
    float* logits; uint32_t S; uint32_t C_pad;
};

struct GapArgs {
    uint32_t layer; uint32_t R; const LayerDev* layers; const TenantDev* tenants;
    const int32_t* row_tenant; const uint32_t* perm; const uint32_t* off; uint32_t T;
    const void* act_in; void* act_out; uint32_t S; uint32_t elem_size;
};

struct HeadArgs {
    uint32_t R; const TenantDev* tenants; const int32_t* row_tenant; const int32_t* pos_of;
    const float* logits; uint32_t C_pad;
    int32_t* labels; float* probs; float* logits_out; int32_t* n_classes; uint32_t row_stride;
};

// Launchers (defined in mt_kernels.hip).  All enqueue on `s` and return the launch status.
hipError_t launch_batcher(const BatchArgs& a, hipStream_t s);
hipError_t launch_gather(const GatherArgs& a, hipStream_t s);
hipError_t launch_gemm(const GemmArgs& a, uint32_t dtype, uint32_t grid, hipStream_t s);
hipError_t launch_gap(const GapArgs& a, hipStream_t s);
hipError_t launch_head(const HeadArgs& a, hipStream_t s);

}  // namespace mt
