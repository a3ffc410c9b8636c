// Device-side helpers shared by the kernels of the multi-tenant worker runtime, written for
// gfx950 (CDNA4, wave64).  The kernels live in:
//
//   batcher.hip     batcher_kernel (+ rank_kernel, place_kernel for large batches): tenant
//                   segmentation of the pending requests (counts, 32-aligned offsets, stable
//                   permutation) and the per-layer grouped-work tile lists, on device
//   fc_stream.hip   fc_kernel: one FC layer index for all tenants, weight-streaming tiles: weight
//                   bricks go from memory into MFMA operands through a register ring, activation
//                   bricks are shared through LDS; fused bias + activation (+ rounding), brick
//                   output, fp32 logits, or softmax/argmax for at most 32 classes
//   fc_big.hip      fc_big_walk_kernel / fc_big_kernel: the same layer index, compute-bound tenant-layers:
//                   256x256 tiles, both operands through an LDS ring filled by direct global->LDS loads;
//                   one workgroup per compute unit walks the tiles (or, for short K, one workgroup per tile)
//   conv.hip        conv_kernel (layers at most 32 channels wide: every wave gathers its own
//                   pixels) and conv_lds_kernel (wider layers: activation bricks gathered once
//                   per tile into LDS and shared by waves side by side over channels; pools on
//                   the way out where it can) and conv_img_kernel (layers whose tiles are whole
//                   output rows of an image or whole small images: the tile's input rows are
//                   copied to LDS once and every tap is read from there): implicit-GEMM 3x3
//                   convolution for all tenants
//   small.hip       gather_kernel / gather_image_kernel (submitted rows -> bricks / padded NHWC),
//                   gap_kernel (global average pooling), head_kernel (softmax + argmax in
//                   submission order), copy_kernel (the yardstick for byte counters)
//
// A DNN is a fixed sequence of layers applied in turn (paper, section 1.1); a worker
// hosts many tenants' DNNs and multiplexes their requests (section 3).  The grouping
// of all tenants' work for one layer index into one launch is this runtime's way of
// doing that multiplexing on one GPU.
#pragma once
#include <algorithm>
#include "mt_internal.h"

namespace mt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kBatchThreads = 1024;
constexpr uint32_t kMaxTenantsPadded = 2048;
constexpr uint32_t kSegsInLds = 64;

__device__ __forceinline__ uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

// One of the run's activation buffers by its number (a layer names the ones it reads and writes);
// selects instead of indexing, so that the kernel arguments stay in scalar registers.
__device__ __forceinline__ void* act_of(const ActBufs& b, uint32_t i)
{
    return i == 0 ? b.p[0] : i == 1 ? b.p[1] : i == 2 ? b.p[2] : b.p[3];
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every global
// load in flight (it fences all address spaces), which would empty the prefetch rings of the
// GEMM loops at each LDS hand-over; here only the LDS counter is waited on.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Direct global -> LDS load of 16 bytes per lane: lane l's bytes land at lds_dst + 16 l
// (lds_dst is wave-uniform and travels in M0).  Written as asm on purpose: the compiler's
// wait-count pass gives up exact vmcnt bookkeeping (it waits for zero) once it sees such loads
// in flight together with ordinary register loads.  A kernel that uses this helper issues no
// register loads while such loads are in flight and waits for the LDS data itself, with an
// explicit vmcnt before the barrier that publishes it.  Nothing else keeps a value in M0.
__device__ __forceinline__ void lds_dma16(const __attribute__((address_space(1))) void* src, void* lds_dst)
{
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(m0v), "v"(src) : "memory", "m0");
}

// The same through a buffer descriptor: lane l's 16 bytes at byte `voff` of the buffer land at lds_dst + 16 l, and a
// lane whose offset lies outside the buffer gets zeros (the hardware's range check of untyped buffers; checked on
// the device: the lane layout is that of the global form, offsets from num_records - 15 on deliver zeros).
// The descriptor: base address, stride 0 (untyped), size in bytes, 32-bit data format.
__device__ __forceinline__ u32x4 buffer_descriptor(const void* base, uint32_t bytes)
{
    const uint64_t b = (uint64_t)base;
    u32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((uint32_t)b);
    d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32) & 0xffffu);
    d[2] = __builtin_amdgcn_readfirstlane(bytes);
    d[3] = 0x00020000u;
    return d;
}
__device__ __forceinline__ void lds_dma16_buffer(const u32x4& desc, uint32_t voff, void* lds_dst)
{
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(m0v), "v"(voff), "s"(desc) : "memory", "m0");
}

// Inclusive prefix sums across lanes with data-parallel-primitive moves (no LDS traffic): shifts
// by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then lane 15 of rows
// 0 and 2 is added to rows 1 and 3, then lane 31 to the upper half.
#define MT_DPP_ADD(v, ctrl, rows) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, rows, 0xf, false)
__device__ __forceinline__ uint32_t row16_inclusive_scan(uint32_t v)
{
    MT_DPP_ADD(v, 0x111, 0xf); MT_DPP_ADD(v, 0x112, 0xf); MT_DPP_ADD(v, 0x114, 0xf); MT_DPP_ADD(v, 0x118, 0xf);   // row_shr:1,2,4,8
    return v;
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v = row16_inclusive_scan(v);
    MT_DPP_ADD(v, 0x142, 0xa);      // row_bcast:15 into rows 1 and 3
    MT_DPP_ADD(v, 0x143, 0xc);      // row_bcast:31 into rows 2 and 3
    return v;
}
#undef MT_DPP_ADD

// How an FC layer is cut into workgroup tiles: `split` column blocks side by side per
// group (the four waves cover them; with split < 4 they also split K), `groups` column
// groups, and the rows of a tile: 64 normally, 32 for the K-split shapes (layers with at
// most 64 outputs): their tiles are short-lived and latency bound, so more and smaller ones
// finish sooner.
__device__ __forceinline__ void fc_shape(uint32_t n_pad, uint32_t split_k, uint32_t* split, uint32_t* groups, uint32_t* tile_rows)
{
    const uint32_t nblk = n_pad / kBrickRows;
    uint32_t s = split_k ? 1u : (nblk >= 3 ? 4u : nblk);
    *split = s;
    *groups = ceil_div(nblk, s);
    *tile_rows = s == 4 ? kTileRows : kTileRows / 2;
}

// ---- shared pieces of the GEMM kernels -----------------------------------------------------
// GELU(x) = x * Phi(x) with the exact (erf) definition, evaluated through the complementary
// error function of z = |x|/sqrt(2) (Abramowitz & Stegun 7.1.26: a degree-5 polynomial in
// t = 1/(1 + p z) times exp(-z^2), absolute error below 1.5e-7).  With h = erfc(z)/2, Phi is
// 1 - h on the positive side and h on the negative one, so x Phi(x) = max(x, 0) - |x| h on both
// (the small negative tail keeps its relative accuracy).  z is carried pre-scaled by
// sqrt(log2 e) so that exp(-z^2) is one multiply and one exp2; the 1/2 sits in the polynomial's
// coefficients.  The error is far below half a bfloat16 ulp of the result, and a library erf
// costs four times as much, which showed in the epilogue of the compute-bound tiles.
// max(x, 0) in one instruction: the compiler's own maximum first quiets a possible signalling NaN with a second
// v_max (it cannot know that MFMA results hold none), one issue slot in fifteen of the GELU below.
__device__ __forceinline__ float max0(float x)
{
    float r;
    asm("v_max_f32 %0, 0, %1" : "=v"(r) : "v"(x));
    return r;
}

__device__ __forceinline__ float gelu(float x)
{
    constexpr float kScale = 0.84932180028801904f;           // sqrt(log2(e) / 2): zs = z * sqrt(log2 e)
    constexpr float kP = 0.3275911f / 1.2011224087864498f;   // p / sqrt(log2 e)
    const float ax = fabsf(x);
    const float zs = ax * kScale;
    const float t = __builtin_amdgcn_rcpf(fmaf(kP, zs, 1.0f));   // one instruction, within 1 ulp: far inside the formula's own 1.5e-7
    const float poly = t * (0.127414796f + t * (-0.142248368f + t * (0.7107068705f + t * (-0.7265760135f + t * 0.5307027145f))));
    const float h = poly * __builtin_amdgcn_exp2f(-zs * zs);
    return fmaf(-ax, h, max0(x));
}

__device__ __forceinline__ float activate(float z, uint32_t act)
{
    if (act == MT_ACT_RELU) return max0(z);
    if (act == MT_ACT_GELU) return gelu(z);
    return z;
}

// The same on a block of values, with the choice made once, outside the loops.
template <int G>
__device__ __forceinline__ void activate_block(f32x4 (&y)[G], uint32_t act)
{
    if (act == MT_ACT_GELU) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) y[g][e] = gelu(y[g][e]);
    } else if (act == MT_ACT_RELU) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) y[g][e] = max0(y[g][e]);
    }
}

// A residual addition done by the convolution in front of it.  y holds this lane's four runs of four
// channels (8 g + 4 lh + {0..3}) of one pixel, bias and the convolution's activation applied: they are
// rounded to T, as the addition would have read them, the other operand's values of the same pixel and
// channels are added, and the addition's activation follows.  `skip` points into the other operand
// where `out` points into the output (null for lanes without a pixel); channels from `nvalid` on do not exist.
template <typename T>
__device__ __forceinline__ void add_residual(f32x4 (&y)[4], const T* skip, uint32_t lh, uint32_t nvalid, uint32_t act)
{
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if (skip != nullptr && 8 * g + 4 * lh < nvalid) {        // channel counts are multiples of 8: a run exists whole or not at all
            T sv[4];
            if constexpr (sizeof(T) == 2) *(uint64_t*)sv = *(const uint64_t*)(skip + 8 * g + 4 * lh);
            else *(u32x4*)sv = *(const u32x4*)(skip + 8 * g + 4 * lh);
#pragma unroll
            for (int e = 0; e < 4; ++e) y[g][e] = (float)(T)y[g][e] + (float)sv[e];
        }
    }
    activate_block<4>(y, act);
}

template <typename T> struct Mma;
// bf16: one 16-byte chunk is a whole MFMA operand (8 consecutive k of one row).
template <> struct Mma<__bf16> {
    static __device__ __forceinline__ void run(f32x16& acc, const u32x4& a, const u32x4& b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
};
// fp32: a chunk holds 4 consecutive k; four 32x32x2 MFMAs consume it, the two lane halves
// supplying the two k slots of each (the same k assignment on both operands).
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(f32x16& acc, const u32x4& a, const u32x4& b)
    {
        const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[0], bf[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[1], bf[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[2], bf[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[3], bf[3], acc, 0, 0, 0);
    }
};

// What a workgroup works on, derived from its block index and the list's tile_base array.
struct Tile {
    uint32_t tenant, m0, rows, n0, split;
};

// XCD-aware numbering: consecutive block indices go to different XCDs (each with its own L2),
// so the logical tile index is chosen such that every XCD gets one contiguous run of tiles;
// tiles that re-read the same weight panel (the row tiles of one column group) then
// share an L2.  Returns false for blocks past the end of the list.
__device__ __forceinline__ bool logical_tile(uint32_t n_tiles, uint32_t* logical)
{
    const uint32_t per_xcd = (n_tiles + 7) / 8, b = blockIdx.x;
    *logical = (b & 7) * per_xcd + (b >> 3);
    return (b >> 3) < per_xcd && *logical < n_tiles;
}

// Variant for the big-tile kernel: the tile order is dealt to the XCDs in chunks of kXcdChunk
// tiles (round robin), so that at any time the whole GPU works on a narrow window of the order
// (about two tenants' panels, which fit the memory-side cache) while the tiles that run together
// on one XCD are still neighbours (L2 reuse).  The grid must be a multiple of 8 * kXcdChunk.
constexpr uint32_t kXcdChunk = 64;
__device__ __forceinline__ bool logical_tile_chunked(uint32_t n_tiles, uint32_t* logical)
{
    const uint32_t b = blockIdx.x, xcd = b & 7, i = b >> 3;
    *logical = ((i / kXcdChunk) * 8 + xcd) * kXcdChunk + (i % kXcdChunk);
    return *logical < n_tiles;
}

// Tenant that owns logical tile `idx` by binary search over a copy of the list in LDS: last t with
// base[t] <= idx (base[T] > idx).  Kept for the big-tile kernel, whose tiles run for ~100 us and
// whose wait counts the compiler only keeps exact while the kernel issues no other register loads
// than the one staging loop at its head.
__device__ __forceinline__ uint32_t find_tenant(const uint32_t* base, uint32_t T, uint32_t idx)
{
    uint32_t lo = 0, hi = T;
    while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (base[mid] <= idx) lo = mid; else hi = mid; }
    return lo;
}

// Tenant that owns a logical tile.  A tile list base[0..T] is non-decreasing with base[0] = 0 and
// base[T] = the number of tiles, so the owner of tile idx is the number of entries base[1..T]
// that are <= idx.  The workgroup counts them together: every thread fetches its entries
// (tile_owner_fetch, all loads issued before anything waits, and before the tile index is
// known), the waves count with one ballot per entry slot and add their counts through `part`
// (LDS, one word per wave, not reused by the caller: no second barrier is needed).  One memory
// round trip and one barrier; a binary search over a copy of the list in LDS took a dozen
// dependent LDS reads and two barriers at the head of every tile.
template <uint32_t THREADS>
struct TileOwner {
    static constexpr uint32_t SLOTS = kMaxTenantsPadded / THREADS;
    uint32_t v[SLOTS];
    __device__ __forceinline__ void fetch(const uint32_t* __restrict__ base, uint32_t T)
    {
#pragma unroll
        for (uint32_t s = 0; s < SLOTS; ++s) {
            const uint32_t j = 1 + s * THREADS + threadIdx.x;
            v[s] = 0xffffffffu;
            if (s * THREADS < T && j <= T) v[s] = base[j];
        }
    }
    // wave-uniform result; every thread of the workgroup must call it
    __device__ __forceinline__ uint32_t owner(uint32_t T, uint32_t idx, uint32_t* part) const
    {
        uint32_t cnt = 0;
#pragma unroll
        for (uint32_t s = 0; s < SLOTS; ++s)
            if (s * THREADS < T) cnt += (uint32_t)__builtin_popcountll(__ballot(v[s] <= idx));
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = cnt;
        __syncthreads();
        uint32_t t = 0;
#pragma unroll
        for (uint32_t w = 0; w < THREADS / 64; ++w) t += part[w];
        return __builtin_amdgcn_readfirstlane(t);
    }
};

}  // namespace mt
