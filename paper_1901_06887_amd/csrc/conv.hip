// Grouped k x k convolution as implicit GEMM (see mt_device.h for the overview).
#include "mt_device.h"
#include <type_traits>

namespace mt {

// ---- helpers of the implicit-GEMM convolutions ---------------------------------------------
// Quotient and remainder by a wave-uniform divisor; image sizes are mostly powers of two, and a
// general 32-bit division costs some thirty vector instructions per lane.
__device__ __forceinline__ void divmod_uniform(uint32_t x, uint32_t d, uint32_t* q, uint32_t* r)
{
    if ((d & (d - 1)) == 0) { *q = x >> __builtin_ctz(d); *r = x & (d - 1); }
    else { *q = x / d; *r = x - *q * d; }
}

// A lane's walk through K = (kernel row, kernel column, channel), one k step at a time.  Inside
// a kernel row the k taps of a pixel are one contiguous run of k * cin input elements, so the
// position is kept as (kernel row th, offset lin inside the run) and the element offset `cur`
// moves by KB per step plus a jump at the end of a run.  Validity is two range tests: the
// left/right taps fall outside the image only near the image's left/right edge, the top/bottom
// kernel rows only near its top/bottom edge.  Steps past the last tap have th == k: invalid.
template <typename T>
struct TapWalk {
    static constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    uint32_t lin, th, run, lo, hi, tlo, thi, step;
    int32_t cur, jump;
    // (ih0, iw0): the input coordinate of the window's top-left tap (may lie outside the image);
    // first: the lane's first element inside the run; step_el: elements per call of next()
    // (at most two runs end per call: step_el <= 2 * k * cin, which holds for every window and
    // channel count the layer set admits: a run is at least 8 elements, a step at most 32, and
    // steps of 32 are only taken where cin is a multiple of 32)
    __device__ __forceinline__ void init(const LayerDev& L, int32_t ih0, int32_t iw0, bool row_ok, uint32_t first, uint32_t step_el)
    {
        const int32_t cin = (int32_t)L.cin, k = (int32_t)L.ksize;
        run = L.ksize * L.cin; lin = first; th = 0; step = step_el;
        lo = (uint32_t)max(0, -iw0) * L.cin; hi = (uint32_t)max(0, min(k, (int32_t)L.in_w - iw0)) * L.cin;
        tlo = (uint32_t)max(0, -ih0); thi = row_ok ? (uint32_t)max(0, min(k, (int32_t)L.in_h - ih0)) : 0;
        cur = (ih0 * (int32_t)L.in_w + iw0) * cin + (int32_t)lin;
        jump = ((int32_t)L.in_w - k) * cin;
        wrap(); wrap();                                            // a first element past the first run (1x1 windows of 8 channels)
    }
    __device__ __forceinline__ void wrap()
    {
        const bool w = lin >= run;
        lin = w ? lin - run : lin; th += w ? 1u : 0u; cur = w ? cur + jump : cur;
    }
    // the 16-byte chunk of this k step inside the image, or -1 when the step reads zeros; moves on
    __device__ __forceinline__ int32_t next()
    {
        const bool ok = (lin >= lo) & (lin < hi) & (th >= tlo) & (th < thi);
        const int32_t chunk = ok ? (int32_t)((uint32_t)cur / EPC) : -1;
        lin += step; cur += (int32_t)step;
        wrap(); wrap();
        return chunk;
    }
};

// The same walk for a whole wave at once, where a step never straddles two taps (cin a multiple of the step): the
// position (tap, offset from the window's top-left tap) is then the same for every lane and lives in scalar
// registers; what differs between lanes is where their window starts and which taps fall outside the image, a
// 64-bit mask per lane (windows up to 7 x 7; steps past the last tap meet no bit).  A lane's load offset is one
// addition and one select: lanes outside the image ask for an offset outside the buffer and get zeros
// (lds_dma16_buffer).  TapWalk::next costs some twenty vector instructions per gathered brick, ten times the MFMAs
// the brick feeds; counters showed the vector unit busy half the time of a convolution launch.
struct UniformTapWalk {
    uint32_t tp, kw, ch, off;                    // tap index kh * k + kw; channel inside the tap; element offset from the top-left tap
    uint32_t cin, k, row_jump, step;
    __device__ __forceinline__ void init(const LayerDev& L, uint32_t step_el)
    {
        tp = 0; kw = 0; ch = 0; off = 0;
        cin = L.cin; k = L.ksize; row_jump = (L.in_w - L.ksize) * L.cin; step = step_el;
    }
    __device__ __forceinline__ void advance()
    {
        ch += step; off += step;
        if (ch == cin) {
            ch = 0; ++tp; ++kw;
            if (kw == k) { kw = 0; off += row_jump; }
        }
    }
};
// taps of a k x k window at (ih0, iw0) that lie inside the image, bit kh * k + kw
__device__ __forceinline__ uint64_t taps_inside(const LayerDev& L, int32_t ih0, int32_t iw0, bool row_ok)
{
    const int32_t k = (int32_t)L.ksize;
    const int32_t w_lo = max(0, -iw0), w_hi = max(0, min(k, (int32_t)L.in_w - iw0));
    const int32_t h_lo = max(0, -ih0), h_hi = row_ok ? max(0, min(k, (int32_t)L.in_h - ih0)) : 0;
    const uint64_t cols = w_hi > w_lo ? ((1ull << w_hi) - 1) & ~((1ull << w_lo) - 1) : 0;
    uint64_t m = 0;
    for (int32_t kh = 0; kh < k; ++kh)
        if (kh >= h_lo && kh < h_hi) m |= cols << (uint32_t)(kh * k);
    return m;
}

// ---- NHWC store of one 32-pixel x 32-channel unit held in the transposed accumulator layout ----
// After an MFMA with the filter brick as row operand, lane (li, lh) holds channels 8g + 4 lh +
// {0..3} of pixel li: stored from there, a wave instruction writes 64 separate 8- or 16-byte
// pieces, and the texture path counts (and takes time for) every one of them; the counters
// showed the convolution kernels bound by exactly that rate.  So the unit goes through a
// wave-private LDS scratch as [pixel][channel] rows and is read back so that consecutive
// lanes hold consecutive 16-byte chunks of a pixel's row: a pixel's 64 (bf16) or 128 (fp32)
// bytes leave in one piece.  Each pixel's destination travels through the scratch as well
// (null for pixels past the end), so the storing lane needs no index arithmetic.
template <typename T> constexpr uint32_t unit_row_stride() { return kBrickRows * sizeof(T) + 16; }
template <typename T> constexpr uint32_t unit_scratch_bytes() { return kBrickRows * unit_row_stride<T>() + kBrickRows * 8; }

template <typename T>
__device__ __forceinline__ void store_unit_nhwc(const f32x4 (&y)[4], T* my_pixel_out, uint32_t n_valid, uint8_t* scratch)
{
    constexpr uint32_t EPC = 16 / sizeof(T), RS = unit_row_stride<T>();
    constexpr uint32_t CP = kBrickRows / EPC;                       // 16-byte chunks per pixel row: 4 (bf16) or 8 (fp32)
    const uint32_t lane = threadIdx.x & 63, li = lane & 31, lh = lane >> 5;
    T** dests = (T**)(scratch + kBrickRows * RS);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        T o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (T)y[g][e];
        uint8_t* p = scratch + li * RS + (8 * g + 4 * lh) * sizeof(T);
        if constexpr (sizeof(T) == 2) *(uint64_t*)p = __builtin_bit_cast(uint64_t, o);
        else *(u32x4*)p = __builtin_bit_cast(u32x4, o);
    }
    if (lh == 0) dests[li] = my_pixel_out;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");             // the wave's own LDS writes have landed
#pragma unroll
    for (uint32_t pass = 0; pass < CP / 2; ++pass) {
        const uint32_t px = pass * (64 / CP) + lane / CP, ch = lane % CP;
        T* dst = dests[px];
        const u32x4 v = *(const u32x4*)(scratch + px * RS + ch * 16);
        if (dst != nullptr && ch * EPC < n_valid) *(u32x4*)(dst + ch * EPC) = v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");             // reads done before the next unit overwrites the scratch
}

// ---- grouped k x k convolution as implicit GEMM ---------------------------------------------
// GEMM view: rows = (request, output pixel), columns = output channels, K = (kh, kw, c_in).
// A workgroup takes 128 consecutive rows of one tenant and up to 128 output channels; each of
// its four waves owns 32 rows and all the channels, and no operand is shared between waves:
// the activation operand of a k step is gathered straight from the NHWC input into MFMA
// registers (16 bytes per lane = 8 channels of one tap; taps outside the image read as
// zeros), the filter bricks come from L1/L2 (a layer's filters are at most ~150 KB and shared
// by every tile of the tenant).  The MFMA takes the filter brick as its row operand and the
// pixels as its column operand, so a lane ends up with runs of four consecutive channels of
// ITS pixel, whose address it already derived for its loads; the unit then leaves through the
// wave's store scratch (store_unit_nhwc).  No barrier anywhere.
template <typename T, int CB>
__device__ __forceinline__ void conv_wave(const GemmArgs& a, const LayerDev& L, uint32_t seg0, uint32_t m0, uint32_t rows_total, uint32_t nb0, uint8_t* scratch)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC, P = 4;
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;
    const uint32_t lane = threadIdx.x & 63, li = lane & 31, lh = lane >> 5;
    const uint32_t nKB = L.K / KB, nKBv = ceil_div(L.k_valid, KB);  // bricks per filter row; k steps that hold real taps
    const uint32_t rpr = L.rows_per_req;

    // this lane's GEMM row: request, output pixel, top-left input coordinate
    const uint32_t m = m0 + li;
    const bool row_ok = m < rows_total;
    const uint32_t mm = row_ok ? m : m0;                           // rows past the end repeat the first one and are dropped
    uint32_t req, pix, oh, ow;
    divmod_uniform(mm, rpr, &req, &pix);
    divmod_uniform(pix, L.out_w, &oh, &ow);
    const int32_t ih0 = (int32_t)(oh * L.stride) - (int32_t)L.pad, iw0 = (int32_t)(ow * L.stride) - (int32_t)L.pad;
    gptr_t img = (gptr_t)((const T*)act_of(a.act, L.in_buf) + (size_t)(seg0 + req) * a.S);
    gptr_t wp = (gptr_t)((const u32x4*)(a.arena + L.w_off) + (size_t)nb0 * nKB * 64 + lane);

    // The next k step's chunk.  Taps outside the image, steps past the last tap and rows past the
    // end read a block of zeros instead: the choice is made on the address, so nothing waits on
    // the loaded value before its MFMA.
    gptr_t zeros = (gptr_t)a.zeros;
    TapWalk<T> walk;
    walk.init(L, ih0, iw0, row_ok, lh * EPC, KB);
    auto load_a = [&]() -> u32x4 {
        const int32_t chunk = walk.next();
        gptr_t p = chunk >= 0 ? img + chunk : zeros;
        return *p;
    };

    f32x16 acc[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    // both operands of a k step travel P steps ahead of their use in register rings
    u32x4 aq[P], wq[P][CB];
    auto load_w = [&](uint32_t j, uint32_t kb) {
#pragma unroll
        for (int c = 0; c < CB; ++c) wq[j][c] = wp[((size_t)c * nKB + kb) * 64];
    };
#pragma unroll
    for (uint32_t j = 0; j < P; ++j) {
        aq[j] = load_a();
        load_w(j, min(j, nKBv - 1));
    }
    const uint32_t full = nKBv / P;
    for (uint32_t g = 0; g < full; ++g) {
#pragma unroll
        for (uint32_t j = 0; j < P; ++j) {
            const uint32_t kb = g * P + j;
#pragma unroll
            for (int c = 0; c < CB; ++c) Mma<T>::run(acc[c], wq[j][c], aq[j]);   // rows = channels, columns = pixels
            aq[j] = load_a();
            load_w(j, min(kb + P, nKBv - 1));
            __builtin_amdgcn_sched_barrier(0);                     // keeps the refills here, P steps ahead of their use
        }
    }
#pragma unroll
    for (uint32_t j = 0; j < P; ++j) {
        const uint32_t kb = full * P + j;
        if (kb < nKBv) {
#pragma unroll
            for (int c = 0; c < CB; ++c) Mma<T>::run(acc[c], wq[j][c], aq[j]);
        }
    }

    // epilogue: the lane holds, for pixel li, channels 8g + 4 lh + {0..3} (g = 0..3) of every
    // channel block: bias, activation, rounding, coalesced store through the wave's scratch
    const float* bias = (const float*)(a.arena + L.b_off);
    T* out = row_ok ? (T*)act_of(a.act, L.out_buf) + (size_t)(seg0 + req) * a.S + (size_t)pix * L.N : nullptr;
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        const uint32_t nbase = (nb0 + c) * kBrickRows;
        f32x4 y[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 bv = *(const f32x4*)(bias + nbase + 8 * g + 4 * lh);   // bias is padded to N_pad
#pragma unroll
            for (int i = 0; i < 4; ++i) y[g][i] = acc[c][4 * g + i] + bv[i];
        }
        activate_block<4>(y, L.act);
        // N is a multiple of 8, so the channels of this block that exist are whole 16-byte chunks for bf16 and pairs of them for fp32
        const uint32_t nvalid = min((uint32_t)kBrickRows, L.N - nbase);
        if (L.fuse_add)
            add_residual<T>(y, out ? (const T*)act_of(a.act, L.in2_buf) + (out - (T*)act_of(a.act, L.out_buf)) + nbase : nullptr, lh, nvalid, L.fuse_add - 1);
        store_unit_nhwc<T>(y, out ? out + nbase : nullptr, nvalid, scratch);
    }
}

// MAXCB bounds the channel blocks of any tile in the launch: narrow layers get a kernel with
// few registers and many resident waves, which is what hides the latency of their short K loops.
template <typename T, int MAXCB>
__global__ __launch_bounds__(256) void conv_kernel(GemmArgs a)
{
    __shared__ uint32_t owner_part[4];
    __shared__ __attribute__((aligned(16))) uint8_t unit_scratch[4 * unit_scratch_bytes<T>()];
    const uint32_t tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint8_t* scratch = unit_scratch + wave * unit_scratch_bytes<T>();
    TileOwner<256> lookup;
    lookup.fetch(a.tile_base, a.T);
    const uint32_t n_tiles = a.tile_base[a.T];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    const uint32_t t = lookup.owner(a.T, idx, owner_part);   // uniform: the tenant's facts come through scalar loads
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t seg0 = a.off[t];
    const uint32_t local = idx - a.tile_base[t];
    // (a row-tiled layer's list counts more tiles than its pixels fill: those beyond the last pixel have nothing to do)
    const uint32_t rows_total = a.M[t] * L.rows_per_req, mt_ = ceil_div(a.M[t] * conv_tile_rows(L.rows_per_req, L.row_tiles), kConvTileRows);
    const uint32_t nb0 = (local / mt_) * (kTileCols / kBrickRows);
    const uint32_t ncb = min((uint32_t)(kTileCols / kBrickRows), L.N_pad / kBrickRows - nb0);
    // no barrier below: the waves are independent; wave w takes row blocks w, w+4, ... of the tile
    for (uint32_t rb = wave; rb < kConvTileRows / kBrickRows; rb += 4) {
        const uint32_t m0 = (local % mt_) * kConvTileRows + rb * kBrickRows;
        if (m0 >= rows_total) break;
        if constexpr (MAXCB == 1) {
            conv_wave<T, 1>(a, L, seg0, m0, rows_total, nb0, scratch);
        } else if constexpr (MAXCB == 2) {
            if (ncb == 1) conv_wave<T, 1>(a, L, seg0, m0, rows_total, nb0, scratch);
            else conv_wave<T, 2>(a, L, seg0, m0, rows_total, nb0, scratch);
        } else {
            if (ncb == 1) conv_wave<T, 1>(a, L, seg0, m0, rows_total, nb0, scratch);
            else if (ncb == 2) conv_wave<T, 2>(a, L, seg0, m0, rows_total, nb0, scratch);
            else if (ncb == 3) conv_wave<T, 3>(a, L, seg0, m0, rows_total, nb0, scratch);
            else conv_wave<T, 4>(a, L, seg0, m0, rows_total, nb0, scratch);
        }
    }
}

// ---- convolution tiles of two or more channel blocks: activation operand shared through LDS --
// Same tile (128 pixels x <= 128 channels) and tile list as conv_kernel, other division of
// labour.  With every wave gathering its own 32 pixels, each wave also streams the whole
// filter bank; here the waves stand side by side instead (NCB = 4: one 32-channel block and
// all four pixel blocks per wave; NCB = 2: 2x2), so a wave streams the filters of one channel
// block only and the gathered activation bricks are shared.  Neither operand passes through
// registers: wave w forms the bricks of pixel block w, and fetches the filter bricks of its
// own channel block, with direct global->LDS loads, one per k step, each lane supplying the
// address of its 16 bytes (for the activations: 8 channels of one tap, or a block of zeros
// for taps outside the image) and the hardware placing lane l at base + 16 l.  The lanes of an
// activation gather stand in pairs on a pixel's 32 bytes of the k step (lane = 2 * pixel +
// half), so the texture path sees 32 accesses per instruction instead of 64, and the MFMA
// operand read (lane (li, lh) takes piece 2 li + lh) touches every bank once.  K is walked in chunks of kConvKC k steps through a ring of kConvNS stages, chunks
// kConvNS - 1 ahead of their use.
constexpr uint32_t kConvKC = 2, kConvNS = 3;
constexpr uint32_t kConvDeepKC = 4, kConvDeepNS = 4;   // chunks and ring of a workgroup that is alone on its CU (see PW below): 128 KiB

// QUAD (every tenant's input channels are a multiple of 4 chunks, i.e. a pixel's share of two k
// steps is 64 contiguous bytes): a gather instruction then takes 16 pixels with four consecutive
// lanes on one pixel's 64 bytes.  The texture path handles a lane quad on one cache line as one
// access, so the gather costs half the accesses of the pair layout; the data then sits in LDS as
// [pixel][chunk] and the MFMA operand read has a 2-way bank conflict.  That trade pays where a wave
// reads two pixel blocks per k step (NCB = 2: 55.2 against 57.3 us on the 32 -> 64 channel layer
// of the CNN mix) and not where it reads four (NCB = 4: 40.4 against 38.1 us on the 64 -> 128
// layer, where the counters showed the conflicts as half of the LDS pipe's busy time), so the
// launcher asks for it with two channel blocks only.
// PW = 1: eight waves; waves 4..7 issue the loads (wave 4 + w what wave w would have issued: the gather of pixel
// block w, the bricks of filter block w) and do nothing else, waves 0..3 read and multiply.  For launches of few
// tiles with a long K (deep layers of small batches): their workgroups sit alone on their CUs, one wave per SIMD,
// and a wave that issues its own loads stands at every one of them for ~100 clocks with no MFMA in the pipe.
// FAST: the gather's walk through the window is shared by the wave (UniformTapWalk): every tenant's cin is a
// multiple of the elements a lane group takes per step, and a tenant's activations are less than 2 GiB.
template <typename T, int NCB, bool QUAD, int PW, bool FAST>
__global__ __launch_bounds__(256 * (1 + PW)) __attribute__((amdgpu_waves_per_eu(PW ? 2 : NCB == 2 ? 4 : 3, NCB == 2 && !PW ? 4 : 3))) void conv_lds_kernel(GemmArgs a)     // PW = 0: as many workgroups per CU as the LDS ring allows: three (48 KiB), four with two filter blocks (36 KiB)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    constexpr uint32_t KC = PW ? kConvDeepKC : kConvKC, NS = PW ? kConvDeepNS : kConvNS;   // k steps per chunk; stages of the ring (chunks are fetched NS - 1 ahead)
    constexpr uint32_t kStageBytes = (4 + NCB) * KC * kBrickBytes;     // 4 pixel blocks + the tile's NCB filter blocks, KC k steps each
    static_assert(!QUAD || KC == 2, "a quad gather covers exactly two k steps");
    constexpr uint32_t WR = 4 / NCB, RBW = 4 / WR;                  // wave rows; pixel blocks per wave
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;
    __shared__ __attribute__((aligned(16))) uint8_t lds[NS * kStageBytes];
    __shared__ uint32_t owner_part[4 * (1 + PW)];
    const uint32_t tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const uint32_t wave_all = __builtin_amdgcn_readfirstlane(tid >> 6), wave = wave_all % 4;
    const bool loader = !PW || wave_all >= 4, worker = !PW || wave_all < 4;     // who issues the loads, who multiplies
    TileOwner<256 * (1 + PW)> lookup;
    lookup.fetch(a.tile_base, a.T);
    const uint32_t n_tiles = a.tile_base[a.T];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    const uint32_t t = lookup.owner(a.T, idx, owner_part);   // uniform: the tenant's facts come through scalar loads
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t seg0 = a.off[t];
    const uint32_t local = idx - a.tile_base[t];
    const uint32_t rpr = L.rows_per_req;
    const uint32_t rows_total = a.M[t] * rpr, mt_ = ceil_div(a.M[t] * conv_tile_rows(rpr, L.row_tiles), kConvTileRows);
    const uint32_t m0 = (local % mt_) * kConvTileRows;
    if (m0 >= rows_total) return;                             // a row-tiled layer's list counts more tiles than its pixels fill
    const uint32_t nb0 = (local / mt_) * (kTileCols / kBrickRows);
    const uint32_t ncb = min((uint32_t)(kTileCols / kBrickRows), L.N_pad / kBrickRows - nb0);
    const uint32_t nKB = L.K / KB, nKBv = ceil_div(L.k_valid, KB);
    const uint32_t n_chunks = ceil_div(nKBv, KC);             // n_chunks * KC <= nKB: K is padded to 64
    const uint32_t wc = wave % NCB, wr = wave / NCB;
    const bool active = wc < ncb;                                  // idle waves still gather; they stream block 0 and drop it

    // gather role: pixel block `wave`.  Pairs: pixel lane/2, half lane%2 of its 32 bytes of a k step.
    // QUAD: pixels lane/4 and lane/4 + 16, chunk lane%4 of the 64 bytes that two k steps take of each.
    constexpr uint32_t NPX = QUAD ? 2 : 1;
    gptr_t zeros = (gptr_t)a.zeros;
    gptr_t img[NPX];
    TapWalk<T> walk[NPX];
    // FAST: the tenant's activations as one buffer; per lane the byte offset of its first element at the window's
    // top-left tap (negative where that tap lies in front of the buffer: such taps are never asked for) and its taps
    UniformTapWalk uwalk[NPX];
    u32x4 in_desc{};
    int32_t lane_off[NPX];
    uint32_t taps_lo[NPX], taps_hi[NPX];
    if constexpr (FAST) in_desc = buffer_descriptor((const T*)act_of(a.act, L.in_buf) + (size_t)seg0 * a.S, a.M[t] * a.S * (uint32_t)sizeof(T));
#pragma unroll
    for (uint32_t i = 0; i < NPX; ++i) {
        const uint32_t gm = m0 + wave * kBrickRows + (QUAD ? (lane >> 2) + 16 * i : (lane >> 1));
        const bool row_ok = gm < rows_total;
        const uint32_t mm = row_ok ? gm : m0;
        uint32_t req, pix, oh, ow;
        divmod_uniform(mm, rpr, &req, &pix);
        divmod_uniform(pix, L.out_w, &oh, &ow);
        const int32_t ih0 = (int32_t)(oh * L.stride) - (int32_t)L.pad, iw0 = (int32_t)(ow * L.stride) - (int32_t)L.pad;
        const uint32_t first = QUAD ? (lane & 3) * EPC : (lane & 1) * EPC;
        if constexpr (FAST) {
            uwalk[i].init(L, QUAD ? 2 * KB : KB);
            lane_off[i] = (int32_t)(req * a.S * (uint32_t)sizeof(T)) + ((ih0 * (int32_t)L.in_w + iw0) * (int32_t)L.cin + (int32_t)first) * (int32_t)sizeof(T);
            const uint64_t m = taps_inside(L, ih0, iw0, row_ok);
            taps_lo[i] = (uint32_t)m; taps_hi[i] = (uint32_t)(m >> 32);
        } else {
            img[i] = (gptr_t)((const T*)act_of(a.act, L.in_buf) + (size_t)(seg0 + req) * a.S);
            walk[i].init(L, ih0, iw0, row_ok, first, QUAD ? 2 * KB : KB);
        }
    }
    gptr_t wp = (gptr_t)((const u32x4*)(a.arena + L.w_off) + (size_t)(nb0 + (active ? wc : 0)) * nKB * 64 + lane);
    const uint32_t last_kb = n_chunks * KC - 1;
    // one k step of a chunk: the gather of this wave's pixel block, the brick of its filter block
    // (pairs: k step kk of all 32 pixels; QUAD: both k steps of pixels 16 kk .. 16 kk + 15)
    auto fetch_gather = [&](uint32_t c, uint32_t kk) {
        uint8_t* dst = lds + (c % NS) * kStageBytes + (wave * KC + kk) * kBrickBytes;
        if constexpr (FAST) {
            UniformTapWalk& u = uwalk[QUAD ? kk : 0];
            const uint32_t tp = u.tp, word = tp < 32 ? taps_lo[QUAD ? kk : 0] : taps_hi[QUAD ? kk : 0];
            const bool inside = (int32_t)(word << (31 - (tp & 31))) < 0;
            const uint32_t voff = inside ? (uint32_t)(lane_off[QUAD ? kk : 0] + (int32_t)(u.off * (uint32_t)sizeof(T))) : 0x80000000u;
            u.advance();
            lds_dma16_buffer(in_desc, voff, dst);
        } else {
            const int32_t chunk = walk[QUAD ? kk : 0].next();
            gptr_t p = chunk >= 0 ? img[QUAD ? kk : 0] + chunk : zeros;
            lds_dma16(p, dst);
        }
    };
    auto fetch_filter = [&](uint32_t c, uint32_t kk) {
        if (wr == 0) lds_dma16(wp + (size_t)min(c * KC + kk, last_kb) * 64, lds + (c % NS) * kStageBytes + ((4 + wc) * KC + kk) * kBrickBytes);   // a filter block is fetched once, by the first wave row
    };
    auto fetch_chunk = [&](uint32_t c) {
#pragma unroll
        for (uint32_t kk = 0; kk < KC; ++kk) { fetch_gather(c, kk); fetch_filter(c, kk); }
    };
    // where lane (li, lh) finds its 16 bytes of k step kk inside a pixel block's area of a stage
    const uint32_t a_lane = QUAD ? (li * 4 + lh) * 16 : (li * 2 + lh) * 16;
    constexpr uint32_t a_kk = QUAD ? 32 : kBrickBytes;
    auto read_w = [&](const uint8_t* st, uint32_t kk, u32x4& wv) { wv = *(const u32x4*)(st + ((4 + wc) * KC + kk) * kBrickBytes + lane * 16); };
    auto read_a = [&](const uint8_t* st, uint32_t kk, u32x4 (&av)[RBW], uint32_t r0, uint32_t r1) {
#pragma unroll
        for (uint32_t r = r0; r < r1; ++r) av[r] = *(const u32x4*)(st + (wr * RBW + r) * KC * kBrickBytes + kk * a_kk + a_lane);
    };

    f32x16 acc[RBW];
#pragma unroll
    for (uint32_t r = 0; r < RBW; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[r][v] = 0.0f;
    auto mma = [&](const u32x4& wv, const u32x4 (&av)[RBW], uint32_t r0, uint32_t r1) {
#pragma unroll
        for (uint32_t r = r0; r < r1; ++r) Mma<T>::run(acc[r], wv, av[r]);       // rows = channels, columns = pixels
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    static_assert((PW || KC == 2) && KC % 2 == 0 && (RBW == 2 || RBW == 4), "the schedules below: chunks of two k steps, or an even number with loader waves");

    // when chunk c is needed, the loads of the NS - 2 younger chunks may still be in flight
    // (waves of the first wave row issue two loads per k step, gather and filter brick, the others one)
    constexpr uint32_t kOut = (NS - 2) * 2 * KC, kOutG = (NS - 2) * KC;
    constexpr int kWaitVm = (int)((kOut & 15) | ((kOut >> 4) << 14) | 0x0070 | 0x0F00), kWaitVmG = (int)((kOutG & 15) | ((kOutG >> 4) << 14) | 0x0070 | 0x0F00);
    auto chunk_barrier = [&] {                                     // chunk c is complete for every wave; every wave holds what it needs of chunk c - 1 in registers
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");         // this wave's LDS reads are done before the slot is handed back
        if (wr == 0) __builtin_amdgcn_s_waitcnt(kWaitVm); else __builtin_amdgcn_s_waitcnt(kWaitVmG);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // The two k steps of a chunk use two operand register sets, X and Y, and the second k step of a
    // chunk is multiplied after the next chunk's barrier, so the MFMA pipe has work the moment the
    // barrier opens; the chunk's four global->LDS loads (with the walk through the window that finds
    // the gather's addresses) and its LDS reads are dealt out between the MFMAs, in the shadow of one
    // already in the pipe.  Issued as one burst behind the barrier, the workgroup's sixteen loads take
    // the L1 -> LDS path ~270 clocks to accept, during which every wave stood at its load instructions
    // with no MFMA in flight: a workgroup alone on its CU spent as long on that as on its MFMAs.
    if (loader) {
#pragma unroll
        for (uint32_t c = 0; c < NS - 1; ++c) fetch_chunk(c);
    }
    chunk_barrier();
    if (loader) fetch_chunk(NS - 1);
    auto load_gather = [&](uint32_t c, uint32_t kk) { if constexpr (!PW) fetch_gather(c, kk); };
    auto load_filter = [&](uint32_t c, uint32_t kk) { if constexpr (!PW) fetch_filter(c, kk); };
    if (worker && PW) {
        // loads are someone else's business: a plain pipeline, the operands of a k step are read while the step
        // before it multiplies, and the barrier of the next chunk stands in front of the read of its first step
        u32x4 w[2], av[2][RBW];
        read_w(lds, 0, w[0]); read_a(lds, 0, av[0], 0, RBW);
        for (uint32_t c = 0; c < n_chunks; ++c) {
            const uint8_t* st = lds + (c % NS) * kStageBytes;
#pragma unroll
            for (uint32_t kk = 0; kk < KC; ++kk) {
                if (kk + 1 < KC) {
                    read_w(st, kk + 1, w[(kk + 1) % 2]); read_a(st, kk + 1, av[(kk + 1) % 2], 0, RBW);
                } else if (c + 1 < n_chunks) {
                    chunk_barrier();
                    const uint8_t* nst = lds + ((c + 1) % NS) * kStageBytes;
                    read_w(nst, 0, w[0]); read_a(nst, 0, av[0], 0, RBW);
                }
                fence();
                mma(w[kk % 2], av[kk % 2], 0, RBW);
                fence();
            }
        }
    } else if (worker) {
        u32x4 xw, yw, xa[RBW], ya[RBW];
        read_w(lds, 0, xw); read_a(lds, 0, xa, 0, RBW);
        read_w(lds, 1, yw); read_a(lds, 1, ya, 0, RBW);
        fence();
        mma(xw, xa, 0, RBW);
        for (uint32_t c = 1; c < n_chunks; ++c) {
            chunk_barrier();
            const uint8_t* st = lds + (c % NS) * kStageBytes;
            const uint32_t nx = c + NS - 1;                       // its slot held chunk c - 1
            fence();
            if constexpr (RBW == 4) {
                mma(yw, ya, 0, 1); fence();
                load_gather(nx, 0); fence();
                mma(yw, ya, 1, 2); fence();
                read_w(st, 0, xw); read_a(st, 0, xa, 0, 1); fence();
                mma(yw, ya, 2, 3); fence();
                load_filter(nx, 0); read_a(st, 0, xa, 1, 4); fence();
                mma(yw, ya, 3, 4); fence();
                load_gather(nx, 1); fence();
                mma(xw, xa, 0, 1); fence();
                read_w(st, 1, yw); read_a(st, 1, ya, 0, 1); load_filter(nx, 1); fence();
                mma(xw, xa, 1, 2); fence();
                read_a(st, 1, ya, 1, 4); fence();
                mma(xw, xa, 2, 4); fence();
            } else {
                mma(yw, ya, 0, 1); fence();
                load_gather(nx, 0); read_w(st, 0, xw); read_a(st, 0, xa, 0, 1); fence();
                mma(yw, ya, 1, 2); fence();
                load_filter(nx, 0); read_a(st, 0, xa, 1, 2); fence();
                mma(xw, xa, 0, 1); fence();
                load_gather(nx, 1); read_w(st, 1, yw); read_a(st, 1, ya, 0, 1); fence();
                mma(xw, xa, 1, 2); fence();
                load_filter(nx, 1); read_a(st, 1, ya, 1, 2); fence();
            }
        }
        mma(yw, ya, 0, RBW);
    } else {
        for (uint32_t c = 1; c < n_chunks; ++c) {                     // the loaders' loop: as many barriers as the workers'
            chunk_barrier();
            fetch_chunk(c + NS - 1);
        }
    }
    // trailing loads have landed and every wave is done with the ring: its memory now serves as
    // the waves' store scratch
    // (this wave's bias values, the same for all its pixel blocks, are fetched in front of that
    // wait: fetched block by block they put a memory round trip per block on the tile's tail)
    const float* bias = (const float*)(a.arena + L.b_off);
    const uint32_t nbase = (nb0 + (active ? wc : 0)) * kBrickRows;
    f32x4 bias_q[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) bias_q[g] = *(const f32x4*)(bias + nbase + 8 * g + 4 * lh);   // bias is padded to N_pad
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    static_assert(NS * kStageBytes >= 4 * unit_scratch_bytes<T>(), "store scratch aliases the ring");
    if (!worker) return;

    // epilogue: lane holds, for pixel li of each of its pixel blocks, channels 8g + 4 lh + {0..3}
    if (!active) return;
    uint8_t* scratch = lds + wave * unit_scratch_bytes<T>();
    if (a.pool && L.pool_fill) {
        // The next layer averages every channel over the image, and the one or two pixel blocks of an
        // image all belong to this wave: average here, from the activations as they would have been
        // stored (rounded to T), and write the pooled row in the brick layout the FC layers read.  The
        // image itself is never written.  Lane (li, lh) puts its values into the scratch as
        // [pixel][channel]; lane (c, half) then adds channel c over pixels 16 half .. 16 half + 15.
        constexpr uint32_t RS = unit_row_stride<T>();
        const uint32_t bpi = rpr / kBrickRows, ch = lane & 31, half = lane >> 5;
        const uint32_t nKBp = L.pool_fill / KB;
        const float inv = 1.0f / (float)rpr;
        float sum = 0.0f;
#pragma unroll
        for (uint32_t r = 0; r < RBW; ++r) {
            const uint32_t blk = wr * RBW + r, mb = m0 + blk * kBrickRows;    // images are whole: a block is valid or not
            f32x4 y[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int i = 0; i < 4; ++i) y[g][i] = acc[r][4 * g + i] + bias_q[g][i];
            }
            __builtin_amdgcn_sched_barrier(0);
            activate_block<4>(y, L.act);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                T o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (T)y[g][e];
                uint8_t* p = scratch + li * RS + (8 * g + 4 * lh) * sizeof(T);
                if constexpr (sizeof(T) == 2) *(uint64_t*)p = __builtin_bit_cast(uint64_t, o);
                else *(u32x4*)p = __builtin_bit_cast(u32x4, o);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (mb < rows_total) {
#pragma unroll
                for (uint32_t p = 0; p < 16; ++p) sum += (float)*(const T*)(scratch + (half * 16 + p) * RS + ch * sizeof(T));
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if ((blk + 1) % bpi == 0) {                                      // the image is complete
                sum += __shfl_xor(sum, 32);
                if (half == 0 && mb < rows_total) {
                    const uint32_t req = mb / rpr, cc = nbase + ch;
                    T* out = (T*)act_of(a.act, L.pool_buf) + (size_t)seg0 * a.S + (size_t)(req / kBrickRows) * nKBp * 64 * EPC;
                    out[((size_t)(cc / KB) * 64 + req % kBrickRows + 32 * ((cc % KB) / EPC)) * EPC + cc % EPC] = (T)(sum * inv);
                }
                sum = 0.0f;
            }
        }
        return;
    }
#pragma unroll
    for (uint32_t r = 0; r < RBW; ++r) {
        const uint32_t m = m0 + (wr * RBW + r) * kBrickRows + li;
        T* out = nullptr;
        if (m < rows_total) {
            uint32_t req, pix;
            divmod_uniform(m, rpr, &req, &pix);
            out = (T*)act_of(a.act, L.out_buf) + (size_t)(seg0 + req) * a.S + (size_t)pix * L.N + nbase;
        }
        f32x4 y[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int i = 0; i < 4; ++i) y[g][i] = acc[r][4 * g + i] + bias_q[g][i];
        }
        __builtin_amdgcn_sched_barrier(0);
        activate_block<4>(y, L.act);
        const uint32_t nvalid = min((uint32_t)kBrickRows, L.N - nbase);
        if (L.fuse_add)
            add_residual<T>(y, out ? (const T*)act_of(a.act, L.in2_buf) + (out - (T*)act_of(a.act, L.out_buf)) : nullptr, lh, nvalid, L.fuse_add - 1);
        store_unit_nhwc<T>(y, out, nvalid, scratch);
    }
}

// ---- convolution tiles whose input fits LDS ----------------------------------------------------
// Tiles of whole output rows of one image, or of whole small images (RowTiling: up to 128 pixel slots, some of
// them empty where the rows do not fill them; x <= 128 channels), for 3x3 layers: the input rows a tile needs are copied
// to LDS once, with contiguous 16-byte loads, into a frame with a zero border (one pixel left
// and right, one row above and below where the image ends), and the nine taps of every pixel are
// read from there.  Against gathering every tap from L2 this moves each input byte once instead
// of 2.25 (stride 2) to 9 (stride 1) times through the texture path, and the walk through K
// becomes scalar arithmetic: a k step lies inside one tap (cin is a multiple of a k step), so its
// LDS offset (kernel row, kernel column, channel chunk) is the same for every lane; lanes differ
// by the fixed address of their pixel's top-left tap.  Pixels are kept 16 bytes apart from a
// multiple of 32 bytes, which spreads the lanes of a stride-2 read over half the banks (2-way
// conflict; stride 1: none).  Filters stream through a register ring per wave as in conv_kernel.
// Sub-images: a tile holds `ni` of them, each `n_oh` output rows of one image.
template <typename T, int NCB, bool TWO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NCB == 1 ? 8 : NCB == 2 ? 4 : 3, NCB == 1 ? 8 : NCB == 2 ? 4 : 3))) void conv_img_kernel(GemmArgs a)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    constexpr uint32_t NB = NCB == 1 ? 2 : NCB == 2 ? 5 : 9;        // frame loads in flight per lane
    constexpr uint32_t P = NCB == 1 ? 4 : 8;                        // filter bricks in flight per wave (one channel block: small tiles, many resident waves)
    static_assert(NCB == 1 || NCB == 2 || NCB == 4, "channel blocks side by side");
    constexpr uint32_t WR = 4 / NCB, RBW = 4 / WR;                  // wave rows; pixel blocks per wave
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;
    extern __shared__ __attribute__((aligned(16))) uint8_t img[];
    __shared__ uint32_t owner_part[4];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), li = lane & 31, lh = lane >> 5;
    TileOwner<256> lookup;
    lookup.fetch(a.tile_base, a.T);
    const uint32_t n_tiles = a.tile_base[a.T];
    // the frame starts as zeros (its border, rows past the image, sub-images past the tenant's last request);
    // written while the tile list is on its way, published by the barrier of the lookup
    for (uint32_t q = tid * 16; q < a.img_lds; q += 256 * 16) *(u32x4*)(img + q) = u32x4{0, 0, 0, 0};
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    const uint32_t t = lookup.owner(a.T, idx, owner_part);   // uniform: the tenant's facts come through scalar loads
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t seg0 = a.off[t], Mt = a.M[t];
    const uint32_t local = idx - a.tile_base[t];
    const uint32_t rpr = L.rows_per_req;
    const RowTiling rt = unpack_row_tiling(L.row_tiles);     // every tenant of such a launch has one
    const uint32_t mt_ = ceil_div(Mt * conv_tile_rows(rpr, L.row_tiles), kConvTileRows);
    const uint32_t tm = local % mt_;
    const uint32_t nb0 = (local / mt_) * (kTileCols / kBrickRows);
    const uint32_t ncb = min((uint32_t)(kTileCols / kBrickRows), L.N_pad / kBrickRows - nb0);
    const uint32_t nKB = L.K / KB, nKBv = ceil_div(L.k_valid, KB);  // cin is a multiple of KB (whole k steps), or half of one
    const uint32_t wc = wave % NCB, wr = wave / NCB;
    const bool active = wc < ncb;

    // geometry of the frame (all wave-uniform)
    const uint32_t st = L.stride, ow_n = L.out_w, iw_n = L.in_w, ih_n = L.in_h, cin = L.cin;
    // TWO: cin == EPC for every tenant (a padded three-channel input in bf16): a pixel is one 16-byte chunk, a k
    // step spans two taps, and the two halves of the wave take one tap each
    constexpr bool two = TWO;
    const uint32_t PB = cin * (uint32_t)sizeof(T) + (two ? 0 : 16), RSB = (iw_n + 2) * PB;   // bytes per pixel slot, per frame row
    const uint32_t ni = rt.ni, spi = kConvTileRows / ni;                          // sub-images of the tile; pixel slots of one
    const uint32_t n_oh = rt.n_oh, n_ih = (n_oh - 1) * st + 3;                    // its output rows, its frame rows
    const uint32_t SUB = n_ih * RSB;
    uint32_t req0 = tm * ni, oh_first = 0;                                        // the first sub-image's request; first output row of the sub-images
    if (ni == 1) { divmod_uniform(tm, rt.tpi, &req0, &oh_first); oh_first *= n_oh; }
    const uint32_t px_t = min(n_oh * ow_n, rpr - oh_first * ow_n);                // pixels of a sub-image in this tile (an image's last tile may be short)

    // the first filter bricks travel while the frame is filled (idle waves stream block 0 and drop it)
    gptr_t wp = (gptr_t)((const u32x4*)(a.arena + L.w_off) + (size_t)(nb0 + (active ? wc : 0)) * nKB * 64 + lane);
    u32x4 wq[P];
#pragma unroll
    for (uint32_t j = 0; j < P; ++j) wq[j] = wp[(size_t)min(j, nKBv - 1) * 64];

    const uint32_t cpp = cin * (uint32_t)sizeof(T) / 16, cpr = iw_n * cpp;       // 16-byte chunks per pixel, per image row
    for (uint32_t i = 0; i < ni; ++i) {
        const uint32_t req = req0 + i;
        if (req >= Mt) break;
        const int32_t ih_first = (int32_t)(oh_first * st) - 1;                   // image row of frame row 0
        const int32_t r_lo = ih_first < 0 ? -ih_first : 0;
        const int32_t r_hi = min((int32_t)n_ih, (int32_t)ih_n - ih_first);       // frame rows [r_lo, r_hi) lie inside the image
        gptr_t src = (gptr_t)((const T*)act_of(a.act, L.in_buf) + (size_t)(seg0 + req) * a.S) + (size_t)(ih_first + r_lo) * cpr;
        const uint32_t n_chunks = (uint32_t)(r_hi - r_lo) * cpr;                 // contiguous in memory
        uint8_t* dst = img + i * SUB + (uint32_t)r_lo * RSB + PB;                // first pixel slot after the left border
        for (uint32_t q0 = 0; q0 < n_chunks; q0 += NB * 256) {                   // NB loads in flight per lane
            u32x4 v[NB];
#pragma unroll
            for (uint32_t j = 0; j < NB; ++j) {
                const uint32_t q = q0 + j * 256 + tid;
                v[j] = src[q < n_chunks ? q : 0];
            }
#pragma unroll
            for (uint32_t j = 0; j < NB; ++j) {
                const uint32_t q = q0 + j * 256 + tid;
                uint32_t r, x, col, c16;
                divmod_uniform(q, cpr, &r, &x);
                divmod_uniform(x, cpp, &col, &c16);
                if (q < n_chunks) *(u32x4*)(dst + r * RSB + col * PB + c16 * 16) = v[j];
            }
        }
    }
    __syncthreads();

    f32x16 acc[RBW];
#pragma unroll
    for (uint32_t r = 0; r < RBW; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[r][v] = 0.0f;
    if (active) {
        // this lane's pixel in each of the wave's pixel blocks: frame address of its top-left tap
        uint32_t base[RBW];
#pragma unroll
        for (uint32_t r = 0; r < RBW; ++r) {
            const uint32_t p = (wr * RBW + r) * kBrickRows + li;
            uint32_t i, pl, ohl, ow;
            divmod_uniform(p, spi, &i, &pl);
            if (pl >= px_t) { i = 0; pl = 0; }                                   // an empty slot multiplies the first pixel; nothing is stored for it
            divmod_uniform(pl, ow_n, &ohl, &ow);
            base[r] = i * SUB + ohl * st * RSB + ow * st * PB + (two ? 0 : lh * 16);
        }
        // position in K (all scalar): channel inside the tap, kernel column, byte offset of the tap's row, of the k step
        uint32_t ch = 0, kw = 0, row_off = 0, off = 0;
        auto advance = [&]() {
            ch += KB; off += KB * (uint32_t)sizeof(T);
            if (ch == cin) {                                       // next tap
                ch = 0; ++kw;
                if (kw == 3) { kw = 0; row_off += RSB; }
                off = row_off + kw * PB;
            }
        };
        // the pixel operands of a k step are read one step ahead of its MFMAs (past the last tap: the frame's last row, unused)
        uint32_t kbi = 0;                                          // two taps per k step: the k step whose operands are in av
        auto two_taps = [&](uint32_t k) -> uint32_t {              // this lane's tap of k step k (taps past the ninth meet zero filters)
            const uint32_t tp = min(2 * k + lh, 8u);
            return (tp / 3) * RSB + (tp % 3) * PB;
        };
        // The K loop over the first NR of the wave's pixel blocks: a tile whose pixels fill only half of them (one 7x7
        // image: 49 of 128 slots) spends half the MFMAs and LDS reads.
        auto k_loop = [&](auto NR_) {
            constexpr uint32_t NR = decltype(NR_)::value;
            u32x4 av[NR];
#pragma unroll
            for (uint32_t r = 0; r < NR; ++r) av[r] = *(const u32x4*)(img + base[r] + (two ? two_taps(0) : 0));
            auto step = [&](const u32x4& wv) {
                uint32_t off_n;
                if (two) { kbi = min(kbi + 1, nKBv - 1); off_n = two_taps(kbi); }
                else { advance(); off_n = min(off, 2 * RSB + 2 * PB + (cin - KB) * (uint32_t)sizeof(T)); }
                u32x4 an[NR];
#pragma unroll
                for (uint32_t r = 0; r < NR; ++r) an[r] = *(const u32x4*)(img + base[r] + off_n);
#pragma unroll
                for (uint32_t r = 0; r < NR; ++r) Mma<T>::run(acc[r], wv, av[r]);   // rows = channels, columns = pixels
#pragma unroll
                for (uint32_t r = 0; r < NR; ++r) av[r] = an[r];
            };
            const uint32_t full = nKBv / P;
            for (uint32_t g = 0; g < full; ++g) {
#pragma unroll
                for (uint32_t j = 0; j < P; ++j) {
                    step(wq[j]);
                    wq[j] = wp[(size_t)min(g * P + j + P, nKBv - 1) * 64];
                }
            }
#pragma unroll
            for (uint32_t j = 0; j < P; ++j)
                if (full * P + j < nKBv) step(wq[j]);
        };
        const uint32_t blocks_used = ceil_div((ni - 1) * spi + px_t, kBrickRows);     // pixel blocks of the tile with a pixel in them
        if (RBW > 1 && blocks_used <= wr * RBW + RBW / 2) k_loop(std::integral_constant<uint32_t, (RBW > 1 ? RBW / 2 : 1)>{});
        else k_loop(std::integral_constant<uint32_t, RBW>{});
    }
    const float* bias = (const float*)(a.arena + L.b_off);
    const uint32_t nbase = (nb0 + (active ? wc : 0)) * kBrickRows;
    f32x4 bias_q[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) bias_q[g] = *(const f32x4*)(bias + nbase + 8 * g + 4 * lh);   // bias is padded to N_pad
    __syncthreads();                                               // every wave is done with the frame: it now serves as store scratch
    if (!active) return;
    uint8_t* scratch = img + wave * unit_scratch_bytes<T>();
#pragma unroll
    for (uint32_t r = 0; r < RBW; ++r) {
        uint32_t i, pl;
        divmod_uniform((wr * RBW + r) * kBrickRows + li, spi, &i, &pl);
        T* out = nullptr;
        if (pl < px_t && req0 + i < Mt)
            out = (T*)act_of(a.act, L.out_buf) + (size_t)(seg0 + req0 + i) * a.S + (size_t)(oh_first * ow_n + pl) * L.N + nbase;
        f32x4 y[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int i = 0; i < 4; ++i) y[g][i] = acc[r][4 * g + i] + bias_q[g][i];
        }
        __builtin_amdgcn_sched_barrier(0);
        activate_block<4>(y, L.act);
        const uint32_t nvalid = min((uint32_t)kBrickRows, L.N - nbase);
        if (L.fuse_add)
            add_residual<T>(y, out ? (const T*)act_of(a.act, L.in2_buf) + (out - (T*)act_of(a.act, L.out_buf)) : nullptr, lh, nvalid, L.fuse_add - 1);
        store_unit_nhwc<T>(y, out, nvalid, scratch);
    }
}

// ---- launcher ------------------------------------------------------------
template <typename T, bool FAST>
static void launch_conv_lds_t(const GemmArgs& a, uint32_t max_cb, bool quad, bool loaders, uint32_t grid, hipStream_t s)
{
    if (max_cb == 2 && quad) hipLaunchKernelGGL((conv_lds_kernel<T, 2, true, 0, FAST>), dim3(grid), dim3(256), 0, s, a);
    else if (max_cb == 2) hipLaunchKernelGGL((conv_lds_kernel<T, 2, false, 0, FAST>), dim3(grid), dim3(256), 0, s, a);
    else if (loaders) hipLaunchKernelGGL((conv_lds_kernel<T, 4, false, 1, FAST>), dim3(grid), dim3(512), 0, s, a);
    else hipLaunchKernelGGL((conv_lds_kernel<T, 4, false, 0, FAST>), dim3(grid), dim3(256), 0, s, a);
}

template <typename T>
static void launch_conv_t(const GemmArgs& a, uint32_t max_cb, bool quad, bool loaders, bool fast, uint32_t grid, hipStream_t s)
{
    if (max_cb <= 1) hipLaunchKernelGGL((conv_kernel<T, 1>), dim3(grid), dim3(256), 0, s, a);
    else if (fast) launch_conv_lds_t<T, true>(a, max_cb, quad, loaders, grid, s);
    else launch_conv_lds_t<T, false>(a, max_cb, quad, loaders, grid, s);
}

// A launch may ask for more dynamic LDS than the 64 KiB a kernel gets without saying so; said once per kernel.
template <typename K>
static hipError_t allow_frame(K kernel)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kConvFrameMaxBytes);
}

template <typename T>
static hipError_t launch_conv_img_t(const GemmArgs& a, uint32_t max_cb, bool two, uint32_t lds_bytes, uint32_t grid, hipStream_t s)
{
    lds_bytes = std::max<uint32_t>(lds_bytes, 4 * unit_scratch_bytes<T>());       // the frame also serves as store scratch
    GemmArgs b = a;
    b.img_lds = lds_bytes;
    if (two && sizeof(T) == 2) {
        if (max_cb <= 1) hipLaunchKernelGGL((conv_img_kernel<T, 1, sizeof(T) == 2>), dim3(grid), dim3(256), lds_bytes, s, b);
        else if (max_cb <= 2) hipLaunchKernelGGL((conv_img_kernel<T, 2, sizeof(T) == 2>), dim3(grid), dim3(256), lds_bytes, s, b);
        else hipLaunchKernelGGL((conv_img_kernel<T, 4, sizeof(T) == 2>), dim3(grid), dim3(256), lds_bytes, s, b);
    } else {
        if (max_cb <= 1) hipLaunchKernelGGL((conv_img_kernel<T, 1, false>), dim3(grid), dim3(256), lds_bytes, s, b);
        else if (max_cb <= 2) hipLaunchKernelGGL((conv_img_kernel<T, 2, false>), dim3(grid), dim3(256), lds_bytes, s, b);
        else hipLaunchKernelGGL((conv_img_kernel<T, 4, false>), dim3(grid), dim3(256), lds_bytes, s, b);
    }
    return hipGetLastError();
}

template <typename T>
static hipError_t prepare_conv_t()
{
    hipError_t e = hipSuccess;
    auto also = [&](hipError_t x) { if (e == hipSuccess) e = x; };
    also(allow_frame(conv_img_kernel<T, 1, false>)); also(allow_frame(conv_img_kernel<T, 2, false>)); also(allow_frame(conv_img_kernel<T, 4, false>));
    also(allow_frame(conv_img_kernel<T, 1, sizeof(T) == 2>)); also(allow_frame(conv_img_kernel<T, 2, sizeof(T) == 2>)); also(allow_frame(conv_img_kernel<T, 4, sizeof(T) == 2>));
    return e;
}
hipError_t prepare_conv(uint32_t dtype) { return dtype == MT_BF16 ? prepare_conv_t<__bf16>() : prepare_conv_t<float>(); }

// img_lds_bytes > 0: every convolution of the layer index qualifies for the LDS-resident-input kernel, whose largest frame is that
// size; img_two: their pixels are one 16-byte chunk (else none is)
hipError_t launch_conv(const GemmArgs& a, uint32_t dtype, uint32_t max_cb, bool quad, uint32_t img_lds_bytes, bool img_two, bool long_k, bool uniform_walk, uint32_t grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 7) / 8 * 8;
    const bool loaders = long_k && grid <= 256;                      // at most one tile per CU, every tenant's K long: waves of their own for the loads
    if (img_lds_bytes) {
        return dtype == MT_BF16 ? launch_conv_img_t<__bf16>(a, max_cb, img_two, img_lds_bytes, grid, s)
                                : launch_conv_img_t<float>(a, max_cb, img_two, img_lds_bytes, grid, s);
    }
    if (dtype == MT_BF16) launch_conv_t<__bf16>(a, max_cb, quad, loaders, uniform_walk, grid, s);
    else launch_conv_t<float>(a, max_cb, quad, loaders, uniform_walk, grid, s);
    return hipGetLastError();
}

}  // namespace mt
