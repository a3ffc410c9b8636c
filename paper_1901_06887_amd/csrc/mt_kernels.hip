// Device code of the multi-tenant worker runtime, written for gfx950 (CDNA4, wave64).
//
//   batcher_kernel      tenant segmentation of the pending requests (counts, 32-aligned offsets,
//                       stable permutation) and the per-layer grouped-work tile lists, on device
//   gather_kernel       submitted rows -> tenant-contiguous bricks (FC models whose layer 0
//                       cannot read the submitted rows itself)
//   gather_image_kernel submitted images -> channel-padded NHWC rows (CNN models)
//   fc_kernel           one FC layer index for all tenants, weight-streaming tiles: weight bricks
//                       go from memory into MFMA operands through a register ring, activation
//                       bricks are shared through LDS; fused bias + activation (+ rounding),
//                       brick output, fp32 logits, or softmax/argmax for at most 32 classes
//   fc_big_kernel       the same layer index, compute-bound tenant-layers: 256x256 tiles, both
//                       operands through an LDS ring filled by direct global->LDS loads
//   conv_kernel         one conv layer index for all tenants, layers at most 32 channels wide:
//                       implicit-GEMM 3x3 convolution, every wave gathers its own pixels
//   conv_lds_kernel     wider conv layers: activation bricks gathered once per tile into LDS by
//                       direct global->LDS loads and shared by waves side by side over channels
//   gap_kernel          global average pooling, NHWC rows -> bricks
//   head_kernel         softmax + argmax, written in submission order
//   copy_kernel         plain copy, the yardstick for byte counters
//
// A DNN is a fixed sequence of layers applied in turn (paper, section 1.1); a worker
// hosts many tenants' DNNs and multiplexes their requests (section 3).  The grouping
// of all tenants' work for one layer index into one launch is this runtime's way of
// doing that multiplexing on one GPU.
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

// Index of the segment that holds submission row r (segments are sorted by row_begin).
__device__ __forceinline__ uint32_t find_segment(const Segment* segs, uint32_t n, uint32_t r)
{
    uint32_t lo = 0, hi = n;            // invariant: segs[lo].row_begin <= r
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].row_begin <= r) lo = mid; else hi = mid;
    }
    return lo;
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

// Exclusive scan of data[0..n) in LDS by the whole workgroup (n <= kMaxTenantsPadded);
// returns the total.  tmp must hold 17 words.
__device__ uint32_t block_exclusive_scan(uint32_t* data, uint32_t n, uint32_t* tmp)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t ipt = ceil_div(n, kBatchThreads);
    const uint32_t begin = tid * ipt, end = min(begin + ipt, n);
    static_assert(kBatchThreads / 64 == 16, "the wave totals are one row of 16 lanes");
    uint32_t s = 0;
    for (uint32_t i = begin; i < end; ++i) s += data[i];
    const uint32_t incl = wave_inclusive_scan(s);
    if (lane == 63) tmp[w] = incl;
    __syncthreads();
    if (w == 0) {
        const uint32_t c = lane < 16 ? tmp[lane] : 0;
        const uint32_t inc = row16_inclusive_scan(c);
        if (lane < 16) tmp[lane] = inc - c;
        if (lane == 15) tmp[16] = inc;
    }
    __syncthreads();
    uint32_t run = tmp[w] + incl - s;
    for (uint32_t i = begin; i < end; ++i) { uint32_t c = data[i]; data[i] = run; run += c; }
    uint32_t total = tmp[16];
    __syncthreads();
    return total;
}

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

constexpr uint32_t kLists = kListKinds * MT_MAX_LAYERS;   // FC, conv and big-FC tile-count arrays of every layer index

// Tenant segmentation and grouped-work descriptors.  One workgroup; every step is
// deterministic: rows of a tenant keep their arrival order (stable counting sort).  Equal
// tenant ids inside a wavefront are found with one ballot per id bit, so a step costs the
// same whatever the tenant mix is.  Latency, not bandwidth, bounds this kernel, so everything
// that does not depend on the rows (tenant and layer facts) is fetched up front, tenant ids
// are fetched one step ahead, and all tile-count arrays are scanned in one pass.
// NSLOT: tenants per thread (1 for up to 1024 tenants, else 2).  ITERS: rows a lane may keep in
// registers (64 * ITERS rows per wave); the launcher picks the smallest instantiation that
// covers the batch, because the unrolled steps of a larger one cost small batches microseconds.
// A row's packed position is known: note it both ways; a rejected row (t < 0: unknown tenant or
// no model) is answered at once with label -1 and zero rows.
__device__ __forceinline__ void place_row(const BatchArgs& a, uint32_t r, int32_t t, uint32_t position)
{
    int32_t pos = -1;
    if (t >= 0) {
        pos = (int32_t)position;
        a.perm[pos] = (int32_t)r;
    } else {
        a.out.labels[r] = -1;
        if (a.out.n_classes) a.out.n_classes[r] = 0;
        for (uint32_t c = 0; c < a.out.row_stride; ++c) {
            if (a.out.probs) a.out.probs[(size_t)r * a.out.row_stride + c] = 0.0f;
            if (a.out.logits) a.out.logits[(size_t)r * a.out.row_stride + c] = 0.0f;
        }
    }
    a.pos_of[r] = pos;
}

// Placement pass for large batches (after rank_kernel and the batcher): one row per thread;
// position = the tenant's first row + rows of the tenant in earlier ranking workgroups + rank.
__global__ __launch_bounds__(kBatchThreads) void place_kernel(BatchArgs a)
{
    const uint32_t r = blockIdx.x * kRankRows + threadIdx.x;
    if (r >= a.R) return;
    uint32_t Tp = 64;
    while (Tp < a.T) Tp <<= 1;
    const int32_t t = a.row_tenant[r];
    place_row(a, r, t, t >= 0 ? a.off[t] + a.hist_g[blockIdx.x * Tp + t] + a.row_rank[r] : 0);
}

// Ranking pass for large batches, spread over the chip: workgroup g takes rows
// [g * kRankRows, (g + 1) * kRankRows), one per thread.  Equal tenants inside a wave are matched
// with ballots as in the batcher; the 16 waves' counts are combined in wave order, so a row's
// rank counts the earlier rows of its tenant in the workgroup (arrival order is kept).
template <bool ONE_SEG>
__global__ __launch_bounds__(kBatchThreads) void rank_kernel(BatchArgs a)
{
    static_assert(kRankRows == (int)kBatchThreads, "one row per thread");
    __shared__ uint32_t whist[(kBatchThreads / 64) * kRankMaxTenants];
    __shared__ Segment seg_l[kSegsInLds];
    const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t T = a.T, R = a.R, r = blockIdx.x * kRankRows + tid;
    uint32_t Tp = 64;
    while (Tp < T) Tp <<= 1;
    const uint32_t bits = T > 1 ? 32 - __builtin_clz(T - 1) : 0;
    const Segment* segs = a.segs;
    if (!ONE_SEG && a.n_segs <= kSegsInLds) {
        for (uint32_t i = tid; i < a.n_segs; i += kBatchThreads) seg_l[i] = a.segs[i];
        segs = seg_l;
    }
    for (uint32_t i = tid; i < (kBatchThreads / 64) * Tp; i += kBatchThreads) whist[i] = 0;
    __syncthreads();
    int32_t t = -1;
    if (r < R) {
        if (ONE_SEG) {
            a.row_src[r] = (const uint8_t*)a.first.src + (size_t)r * a.first.row_stride * a.elem_size;
            t = a.first.ids ? a.first.ids[r] : a.first.tenant;
        } else {
            const Segment& sg = segs[find_segment(segs, a.n_segs, r)];
            a.row_src[r] = (const uint8_t*)sg.src + (size_t)(r - sg.row_begin) * sg.row_stride * a.elem_size;
            t = sg.ids ? sg.ids[r - sg.row_begin] : sg.tenant;
        }
        if (t < 0 || (uint32_t)t >= T || !a.tenants[t].registered) t = -1;
        a.row_tenant[r] = t;
    }
    uint64_t peers = __ballot(t >= 0);
    for (uint32_t b = 0; b < bits; ++b) {
        const bool bit = (t >> b) & 1;
        const uint64_t m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    const uint32_t rank = __popcll(peers & ((1ull << lane) - 1));
    if (t >= 0 && rank == 0) whist[w * Tp + t] = __popcll(peers);        // the first of its tenant in this wave
    __syncthreads();
    for (uint32_t u = tid; u < Tp; u += kBatchThreads) {
        uint32_t cnt[kBatchThreads / 64];
#pragma unroll
        for (uint32_t i = 0; i < kBatchThreads / 64; ++i) cnt[i] = whist[i * Tp + u];
        uint32_t run = 0;
#pragma unroll
        for (uint32_t i = 0; i < kBatchThreads / 64; ++i) { whist[i * Tp + u] = run; run += cnt[i]; }
        a.hist_g[blockIdx.x * Tp + u] = run;
    }
    __syncthreads();
    if (t >= 0) a.row_rank[r] = whist[w * Tp + t] + rank;
}

template <bool ONE_SEG, int NSLOT, int ITERS, bool PRE = false>
__global__ __launch_bounds__(kBatchThreads) void batcher_kernel(BatchArgs a)
{
    __shared__ uint32_t hist[kHistEntries];
    __shared__ uint32_t Ml[kMaxTenantsPadded];
    __shared__ uint32_t offl[kMaxTenantsPadded];
    __shared__ uint8_t regl[kMaxTenantsPadded];
    __shared__ uint32_t tmp[17];
    __shared__ uint32_t wtot[kBatchThreads / 64][kLists];
    __shared__ Segment seg_l[kSegsInLds];
    __shared__ uint32_t big_total[MT_MAX_LAYERS];
    __shared__ uint32_t carry_l[kLists];

    const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t T = a.T, R = a.R;
    if (tid < MT_MAX_LAYERS) big_total[tid] = 0;       // first read is several barriers away
    uint32_t Tp = 64;
    while (Tp < T) Tp <<= 1;
    const uint32_t bits = T > 1 ? 32 - __builtin_clz(T - 1) : 0;      // valid ids are below T
    constexpr uint32_t nslots = NSLOT;
    constexpr uint32_t kRegIters = ITERS;

    // Every global load the kernel depends on is issued before the first wait: the lane's tenant
    // ids (register path, below), the tenant facts and -- unconditionally, so that they do not
    // wait for the tenant facts -- the layer facts of tenants tid and tid + 1024.
    // PRE: the rows were ranked by rank_kernel; its workgroups stand where the waves stand otherwise
    const uint32_t nw = PRE ? a.n_rank_groups : min(kBatchThreads / 64, (uint32_t)kHistEntries / Tp);
    const uint32_t chunk = PRE ? (uint32_t)kRankRows : ceil_div(ceil_div(R, nw), 64) * 64;          // rows per wave
    const bool in_regs = !PRE && ONE_SEG && chunk <= 64 * kRegIters;     // a lane keeps its rows' ids and ranks in registers
    const uint32_t begin = w * chunk, end = w < nw ? min(begin + chunk, R) : begin;
    int32_t tq[kRegIters];               // first the submitted id, then rank << 11 | tenant (or -1): ids and in-wave ranks are below 2048
    static_assert(kMaxTenantsPadded <= 2048 && 64 * kRegIters <= (1u << 21), "packing of tenant and rank");
    if (in_regs) {
#pragma unroll
        for (uint32_t it = 0; it < kRegIters; ++it) {
            const uint32_t r = begin + it * 64 + lane;
            tq[it] = -1;
            if (r < end) {
                a.row_src[r] = (const uint8_t*)a.first.src + (size_t)r * a.first.row_stride * a.elem_size;
                tq[it] = a.first.ids ? a.first.ids[r] : a.first.tenant;
            }
        }
    }

    // column groups per layer (0 = no tiles), rows per request with the kind in the top bit
    // (1 = conv; FC: 64-row tiles count 1, 32-row tiles 2), padded width; from the 64 bytes of
    // layer facts the host keeps per tenant
    uint32_t grp[NSLOT][MT_MAX_LAYERS], rpr[NSLOT][MT_MAX_LAYERS], npad[NSLOT][MT_MAX_LAYERS];
    static_assert(MT_MAX_LAYERS == 8, "a tenant's layer facts are four 16-byte loads");
#pragma unroll
    for (uint32_t slot = 0; slot < nslots; ++slot) {
        const uint32_t t = tid + slot * kBatchThreads;
        const bool live = t < T;
        u32x4 q[4] = {};
        uint32_t reg = 0;
        if (live) {
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i) q[i] = ((const u32x4*)a.facts)[t * 4 + i];
            reg = a.tenants[t].registered;
        }
        if (t < Tp) regl[t] = live && reg;
#pragma unroll
        for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
            const uint32_t w0 = reg ? q[l / 2][2 * (l % 2)] : 0, w1 = q[l / 2][2 * (l % 2) + 1];
            const bool conv = w0 >> 31;
            grp[slot][l] = w0 & 0x3fffffffu;
            rpr[slot][l] = conv ? (w1 | 0x80000000u) : 1u + ((w0 >> 30) & 1);
            npad[slot][l] = conv ? 0 : w1;
        }
    }

    // the segment table sits in host memory: stage it in LDS when it is small
    const Segment* segs = a.segs;
    if (!ONE_SEG && a.n_segs <= kSegsInLds) {
        for (uint32_t i = tid; i < a.n_segs; i += kBatchThreads) seg_l[i] = a.segs[i];
        segs = seg_l;
    }
    for (uint32_t i = tid; i < nw * Tp; i += kBatchThreads) hist[i] = PRE ? a.hist_g[i] : 0;
    __syncthreads();

    // pass 1: per-wave histograms and in-wave ranks.  One step ranks 64 rows: equal tenant ids
    // are matched with one ballot per id bit.
    auto rank_step = [&](int32_t& t, uint32_t& rank_out) {
        if (t < 0 || (uint32_t)t >= T || !regl[t]) t = -1;
        uint64_t peers = __ballot(t >= 0);
        for (uint32_t b = 0; b < bits; ++b) {
            const bool bit = (t >> b) & 1;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const bool ok = t >= 0;
        const uint32_t leader = ok ? (uint32_t)__ffsll((unsigned long long)peers) - 1 : lane;
        const uint32_t rank = __popcll(peers & ((1ull << lane) - 1));
        uint32_t old = 0;
        if (ok && lane == leader) {
            old = hist[w * Tp + t];
            hist[w * Tp + t] = old + __popcll(peers);
        }
        old = __shfl(old, leader);
        rank_out = old + rank;
    };
    if (in_regs) {
#pragma unroll
        for (uint32_t it = 0; it < kRegIters; ++it) {
            if (begin + it * 64 < end) {                     // wave-uniform
                uint32_t rank;
                rank_step(tq[it], rank);
                const uint32_t r = begin + it * 64 + lane;
                if (r < end) a.row_tenant[r] = tq[it];
                if (tq[it] >= 0) tq[it] |= (int32_t)(rank << 11);
            }
        }
    } else if (!PRE && w < nw) {
        auto fetch_id = [&](uint32_t r) -> int32_t {
            if (r >= end) return -1;
            if (ONE_SEG) {                      // the whole batch is one submission: no table lookup
                a.row_src[r] = (const uint8_t*)a.first.src + (size_t)r * a.first.row_stride * a.elem_size;
                return a.first.ids ? a.first.ids[r] : a.first.tenant;
            }
            const Segment& sg = segs[find_segment(segs, a.n_segs, r)];
            a.row_src[r] = (const uint8_t*)sg.src + (size_t)(r - sg.row_begin) * sg.row_stride * a.elem_size;
            return sg.ids ? sg.ids[r - sg.row_begin] : sg.tenant;
        };
        int32_t t_next = begin < end ? fetch_id(begin + lane) : -1;
        for (uint32_t base = begin; base < end; base += 64) {
            const uint32_t r = base + lane;
            int32_t t = t_next;
            if (base + 64 < end) t_next = fetch_id(r + 64);
            uint32_t rank;
            rank_step(t, rank);
            if (r < end) { a.row_tenant[r] = t; if (t >= 0) a.row_rank[r] = rank; }
        }
    }
    __syncthreads();

    // pass 2: per-tenant totals, per-wave bases, tenant offsets (each tenant starts a 32-row block)
    for (uint32_t t = tid; t < Tp; t += kBatchThreads) {
        uint32_t s = 0;
        for (uint32_t i0 = 0; i0 < nw; i0 += 16) {            // 16 reads in flight together
            uint32_t cnt[16];
#pragma unroll
            for (uint32_t i = 0; i < 16; ++i) cnt[i] = i0 + i < nw ? hist[(i0 + i) * Tp + t] : 0;
#pragma unroll
            for (uint32_t i = 0; i < 16; ++i) { if (i0 + i < nw) hist[(i0 + i) * Tp + t] = s; s += cnt[i]; }
        }
        Ml[t] = s; offl[t] = ceil_div(s, kBrickRows) * kBrickRows;
    }
    __syncthreads();
    const uint32_t total = block_exclusive_scan(offl, Tp, tmp);
    for (uint32_t t = tid; t < T; t += kBatchThreads) {
        a.M[t] = Ml[t]; a.off[t] = offl[t];
        if (Ml[t]) { atomicAdd(&a.served[2 * t], (unsigned long long)Ml[t]); atomicAdd(&a.served[2 * t + 1], 1ull); }
        const uint32_t pend = offl[t] + ceil_div(Ml[t], kBrickRows) * kBrickRows;
        for (uint32_t p = offl[t] + Ml[t]; p < pend; ++p) a.perm[p] = -1;      // padding rows of the last block
    }
    if (tid == 0) a.off[T] = total;

    // pass 3: packed position of every row (pre-ranked batches: place_kernel, from the prefixes
    // over the ranking workgroups that are handed back here)
    auto place = [&](uint32_t r, int32_t t, uint32_t rank, uint32_t wave_of_row) {
        place_row(a, r, t, t >= 0 ? offl[t] + hist[wave_of_row * Tp + t] + rank : 0);
    };
    if (PRE) {
        for (uint32_t i = tid; i < nw * Tp; i += kBatchThreads) a.hist_g[i] = hist[i];
    } else if (in_regs) {
#pragma unroll
        for (uint32_t it = 0; it < kRegIters; ++it) {
            const uint32_t r = begin + it * 64 + lane;
            if (r < end) place(r, tq[it] < 0 ? -1 : (tq[it] & 2047), (uint32_t)tq[it] >> 11, w);
        }
    } else {
#pragma unroll 4
        for (uint32_t r = tid; r < R; r += kBatchThreads) {
            const int32_t t = a.row_tenant[r];
            place(r, t, t >= 0 ? a.row_rank[r] : 0, r / chunk);
        }
    }

    // Big tiles pay only when a layer index has enough of them to fill the chip; below that the
    // streaming kernel takes those tenants too, side by side with everyone else's tiles.
    uint32_t big_layers = 0;                   // bit l: layer index l is served with big tiles where a tenant qualifies
    if (a.big_enabled) {
        uint32_t bt[MT_MAX_LAYERS];
#pragma unroll
        for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) bt[l] = 0;
#pragma unroll
        for (uint32_t slot = 0; slot < nslots; ++slot) {
            const uint32_t t = tid + slot * kBatchThreads;
            const uint32_t Mt = t < Tp ? Ml[t] : 0;
#pragma unroll
            for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
                const uint32_t rr = rpr[slot][l], np = npad[slot][l];
                const uint32_t g = grp[slot][l];
                if (g && !(rr >> 31) && fc_is_big(Mt, np)) bt[l] += ceil_div(big_rows(Mt), kBigTile) * ceil_div(np, kBigTile);
            }
        }
#pragma unroll
        for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
            uint32_t v = bt[l];
            if (__any(v != 0)) {
                for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
                if (lane == 0) atomicAdd(&big_total[l], v);
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) big_layers |= (big_total[l] >= a.big_min_tiles ? 1u : 0u) << l;
    }
    if (tid == 0) *a.big_layers = big_layers;   // the FC kernels split a qualifying tenant's rows by it

    // pass 4: tile counts of every (kind, layer) list, scanned over tenants in one vector scan.
    // Only the exclusive in-wave prefix of each list stays in registers across the barriers; the
    // running total over slots lives in LDS.
    if (tid < kLists) carry_l[tid] = 0;
#pragma unroll
    for (uint32_t slot = 0; slot < nslots; ++slot) {
        const uint32_t t = tid + slot * kBatchThreads;
        const uint32_t Mt = t < Tp ? Ml[t] : 0;
        uint32_t excl[kLists];
        auto wave_scan = [&](uint32_t i, uint32_t c) {
            uint32_t v = c;
            if ((a.list_mask >> i) & 1) v = wave_inclusive_scan(c);       // lists no registered model contributes to are skipped
            excl[i] = v - c;
            if (lane == 63) wtot[w][i] = v;
        };
#pragma unroll
        for (uint32_t l = 0; l < MT_MAX_LAYERS; ++l) {
            const uint32_t g = grp[slot][l], rr = rpr[slot][l], np = npad[slot][l];
            const bool conv = rr >> 31;
            const bool big = !conv && ((big_layers >> l) & 1) && fc_is_big(Mt, np);
            // conv: rows = requests * output pixels per tile; FC: rr = 1 (64-row tiles) or 2 (32-row tiles),
            // over the rows that big tiles leave
            const uint32_t Mb = big ? big_rows(Mt) : 0;
            static_assert(kTileRows == 64, "FC tiles have 64 >> (rr - 1) rows");
            const uint32_t fc_shift = 7 - rr;                           // log2 of the FC tile's rows (rr is 1 or 2 there)
            const uint32_t tiles = (g && Mt) ? (conv ? ceil_div(Mt * (rr & 0x7fffffffu), kConvTileRows)
                                                     : (Mt - Mb + (1u << fc_shift) - 1) >> fc_shift) * g : 0;
            wave_scan(l, conv ? 0 : tiles);
            wave_scan(MT_MAX_LAYERS + l, conv ? tiles : 0);
            wave_scan(2 * MT_MAX_LAYERS + l, ceil_div(Mb, kBigTile) * ceil_div(np, kBigTile));
        }
        __syncthreads();
        if (tid < kLists * 16) {                 // a row of 16 lanes per list: exclusive prefix of its 16 wave totals
            const uint32_t i = tid >> 4, ww = tid & 15;
            const uint32_t x = wtot[ww][i], run = carry_l[i];
            const uint32_t inc = row16_inclusive_scan(x);
            wtot[ww][i] = run + inc - x;
            if (ww == 15) carry_l[i] = run + inc;
        }
        __syncthreads();
#pragma unroll
        for (uint32_t i = 0; i < kLists; ++i)              // lists outside the mask are never read
            if (((a.list_mask >> i) & 1) && t < T) a.tile_base[(size_t)i * (T + 1) + t] = wtot[w][i] + excl[i];
        __syncthreads();
    }
    if (tid < kLists && ((a.list_mask >> tid) & 1)) a.tile_base[(size_t)tid * (T + 1) + T] = carry_l[tid];
}

// ---- gather ------------------------------------------------------------------------------
// Images (first layer is a convolution): one workgroup per packed row, one thread per pixel;
// channels are padded with zeros to a multiple of 8 so that every tap of the implicit GEMM is
// a whole number of 16-byte chunks.
template <typename T>
__device__ void gather_image(const GatherArgs& a, const TenantDev& td, uint32_t p, uint32_t r)
{
    constexpr uint32_t EPC = 16 / sizeof(T);
    const T* src = (const T*)a.row_src[r];
    T* dst = (T*)a.act + (size_t)p * a.S;
    const uint32_t ci = td.in_cin ? td.in_cin : kChanPad, cp = td.in_cin ? td.in_cin_pad : kChanPad;
    const uint32_t npix = td.in_len / ci;
    for (uint32_t pix = threadIdx.x; pix < npix; pix += blockDim.x) {
        for (uint32_t g = 0; g < cp; g += EPC) {
            alignas(16) T tmp[EPC];
#pragma unroll
            for (uint32_t c = 0; c < EPC; ++c) tmp[c] = g + c < ci ? src[(size_t)pix * ci + g + c] : (T)0.0f;
            *(u32x4*)(dst + (size_t)pix * cp + g) = *(const u32x4*)tmp;
        }
    }
    for (uint32_t e = npix * cp + threadIdx.x; e < td.in_fill; e += blockDim.x) dst[e] = (T)0.0f;
}

__global__ __launch_bounds__(256) void gather_image_kernel(GatherArgs a)
{
    const uint32_t p = blockIdx.x;
    if (p >= a.off[a.T]) return;
    const int32_t r = a.perm[p];
    if (r < 0) return;
    const TenantDev td = a.tenants[a.row_tenant[r]];
    if (td.in_layout == kLayoutBricks) return;
    if (a.elem_size == 2) gather_image<__bf16>(a, td, p, (uint32_t)r); else gather_image<float>(a, td, p, (uint32_t)r);
}

// Vectors (first layer is FC): one workgroup per block of 32 packed rows, written as bricks.
template <typename T>
__device__ void gather_bricks(const GatherArgs& a, const TenantDev& td, uint32_t t, uint32_t p0)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t li = lane & 31, lh = lane >> 5;
    const uint32_t nKB = a.layers[t * MT_MAX_LAYERS].K / KB;
    const uint32_t seg0 = a.off[t];
    const int32_t r = a.perm[p0 + li];
    const T* src = r >= 0 ? (const T*)a.row_src[r] : nullptr;
    u32x4* dst = (u32x4*)((T*)a.act + (size_t)seg0 * a.S) + (size_t)((p0 - seg0) / kBrickRows) * nKB * 64 + lane;
    const uint32_t n = td.in_len;
    // Rows that are 16-byte aligned and a whole number of chunks long (the usual case) are copied
    // with four loads in flight per lane and no branch around them: chunks past the row's end
    // and padding rows read a block of zeros instead.
    const bool lane_ok = src == nullptr || (((uintptr_t)src & 15) == 0);
    if (n % EPC == 0 && __all(lane_ok)) {
        typedef const __attribute__((address_space(1))) u32x4* gptr_t;
        gptr_t row = (gptr_t)src, zeros = (gptr_t)a.zeros;
        const uint32_t nch = src ? n / EPC : 0;              // chunks this lane may read
        for (uint32_t kb0 = wave; kb0 < nKB; kb0 += 16) {
            u32x4 v[4];
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) {
                const uint32_t ch = (kb0 + 4 * j) * 2 + lh;
                v[j] = *(ch < nch ? row + ch : zeros);
            }
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j)
                if (kb0 + 4 * j < nKB) dst[(size_t)(kb0 + 4 * j) * 64] = v[j];
        }
        return;
    }
    for (uint32_t kb = wave; kb < nKB; kb += 4) {
        const uint32_t k = kb * KB + lh * EPC;
        u32x4 v = {0, 0, 0, 0};
        if (src && k < n) {
            if (k + EPC <= n && (((uintptr_t)(src + k)) & 15) == 0) {
                v = *(const u32x4*)(src + k);
            } else {
                alignas(16) T tmp[EPC];
#pragma unroll
                for (uint32_t e = 0; e < EPC; ++e) tmp[e] = k + e < n ? src[k + e] : (T)0.0f;
                v = *(const u32x4*)tmp;
            }
        }
        dst[(size_t)kb * 64] = v;
    }
}

__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a)
{
    const uint32_t p0 = blockIdx.x * kBrickRows;
    if (p0 >= a.off[a.T]) return;
    const int32_t r0 = a.perm[p0];        // the first row of a block is always a real request
    const uint32_t t = (uint32_t)a.row_tenant[r0];
    const TenantDev td = a.tenants[t];
    if (td.in_layout != kLayoutBricks) return;               // images have their own kernel
    if (a.elem_size == 2) gather_bricks<__bf16>(a, td, t, p0); else gather_bricks<float>(a, td, t, p0);
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
__device__ __forceinline__ float gelu(float x)
{
    constexpr float kScale = 0.84932180028801904f;           // sqrt(log2(e) / 2): zs = z * sqrt(log2 e)
    constexpr float kP = 0.3275911f / 1.2011224087864498f;   // p / sqrt(log2 e)
    const float ax = fabsf(x);
    const float zs = ax * kScale;
    const float t = __frcp_rn(fmaf(kP, zs, 1.0f));
    const float poly = t * (0.127414796f + t * (-0.142248368f + t * (0.7107068705f + t * (-0.7265760135f + t * 0.5307027145f))));
    const float h = poly * __builtin_amdgcn_exp2f(-zs * zs);
    return fmaf(-ax, h, fmaxf(x, 0.0f));
}

__device__ __forceinline__ float activate(float z, uint32_t act)
{
    if (act == MT_ACT_RELU) return fmaxf(z, 0.0f);
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
            for (int e = 0; e < 4; ++e) y[g][e] = fmaxf(y[g][e], 0.0f);
    }
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

// Tenant that owns logical tile `idx`: last t with base[t] <= idx (base is in LDS, base[T] > idx).
__device__ __forceinline__ uint32_t find_tenant(const uint32_t* base, uint32_t T, uint32_t idx)
{
    uint32_t lo = 0, hi = T;
    while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (base[mid] <= idx) lo = mid; else hi = mid; }
    return lo;
}

// ---- grouped FC ------------------------------------------------------------------------------
// A workgroup of four waves owns up to 64 rows (RB row blocks of 32) of one tenant and
// `split` column blocks of 32.  Weight bricks never touch LDS: every wave streams the bricks
// of its own column block straight from memory into MFMA B operands through a ring of
// registers that keeps P bricks in flight.
//   split == 4 (the common case): the four waves share the same activation bricks, so those
//     are staged once per workgroup in LDS, 16 bricks per chunk, double buffered, one barrier
//     per chunk; LDS reads of a brick are 16 contiguous bytes per lane, conflict free.
//   split < 4 (layers with at most 64 outputs): the waves also split K between them, read
//     their own activation bricks directly, and the partial sums are added in a fixed order
//     through LDS (deterministic, no atomics).
constexpr uint32_t kRedFloats = 4 * 16 * 64;                 // one f32x16 per lane per wave
constexpr uint32_t kTrRowBytes = 32 * 4 + 16;                // transposition scratch row (fp32 worst case)
constexpr uint32_t kTrBytes = 32 * kTrRowBytes;
constexpr uint32_t kChunkBricks = 16;                        // activation bricks per LDS stage
constexpr uint32_t kStageBytes = kChunkBricks * kBrickBytes;
// LDS of the FC kernel, 34 KiB so that four workgroups fit a CU.  K loop: two activation
// stages (split == 4).  After the K loop: reduction scratch (split < 4 only) at offset 0 and
// transposition scratch at kTrOffset; both alias the stages, separated from them by barriers.
constexpr uint32_t kTrOffset = kRedFloats * 4;
constexpr uint32_t kFcLdsBytes = kTrOffset + 4 * kTrBytes;
static_assert(kFcLdsBytes >= 2 * kStageBytes, "the two activation stages must fit");

// split == 4: activations through LDS, weights through the register ring.
template <typename T, int RB, bool GATHER>
__device__ __forceinline__ void fc_accumulate_shared(const GemmArgs& a, const Tile& tl, const LayerDev& L, uint32_t seg0,
                                                     uint32_t nb, bool active, uint8_t* stages, f32x16 (&acc)[RB])
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    constexpr uint32_t KC = kChunkBricks / RB;               // k steps per chunk: 16 or 8
    constexpr uint32_t P = 16;                               // weight bricks in flight per wave
    constexpr uint32_t U = P > KC ? P : KC;                  // unrolled block of k steps
    static_assert(U == P && U % KC == 0, "the tail relies on U == P");
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t nKB = L.K / KB;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    const uint32_t nb_eff = active ? nb : 0;                 // idle waves still help staging; they stream block 0 and drop it
    const u32x4* wp = (const u32x4*)(a.arena + L.w_off) + (size_t)nb_eff * nKB * 64 + lane;
    const u32x4* xbase = (const u32x4*)((const T*)a.act_in + (size_t)seg0 * a.S) + lane;

    // this wave stages bricks q = 4*wave .. 4*wave+3 of every chunk: row block q / KC, k step q % KC
    const u32x4* xsrc[4]; uint32_t xkk[4];
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        const uint32_t q = wave * 4 + j, r = q / KC;
        xkk[j] = q % KC;
        const uint32_t rbi = tl.m0 / kBrickRows + min(r, nrb - 1);     // blocks past the tile repeat its last one
        xsrc[j] = xbase + (size_t)rbi * nKB * 64;
    }
    // GATHER (layer 0): the bricks are formed on the fly from the submitted rows; this wave's
    // four bricks lie in one row block, so a lane reads from one row (null for padding rows)
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;     // submitted rows live in global memory
    gptr_t rowp = nullptr;
    bool row_ok = false;
    if (GATHER) {
        const uint32_t p0 = seg0 + (tl.m0 / kBrickRows + min(wave * 4 / KC, nrb - 1)) * kBrickRows;
        const int32_t r = a.perm[p0 + (lane & 31)];
        row_ok = r >= 0;
        // padding rows read the block's first row (always a real request) and discard it: no branch around the load
        rowp = (gptr_t)a.row_src[row_ok ? r : a.perm[p0]];
    }
    auto load_chunk = [&](uint32_t c, u32x4 (&xr)[4]) {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            if (GATHER) {
                const uint32_t k = (c * KC + xkk[j]) * KB + (lane >> 5) * EPC;
                const bool ok = row_ok && k < L.k_valid;
                const u32x4 v = rowp[(ok ? k : 0) / EPC];
                xr[j] = ok ? v : u32x4{0, 0, 0, 0};
            } else {
                xr[j] = xsrc[j][(size_t)min(c * KC + xkk[j], nKB - 1) * 64];
            }
        }
    };
    auto store_chunk = [&](uint32_t stage, const u32x4 (&xr)[4]) {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) *(u32x4*)(stages + stage * kStageBytes + (wave * 4 + j) * kBrickBytes + lane * 16) = xr[j];
    };

    // K is walked in blocks of U steps, unrolled, so that ring slots (step % P) and, where a
    // block spans two chunks, LDS stages are compile-time constants.  Slot s % P holds step s
    // from P steps before its use until its MFMAs; it is refilled with step s + P right after.
    // Loads return in order, so waiting for an activation load also waits for every weight
    // load issued before it.  The activation bricks of a chunk are therefore fetched as far
    // ahead as the weight ring reaches (NX chunks = P steps): by the time they are waited for,
    // every older weight load is one whose MFMA is due anyway, and the ring keeps its depth
    // across chunk boundaries (with one chunk of lookahead the 64-row tiles, whose chunks are 8
    // steps, had only the newest 8 weight loads in flight at every boundary; worth 1-2 % on the
    // skewed mixes).
    constexpr uint32_t NX = P / KC;                           // 1 (32-row tiles) or 2
    static_assert(NX >= 1 && U % (NX * KC) == 0, "a block of U steps starts with staging slot 0");
    u32x4 bq[P], xr[NX][4];
#pragma unroll
    for (uint32_t j = 0; j < P; ++j) bq[j] = wp[(size_t)min(j, nKB - 1) * 64];
    load_chunk(0, xr[0]);
    store_chunk(0, xr[0]);
#pragma unroll
    for (uint32_t i = 1; i <= NX; ++i) load_chunk(i, xr[i % NX]);   // zeros / clamped past the last chunk
    uint32_t c = 0;                                           // chunk being consumed; it lives in stage c & 1
    const uint8_t* st = stages + lane * 16;
    auto next_chunk = [&](uint32_t slot) {                    // slot = (c + 1) % NX, a constant at every call site
        lds_barrier();                                        // stage c&1 is complete; stage (c+1)&1 is free again
        store_chunk((c + 1) & 1, xr[slot]);
        load_chunk(c + 1 + NX, xr[slot]);
        st = stages + (c & 1) * kStageBytes + lane * 16;
        ++c;
    };
    const uint32_t n_blocks = nKB / U;
    for (uint32_t blk = 0; blk < n_blocks; ++blk) {
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (u % KC == 0) next_chunk((u / KC + 1) % NX);
            u32x4 av[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) av[r] = *(const u32x4*)(st + (r * KC + u % KC) * kBrickBytes);
#pragma unroll
            for (int r = 0; r < RB; ++r) Mma<T>::run(acc[r], av[r], bq[u % P]);
            bq[u % P] = wp[(size_t)min(blk * U + u + P, nKB - 1) * 64];
            // keeps the compiler from hoisting every LDS read of the block to its top (registers)
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const uint32_t rem = nKB - n_blocks * U;                  // < U == P: the ring already holds these steps
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
        if (u < rem) {
            if (u % KC == 0) next_chunk((u / KC + 1) % NX);
#pragma unroll
            for (int r = 0; r < RB; ++r) Mma<T>::run(acc[r], *(const u32x4*)(st + (r * KC + u % KC) * kBrickBytes), bq[u % P]);
        }
    }
}

// split < 4: every wave reads the activation bricks of its own K range directly.
template <typename T, int RB, int P, bool GATHER>
__device__ __forceinline__ void fc_accumulate_direct(const GemmArgs& a, const Tile& tl, const LayerDev& L, uint32_t seg0,
                                                     uint32_t nb, uint32_t kq, uint32_t ks, f32x16 (&acc)[RB])
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t nKB = L.K / KB;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    const uint32_t cnt = nKB / ks, kb0 = kq * cnt;
    const u32x4* wp = (const u32x4*)(a.arena + L.w_off) + ((size_t)nb * nKB + kb0) * 64 + lane;
    const u32x4* xbase = (const u32x4*)((const T*)a.act_in + (size_t)seg0 * a.S) + lane;
    const u32x4* xp[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const uint32_t rbi = tl.m0 / kBrickRows + min((uint32_t)r, nrb - 1);
        xp[r] = xbase + ((size_t)rbi * nKB + kb0) * 64;
    }
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;     // submitted rows live in global memory
    gptr_t rowp[RB]; bool row_ok[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        rowp[r] = nullptr; row_ok[r] = false;
        if (GATHER) {
            const uint32_t p0 = seg0 + (tl.m0 / kBrickRows + min((uint32_t)r, nrb - 1)) * kBrickRows;
            const int32_t row = a.perm[p0 + (lane & 31)];
            row_ok[r] = row >= 0;
            rowp[r] = (gptr_t)a.row_src[row_ok[r] ? row : a.perm[p0]];   // padding rows read a real row and discard it
        }
    }
    auto load_x = [&](int r, uint32_t kk) -> u32x4 {
        if (GATHER) {
            const uint32_t k = (kb0 + kk) * KB + (lane >> 5) * EPC;
            const bool ok = row_ok[r] && k < L.k_valid;
            const u32x4 v = rowp[r][(ok ? k : 0) / EPC];
            return ok ? v : u32x4{0, 0, 0, 0};
        }
        return xp[r][(size_t)kk * 64];
    };
    u32x4 bq[P], aq[RB][P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint32_t kk = min((uint32_t)j, cnt - 1);
        bq[j] = wp[(size_t)kk * 64];
#pragma unroll
        for (int r = 0; r < RB; ++r) aq[r][j] = load_x(r, kk);
    }
    // steady state: straight-line groups of P bricks, each slot refilled right after use; the
    // clamped refill index re-reads the last brick instead of branching
    const uint32_t full = cnt / P;
    for (uint32_t g = 0; g < full; ++g) {
#pragma unroll
        for (int j = 0; j < P; ++j) {
#pragma unroll
            for (int r = 0; r < RB; ++r) Mma<T>::run(acc[r], aq[r][j], bq[j]);
            const uint32_t kk = min(g * P + j + P, cnt - 1);
            bq[j] = wp[(size_t)kk * 64];
#pragma unroll
            for (int r = 0; r < RB; ++r) aq[r][j] = load_x(r, kk);
        }
    }
    const uint32_t rem = cnt - full * P;                      // the slots already hold the remaining bricks
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if ((uint32_t)j < rem) {
#pragma unroll
            for (int r = 0; r < RB; ++r) Mma<T>::run(acc[r], aq[r][j], bq[j]);
        }
    }
}

template <typename T, int RB, int P, bool GATHER>
__device__ __forceinline__ void fc_tile(const GemmArgs& a, const Tile& tl, const LayerDev& L, uint32_t Mt, uint8_t* smem)
{
    const uint32_t t = tl.tenant, split = tl.split;
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t li = lane & 31, lh = lane >> 5;
    const uint32_t ks = 4 / split;
    const uint32_t nb = tl.n0 / kBrickRows + (wave % split), kq = wave / split;
    const bool active = nb < L.N_pad / kBrickRows;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    const uint32_t seg0 = a.off[t];
    float* red = (float*)smem;                                // both alias the stages, used after the K loop only
    uint8_t* tr = smem + kTrOffset;

    f32x16 acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[r][v] = 0.0f;

    if (ks == 1) {
        fc_accumulate_shared<T, RB, GATHER>(a, tl, L, seg0, nb, active, smem, acc);
    } else {
        if (active) fc_accumulate_direct<T, RB, P, GATHER>(a, tl, L, seg0, nb, kq, ks, acc);
        // waves with kq > 0 hand their partial sums to the kq == 0 wave of the same column block
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            __syncthreads();
            if (active && kq > 0 && (uint32_t)r < nrb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) red[wave * 1024 + v * 64 + lane] = acc[r][v];
            }
            __syncthreads();
            if (active && kq == 0 && (uint32_t)r < nrb) {
                for (uint32_t q = 1; q < ks; ++q) {
                    const uint32_t src = (wave % split) + split * q;
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[r][v] += red[src * 1024 + v * 64 + lane];
                }
            }
        }
    }

    const bool writer = active && kq == 0;
    const uint32_t n = nb * kBrickRows + li;
    const float* bias = (const float*)(a.arena + L.b_off);
    const float bv = writer ? bias[n] : 0.0f;
    if (L.is_last && a.fuse_head && split == 1) {
        // at most 32 classes: the writer wave holds whole rows of logits.  Transpose them
        // through LDS so that one lane owns one request, then softmax, argmax and the outputs.
        float* trw = (float*)(smem + kTrOffset + wave * kTrBytes);
        constexpr uint32_t FRS = kTrRowBytes / 4;
        const uint32_t C = L.N;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            __syncthreads();
            if (writer && (uint32_t)r < nrb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) trw[(8 * (v >> 2) + 4 * lh + (v & 3)) * FRS + li] = acc[r][v] + bv;
            }
            __syncthreads();
            const uint32_t m = tl.m0 + r * kBrickRows + li;
            if (writer && (uint32_t)r < nrb && lh == 0 && m < Mt) {
                const float* z = trw + li * FRS;
                const uint32_t sub = (uint32_t)a.perm[seg0 + m];
                float mx = z[0]; int32_t best = 0;
                for (uint32_t c = 1; c < C; ++c) if (z[c] > mx) { mx = z[c]; best = (int32_t)c; }   // lowest index on ties
                float sum = 0.0f;
                for (uint32_t c = 0; c < C; ++c) sum += __expf(z[c] - mx);
                const float inv = 1.0f / sum;
                a.out.labels[sub] = best;
                if (a.out.n_classes) a.out.n_classes[sub] = (int32_t)C;
                for (uint32_t c = 0; c < a.out.row_stride; ++c) {
                    if (a.out.probs) a.out.probs[(size_t)sub * a.out.row_stride + c] = c < C ? __expf(z[c] - mx) * inv : 0.0f;
                    if (a.out.logits) a.out.logits[(size_t)sub * a.out.row_stride + c] = c < C ? z[c] : 0.0f;
                }
            }
        }
        return;
    }
    if (L.is_last) {
        if (!writer || n >= L.N) return;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t m = tl.m0 + r * kBrickRows + 8 * (v >> 2) + 4 * lh + (v & 3);
                if ((uint32_t)r < nrb && m < Mt) a.logits[(size_t)(seg0 + m) * a.C_pad + n] = acc[r][v] + bv;
            }
        }
        return;
    }
    // hidden layer: bias, activation, rounding; transpose the 32x32 block through LDS so that
    // every lane ends up with 16 contiguous output bytes, then store whole bricks
    constexpr uint32_t TRS = 32 * sizeof(T) + 16;
    uint8_t* trw = tr + wave * kTrBytes;
    const uint32_t nKB_out = L.out_fill / KB;
    u32x4* obase = (u32x4*)((T*)a.act_out + (size_t)seg0 * a.S) + lane;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        __syncthreads();
        if (writer && (uint32_t)r < nrb) {
            f32x4 y[4];
#pragma unroll
            for (int v = 0; v < 16; ++v) y[v >> 2][v & 3] = acc[r][v] + bv;
            activate_block<4>(y, L.act);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t ml = 8 * (v >> 2) + 4 * lh + (v & 3);
                *(T*)(trw + ml * TRS + li * sizeof(T)) = (T)(n < L.N ? y[v >> 2][v & 3] : 0.0f);
            }
        }
        __syncthreads();
        if (writer && (uint32_t)r < nrb) {
#pragma unroll
            for (uint32_t c = 0; c < kBrickRows / KB; ++c) {
                const u32x4 chunk = *(const u32x4*)(trw + li * TRS + (c * KB + lh * EPC) * sizeof(T));
                const uint32_t kb_out = nb * (kBrickRows / KB) + c;
                obase[((size_t)(tl.m0 / kBrickRows + r) * nKB_out + kb_out) * 64] = chunk;
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void fc_kernel(GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[kFcLdsBytes];    // also holds tile_base during the lookup
    uint32_t* base_l = (uint32_t*)smem;
    static_assert(kFcLdsBytes >= (kMaxTenantsPadded + 1) * 4, "tile_base must fit");
    const uint32_t n_tiles = a.tile_base[a.T];
    for (uint32_t i = threadIdx.x; i <= a.T; i += 256) base_l[i] = a.tile_base[i];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    __syncthreads();
    Tile tl;
    tl.tenant = __builtin_amdgcn_readfirstlane(find_tenant(base_l, a.T, idx));   // uniform: the tenant's facts come through scalar loads
    const uint32_t local = __builtin_amdgcn_readfirstlane(idx - base_l[tl.tenant]);
    __syncthreads();                                          // the lookup is over before anything reuses smem
    const LayerDev L = a.layers[tl.tenant * MT_MAX_LAYERS + a.layer];
    const uint32_t Mt = a.M[tl.tenant];
    uint32_t groups, trows;
    fc_shape(L.N_pad, a.fc_split_k, &tl.split, &groups, &trows);
    // where big tiles serve this tenant-layer, only the rows they leave are tiled here
    const bool big = ((*a.big_layers >> a.layer) & 1) && fc_is_big(Mt, L.N_pad);
    const uint32_t first = big ? big_rows(Mt) : 0;
    const uint32_t mt_ = ceil_div(Mt - first, trows);
    tl.m0 = first + (local % mt_) * trows;
    tl.rows = min(trows, Mt - tl.m0);
    tl.n0 = (local / mt_) * tl.split * kBrickRows;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    if (a.gather) {
        if (nrb <= 1) fc_tile<T, 1, 8, true>(a, tl, L, Mt, smem);
        else fc_tile<T, 2, 4, true>(a, tl, L, Mt, smem);
    } else {
        if (nrb <= 1) fc_tile<T, 1, 8, false>(a, tl, L, Mt, smem);
        else fc_tile<T, 2, 4, false>(a, tl, L, Mt, smem);
    }
}

// ---- grouped FC, big tiles ---------------------------------------------------------------
// Tenant-layers with at least kBigMinRows requests are compute bound.  They are cut into
// 256x256 output tiles; a workgroup of eight waves (2x4, 128x64 = 4x2 MFMA blocks per wave, two
// waves per SIMD so that one wave's operand fetches overlap the other's MFMAs) walks K two
// bricks at a time through a ring of four 32 KiB LDS stages.  Both operands arrive as bricks, so a
// stage is filled with straight 1 KiB copies (each wave copies two of the 16 row/column blocks) and
// read back with conflict-free 16-byte-per-lane loads.  Per k step a workgroup moves 16 KiB from L2
// for 64 MFMAs (half the operand traffic per flop of the 128x128 streaming tile) and reads
// 48 KiB from LDS, ~60 % of what the LDS pipe sustains with two waves per SIMD.
constexpr uint32_t kBigKS = 2;                                                   // k steps per stage
constexpr uint32_t kBigNS = 4;                                                   // stages in the LDS ring
constexpr uint32_t kBigBlocks = kBigTile / kBrickRows;                            // 8 row blocks, 8 column blocks
constexpr uint32_t kBigStageBytes = 2 * kBigBlocks * kBigKS * kBrickBytes;        // 32 KiB
constexpr uint32_t kBigGroup = 4;                                                 // row tiles that sweep the columns together

// WV waves per workgroup: 8 (2x4, 128x64 per wave) or 4 (2x2, 128x128 per wave, one wave per SIMD
// with its accumulators in the second half of the 512-entry register file).
template <typename T, int WV>
__global__ __launch_bounds__(WV * 64) void fc_big_kernel(GemmArgs a)
{
    constexpr uint32_t WN = WV / 2;                          // waves side by side
    constexpr uint32_t CJ = kBigBlocks / WN;                 // column blocks per wave (2 or 4)
    constexpr uint32_t BPW = 2 * kBigBlocks / WV;            // row/column blocks a wave stages (2 or 4)
    constexpr uint32_t LPS = BPW * kBigKS;                   // loads a wave issues per stage
    __shared__ __attribute__((aligned(16))) uint8_t stages[kBigNS * kBigStageBytes];
    uint8_t* const stage0 = stages;
    static_assert(kBigStageBytes >= (kMaxTenantsPadded + 1) * 4, "tile_base must fit the first stage");
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t li = lane & 31, lh = lane >> 5;

    uint32_t* base_l = (uint32_t*)stage0;                   // tile_base during the lookup
    const uint32_t n_tiles = a.tile_base[a.T];
    for (uint32_t i = tid; i <= a.T; i += WV * 64) base_l[i] = a.tile_base[i];
    uint32_t idx;
    if (!logical_tile_chunked(n_tiles, &idx)) return;
    __syncthreads();
    const uint32_t t = __builtin_amdgcn_readfirstlane(find_tenant(base_l, a.T, idx));   // uniform: the tenant's facts come through scalar loads
    const uint32_t local = __builtin_amdgcn_readfirstlane(idx - base_l[t]);
    __syncthreads();
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t Mt = a.M[t], seg0 = a.off[t];
    const uint32_t nKB = L.K / KB;
    // tile order inside a tenant: groups of kBigGroup row tiles sweep all column tiles together, so
    // the tiles that run at the same time on one XCD share few activation and weight panels (L2 reuse)
    const uint32_t Mb = big_rows(Mt);                      // a short remainder is the streaming kernel's
    const uint32_t mt_ = ceil_div(Mb, kBigTile), nt_ = ceil_div(L.N_pad, kBigTile);
    const uint32_t per_group = kBigGroup * nt_, grp = local / per_group, first_m = grp * kBigGroup;
    const uint32_t gsz = min(mt_ - first_m, kBigGroup), in_grp = local - grp * per_group;
    const uint32_t m0 = (first_m + in_grp % gsz) * kBigTile, n0 = (in_grp / gsz) * kBigTile;
    const uint32_t rows = min((uint32_t)kBigTile, Mb - m0), nrb = ceil_div(rows, kBrickRows);
    const uint32_t ncb = min(kBigBlocks, L.N_pad / kBrickRows - n0 / kBrickRows);
    const uint32_t wm = wave / WN, wn = wave % WN;

    // staging: waves 0..3 copy the 8 activation row blocks, waves 4..7 the 8 weight column blocks
    // (blocks past the tile or the layer repeat the last valid one)
    // staging: the first half of the waves copies the 8 activation row blocks, the second half the
    // 8 weight column blocks, BPW blocks each (blocks past the tile or the layer repeat the last valid one)
    const u32x4* lp[BPW];
    {
        const u32x4* xbase = (const u32x4*)((const T*)a.act_in + (size_t)seg0 * a.S) + lane;
        const u32x4* wbase = (const u32x4*)(a.arena + L.w_off) + lane;
#pragma unroll
        for (uint32_t i = 0; i < BPW; ++i) {
            if (wave < WV / 2) lp[i] = xbase + (size_t)(m0 / kBrickRows + min(wave * BPW + i, nrb - 1)) * nKB * 64;
            else lp[i] = wbase + (size_t)(n0 / kBrickRows + min((wave - WV / 2) * BPW + i, ncb - 1)) * nKB * 64;
        }
    }
    f32x16 acc[4][CJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < (int)CJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Operands travel HBM/L2 -> LDS without passing through registers (16 bytes per lane, the
    // hardware places lane l at base + 16 l, which is exactly a brick), three stages ahead of
    // their use.  A wave issues four such loads per stage, so "stage s has landed" is "at most
    // eight of my loads are outstanding"; the barrier that follows extends that to every wave's
    // share and also says that everyone is done reading the stage about to be overwritten.
    typedef const __attribute__((address_space(1))) void* gvoid_t;
    typedef __attribute__((address_space(3))) void* lvoid_t;
    auto issue_stage = [&](uint32_t slot, uint32_t s) {      // data of stage s into ring slot `slot`
        uint8_t* dst = stages + (slot % kBigNS) * kBigStageBytes + (wave * BPW) * kBigKS * kBrickBytes;
#pragma unroll
        for (uint32_t i = 0; i < BPW; ++i)
#pragma unroll
            for (uint32_t kk = 0; kk < kBigKS; ++kk)
                __builtin_amdgcn_global_load_lds((gvoid_t)(lp[i] + (size_t)(s * kBigKS + kk) * 64),
                                                 (lvoid_t)(dst + (i * kBigKS + kk) * kBrickBytes), 16, 0, 0);
    };
    // MFMA operands of one k step: 4 activation bricks and 2 weight bricks of this wave
    auto read_ops = [&](const uint8_t* buf, uint32_t kk, u32x4 (&a4)[4], u32x4 (&b2)[CJ]) {
        const uint8_t* ab = buf + (wm * 4 * kBigKS) * kBrickBytes + lane * 16;
        const uint8_t* bb = buf + ((kBigBlocks + wn * CJ) * kBigKS) * kBrickBytes + lane * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i) a4[i] = *(const u32x4*)(ab + (i * kBigKS + kk) * kBrickBytes);
#pragma unroll
        for (int j = 0; j < (int)CJ; ++j) b2[j] = *(const u32x4*)(bb + (j * kBigKS + kk) * kBrickBytes);
    };
    auto mma_rows = [&](const u32x4 (&a4)[4], const u32x4 (&b2)[CJ], int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < (int)CJ; ++j) Mma<T>::run(acc[i][j], b2[j], a4[i]);   // weights as the row operand: see the epilogue
    };
    auto mma_all = [&](const u32x4 (&a4)[4], const u32x4 (&b2)[CJ]) { mma_rows(a4, b2, 0, 4); };
    static_assert(kBigKS == 2, "the loop below is written for two k steps per stage");

    // The two k steps of a stage use two operand register sets, X and Y.  LDS reads of one set
    // are always issued in front of the MFMAs of the other, and the second k step of a stage is
    // multiplied after the next stage's barrier, so neither the LDS latency nor the barrier
    // leaves the MFMA pipe without work.
    const uint32_t n_stages = nKB / kBigKS, last = n_stages - 1;   // nKB is a multiple of 4: at least two stages
    // The waits are spelled with the builtin so that the compiler's own wait-count bookkeeping
    // sees them (an asm wait is invisible to it, and it would then wait again, too strictly);
    // the empty asm statements keep memory operations from moving across the barrier.
    // Encoding: vmcnt in bits 3:0 (and 15:14), expcnt 6:4, lgkmcnt 11:8; a field at its maximum does not wait.
    constexpr uint32_t kOut = 2 * LPS;                       // loads of the two younger stages may stay in flight
    constexpr int kWaitVm = (int)((kOut & 15) | ((kOut >> 4) << 14) | 0x0070 | 0x0F00), kWaitVmLgkm0 = kWaitVm & ~0x0F00;
    auto ring_barrier = [&](bool lds_too) {
        if (lds_too) __builtin_amdgcn_s_waitcnt(kWaitVmLgkm0); else __builtin_amdgcn_s_waitcnt(kWaitVm);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
#pragma unroll
    for (uint32_t s = 0; s < kBigNS - 1; ++s) issue_stage(s, min(s, last));
    ring_barrier(false);                                                     // stage 0 is complete for every wave
    issue_stage(kBigNS - 1, min(kBigNS - 1, last));
    // A wave whose four row blocks all lie past the end of a ragged tile only helps with staging
    // and barriers (its own loop, so that the working loop stays free of branches); its SIMD's
    // MFMA pipe is left to the wave that has rows.
    if (__builtin_amdgcn_readfirstlane(wm * 4 < nrb)) {
        u32x4 xa[4], xb[CJ], ya[4], yb[CJ];
        read_ops(stages, 0, xa, xb);
        read_ops(stages, 1, ya, yb);
        __builtin_amdgcn_sched_barrier(0);
        mma_all(xa, xb);
        for (uint32_t s = 1; s < n_stages; ++s) {
            // stage s is complete for every wave; every wave holds what it needs of stage s - 1 in
            // registers, so ring slot (s + 3) % 4 can be refilled
            ring_barrier(true);
            issue_stage(s + kBigNS - 1, min(s + kBigNS - 1, last));   // past the end: a harmless repeat keeps the count uniform
            const uint8_t* buf = stages + (s % kBigNS) * kBigStageBytes;
            read_ops(buf, 0, xa, xb);
            __builtin_amdgcn_sched_barrier(0);
            mma_all(ya, yb);                                          // second k step of stage s - 1
            __builtin_amdgcn_sched_barrier(0);
            mma_rows(xa, xb, 0, 1);                                   // first k step of stage s; its operands had the MFMAs above to arrive
            __builtin_amdgcn_sched_barrier(0);
            read_ops(buf, 1, ya, yb);                                 // issued behind the wait for X, so that wait does not cover them
            __builtin_amdgcn_sched_barrier(0);
            mma_rows(xa, xb, 1, 4);
            __builtin_amdgcn_sched_barrier(0);
        }
        mma_all(ya, yb);
    } else {
        for (uint32_t s = 1; s < n_stages; ++s) {
            ring_barrier(true);
            issue_stage(s + kBigNS - 1, min(s + kBigNS - 1, last));
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // trailing repeats landed, all reads done

    // epilogue.  The MFMAs took the weight bricks as their row operand, so a lane holds, for
    // activation row li of each block, outputs n = 8g + 4 lh + {0..3} (g = 0..3): runs of four
    // consecutive outputs of ITS row.  fp32: a run is a lane's 16 bytes of an output brick.
    // bf16: two lanes (lh = 0, 1) hold the halves of every 8-output run; one exchange between
    // the wave's halves per dword (v_permlane32_swap) leaves lanes lh = 0 with runs 0 and 2 and
    // lanes lh = 1 with runs 1 and 3, again a lane's 16 bytes of an output brick.  No LDS.  The
    // blocks are walked with a scheduling fence after each, which keeps the register need of the
    // epilogue at one block.
    const float* bias = (const float*)(a.arena + L.b_off);
    const uint32_t nKB_out = L.out_fill / KB;
    auto block = [&](const f32x16& blk, uint32_t i, uint32_t j) {
        const uint32_t rb = wm * 4 + i;
        if (rb < nrb && wn * CJ + j < ncb) {
            const uint32_t nb = n0 / kBrickRows + wn * CJ + j, nl = nb * kBrickRows + 4 * lh;   // first output of this lane's runs
            const uint32_t mb = m0 + rb * kBrickRows;          // first row of the block inside the tenant
            f32x4 y[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 bq = *(const f32x4*)(bias + nl + 8 * g);                            // bias is padded to N_pad
#pragma unroll
                for (int e = 0; e < 4; ++e) y[g][e] = blk[4 * g + e] + bq[e];
            }
            if (L.is_last) {
                if (mb + li < Mt) {
                    float* row = a.logits + (size_t)(seg0 + mb + li) * a.C_pad;
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        if (nl + 8 * g < L.N) *(f32x4*)(row + nl + 8 * g) = y[g];                 // may run into the row's padding (C_pad >= N_pad)
                }
            } else {
                u32x4* out = (u32x4*)((T*)a.act_out + (size_t)seg0 * a.S) +
                             ((size_t)(mb / kBrickRows) * nKB_out + nb * (kBrickRows / KB)) * 64 + lane;
                // outputs past N need no masking: their weight rows and bias are zero padding, and
                // every activation of the layer set maps 0 to 0
                activate_block<4>(y, L.act);
                if constexpr (sizeof(T) == 4) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) out[g * 64] = __builtin_bit_cast(u32x4, y[g]);   // brick g of the block, half lh
                } else {
                    uint32_t pk[4][2];                                                          // run halves as two packed dwords
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        T o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (T)y[g][e];
                        const uint64_t q = __builtin_bit_cast(uint64_t, o);
                        pk[g][0] = (uint32_t)q; pk[g][1] = (uint32_t)(q >> 32);
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {                                              // runs (0,1) -> brick 0 of the block, (2,3) -> brick 1
                        const auto s0 = __builtin_amdgcn_permlane32_swap(pk[2 * h][0], pk[2 * h + 1][0], false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(pk[2 * h][1], pk[2 * h + 1][1], false, false);
                        out[h * 64] = u32x4{s0[0], s1[0], s0[1], s1[1]};
                    }
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < (int)CJ; ++j) block(acc[i][j], i, j);
}

// ---- helpers of the implicit-GEMM convolutions ---------------------------------------------
// Quotient and remainder by a wave-uniform divisor; image sizes are mostly powers of two, and a
// general 32-bit division costs some thirty vector instructions per lane.
__device__ __forceinline__ void divmod_uniform(uint32_t x, uint32_t d, uint32_t* q, uint32_t* r)
{
    if ((d & (d - 1)) == 0) { *q = x >> __builtin_ctz(d); *r = x & (d - 1); }
    else { *q = x / d; *r = x - *q * d; }
}

// A lane's walk through K = (kernel row, kernel column, channel), one k step at a time.  Inside
// a kernel row the three taps of a pixel are one contiguous run of 3 * cin input elements, so the
// position is kept as (kernel row th, offset lin inside the run) and the element offset `cur`
// moves by KB per step plus a jump at the end of a run.  Validity is two range tests: the
// left/right tap falls outside the image only at the image's left/right edge, the top/bottom
// kernel row only at its top/bottom edge.  Steps past the last tap have th == 3: invalid.
template <typename T>
struct TapWalk {
    static constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    uint32_t lin, th, run, lo, hi, tlo, thi, step;
    int32_t cur, jump;
    // first: the lane's first element inside the run; step_el: elements per call of next()
    // (at most one run ends per call: step_el <= 3 * cin)
    __device__ __forceinline__ void init(const LayerDev& L, int32_t ih0, int32_t iw0, bool row_ok, uint32_t first, uint32_t step_el)
    {
        const int32_t cin = (int32_t)L.cin;
        run = 3 * L.cin; lin = first; th = 0; step = step_el;
        lo = iw0 < 0 ? L.cin : 0; hi = iw0 + 2 >= (int32_t)L.in_w ? 2 * L.cin : 3 * L.cin;
        tlo = ih0 < 0 ? 1 : 0; thi = row_ok ? (ih0 + 2 >= (int32_t)L.in_h ? 2 : 3) : 0;
        cur = (ih0 * (int32_t)L.in_w + iw0) * cin + (int32_t)lin;
        jump = ((int32_t)L.in_w - 3) * cin;
    }
    // the 16-byte chunk of this k step inside the image, or -1 when the step reads zeros; moves on
    __device__ __forceinline__ int32_t next()
    {
        const bool ok = (lin >= lo) & (lin < hi) & (th >= tlo) & (th < thi);
        const int32_t chunk = ok ? (int32_t)((uint32_t)cur / EPC) : -1;
        lin += step; cur += (int32_t)step;
        const bool wrap = lin >= run;
        lin = wrap ? lin - run : lin; th += wrap ? 1u : 0u; cur = wrap ? cur + jump : cur;
        return chunk;
    }
};

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

// ---- grouped 3x3 convolution as implicit GEMM ---------------------------------------------
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
    const int32_t ih0 = (int32_t)(oh * L.stride) - 1, iw0 = (int32_t)(ow * L.stride) - 1;
    gptr_t img = (gptr_t)((const T*)a.act_in + (size_t)(seg0 + req) * a.S);
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
    T* out = row_ok ? (T*)a.act_out + (size_t)(seg0 + req) * a.S + (size_t)pix * L.N : nullptr;
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
        store_unit_nhwc<T>(y, out ? out + nbase : nullptr, min((uint32_t)kBrickRows, L.N - nbase), scratch);
    }
}

// MAXCB bounds the channel blocks of any tile in the launch: narrow layers get a kernel with
// few registers and many resident waves, which is what hides the latency of their short K loops.
template <typename T, int MAXCB>
__global__ __launch_bounds__(256) void conv_kernel(GemmArgs a)
{
    __shared__ uint32_t base_l[kMaxTenantsPadded + 1];
    __shared__ __attribute__((aligned(16))) uint8_t unit_scratch[4 * unit_scratch_bytes<T>()];
    const uint32_t tid = threadIdx.x, wave = tid >> 6;
    uint8_t* scratch = unit_scratch + wave * unit_scratch_bytes<T>();
    const uint32_t n_tiles = a.tile_base[a.T];
    for (uint32_t i = tid; i <= a.T; i += 256) base_l[i] = a.tile_base[i];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    __syncthreads();
    const uint32_t t = __builtin_amdgcn_readfirstlane(find_tenant(base_l, a.T, idx));   // uniform: the tenant's facts come through scalar loads
    const uint32_t local = __builtin_amdgcn_readfirstlane(idx - base_l[t]);
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t seg0 = a.off[t];
    const uint32_t rows_total = a.M[t] * L.rows_per_req, mt_ = ceil_div(rows_total, kConvTileRows);
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
// for taps outside the image) and the hardware placing lane l at base + 16 l, which is brick
// order.  K is walked in chunks of kConvKC k steps through a ring of kConvNS stages, chunks
// kConvNS - 1 ahead of their use.
constexpr uint32_t kConvKC = 2, kConvNS = 3;
constexpr uint32_t kConvStageBytes = 8 * kConvKC * kBrickBytes;      // 4 pixel blocks + 4 filter areas, kConvKC k steps each

// QUAD (every tenant's input channels are a multiple of 4 chunks, i.e. a pixel's share of two k
// steps is 64 contiguous bytes): a gather instruction then takes 16 pixels with four consecutive
// lanes on one pixel's 64 bytes, instead of 32 pixels with one 16-byte piece per lane.  The
// texture path handles a lane quad on one cache line as one access, so the gather costs a quarter
// of the accesses.  The hardware's lane placement then yields [pixel][chunk] order instead of
// brick order; the MFMA operand read picks its 16 bytes from there (a 2-way bank conflict, on a
// path that has the time).
template <typename T, int NCB, bool QUAD>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void conv_lds_kernel(GemmArgs a)     // three workgroups per CU is what the LDS ring allows
{
    static_assert(!QUAD || kConvKC == 2, "a quad gather covers exactly two k steps");
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    constexpr uint32_t WR = 4 / NCB, RBW = 4 / WR;                  // wave rows; pixel blocks per wave
    typedef const __attribute__((address_space(1))) u32x4* gptr_t;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kConvNS * kConvStageBytes];
    static_assert(kConvNS * kConvStageBytes >= (kMaxTenantsPadded + 1) * 4, "tile_base must fit");
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, li = lane & 31, lh = lane >> 5;
    uint32_t* base_l = (uint32_t*)lds;
    const uint32_t n_tiles = a.tile_base[a.T];
    for (uint32_t i = tid; i <= a.T; i += 256) base_l[i] = a.tile_base[i];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    __syncthreads();
    const uint32_t t = __builtin_amdgcn_readfirstlane(find_tenant(base_l, a.T, idx));   // uniform: the tenant's facts come through scalar loads
    const uint32_t local = __builtin_amdgcn_readfirstlane(idx - base_l[t]);
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    const uint32_t seg0 = a.off[t];
    const uint32_t rpr = L.rows_per_req;
    const uint32_t rows_total = a.M[t] * rpr, mt_ = ceil_div(rows_total, kConvTileRows);
    const uint32_t m0 = (local % mt_) * kConvTileRows;
    const uint32_t nb0 = (local / mt_) * (kTileCols / kBrickRows);
    const uint32_t ncb = min((uint32_t)(kTileCols / kBrickRows), L.N_pad / kBrickRows - nb0);
    const uint32_t nKB = L.K / KB, nKBv = ceil_div(L.k_valid, KB);
    const uint32_t n_chunks = ceil_div(nKBv, kConvKC);             // n_chunks * kConvKC <= nKB: K is padded to 64
    const uint32_t wc = wave % NCB, wr = wave / NCB;
    const bool active = wc < ncb;                                  // idle waves still gather; they stream block 0 and drop it

    // gather role: pixel block `wave`.  Plain: this lane's pixel li, 16 bytes per k step.  QUAD:
    // pixels lane/4 and lane/4 + 16, chunk lane%4 of the 64 bytes that two k steps take of each.
    constexpr uint32_t NPX = QUAD ? 2 : 1;
    gptr_t zeros = (gptr_t)a.zeros;
    gptr_t img[NPX];
    TapWalk<T> walk[NPX];
#pragma unroll
    for (uint32_t i = 0; i < NPX; ++i) {
        const uint32_t gm = m0 + wave * kBrickRows + (QUAD ? (lane >> 2) + 16 * i : li);
        const bool row_ok = gm < rows_total;
        const uint32_t mm = row_ok ? gm : m0;
        uint32_t req, pix, oh, ow;
        divmod_uniform(mm, rpr, &req, &pix);
        divmod_uniform(pix, L.out_w, &oh, &ow);
        img[i] = (gptr_t)((const T*)a.act_in + (size_t)(seg0 + req) * a.S);
        walk[i].init(L, (int32_t)(oh * L.stride) - 1, (int32_t)(ow * L.stride) - 1, row_ok,
                     QUAD ? (lane & 3) * EPC : lh * EPC, QUAD ? 2 * KB : KB);
    }
    gptr_t wp = (gptr_t)((const u32x4*)(a.arena + L.w_off) + (size_t)(nb0 + (active ? wc : 0)) * nKB * 64 + lane);
    const uint32_t last_kb = n_chunks * kConvKC - 1;
    // The next kConvKC k steps of this wave's pixel block and of its filter block: 2 * kConvKC
    // loads.  Chunks past the end gather zeros (th >= 3) and repeat the last filter bricks, which
    // keeps the number of loads per round, and with it the wait below, uniform.
    auto fetch_chunk = [&](uint32_t c) {
        uint8_t* dst = lds + (c % kConvNS) * kConvStageBytes;
#pragma unroll
        for (uint32_t kk = 0; kk < kConvKC; ++kk) {
            // plain: k step kk of all 32 pixels; QUAD: both k steps of pixels 16 kk .. 16 kk + 15
            const int32_t chunk = walk[QUAD ? kk : 0].next();
            gptr_t p = chunk >= 0 ? img[QUAD ? kk : 0] + chunk : zeros;
            lds_dma16(p, dst + (wave * kConvKC + kk) * kBrickBytes);
            lds_dma16(wp + (size_t)min(c * kConvKC + kk, last_kb) * 64, dst + ((4 + wave) * kConvKC + kk) * kBrickBytes);
        }
    };
    // where lane (li, lh) finds its 16 bytes of k step kk inside a pixel block's area of a stage
    const uint32_t a_lane = QUAD ? (li * 4 + lh) * 16 : lane * 16;
    constexpr uint32_t a_kk = QUAD ? 32 : kBrickBytes;

    f32x16 acc[RBW];
#pragma unroll
    for (uint32_t r = 0; r < RBW; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[r][v] = 0.0f;

    __syncthreads();                                               // the lookup is over before the ring reuses the memory
#pragma unroll
    for (uint32_t c = 0; c < kConvNS - 1; ++c) fetch_chunk(c);
    // when chunk c is needed, the loads of the kConvNS - 2 younger chunks may still be in flight
    constexpr uint32_t kOut = (kConvNS - 2) * 2 * kConvKC;
    constexpr int kWaitVm = (int)((kOut & 15) | ((kOut >> 4) << 14) | 0x0070 | 0x0F00);
    for (uint32_t c = 0; c < n_chunks; ++c) {
        __builtin_amdgcn_s_waitcnt(kWaitVm);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();                              // chunk c is complete for every wave; everyone is done with chunk c - 1
        asm volatile("" ::: "memory");
        fetch_chunk(c + kConvNS - 1);
        const uint8_t* st = lds + (c % kConvNS) * kConvStageBytes;
#pragma unroll
        for (uint32_t kk = 0; kk < kConvKC; ++kk) {
            const u32x4 wv = *(const u32x4*)(st + ((4 + wave) * kConvKC + kk) * kBrickBytes + lane * 16);
#pragma unroll
            for (uint32_t r = 0; r < RBW; ++r) {
                const u32x4 av = *(const u32x4*)(st + (wr * RBW + r) * kConvKC * kBrickBytes + kk * a_kk + a_lane);
                Mma<T>::run(acc[r], wv, av);                       // rows = channels, columns = pixels
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");         // this wave's LDS reads of the chunk are done before its next barrier
    }
    // trailing loads have landed and every wave is done with the ring: its memory now serves as
    // the waves' store scratch
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    static_assert(kConvNS * kConvStageBytes >= 4 * unit_scratch_bytes<T>(), "store scratch aliases the ring");

    // epilogue: lane holds, for pixel li of each of its pixel blocks, channels 8g + 4 lh + {0..3}
    if (!active) return;
    uint8_t* scratch = lds + wave * unit_scratch_bytes<T>();
    const float* bias = (const float*)(a.arena + L.b_off);
    const uint32_t nbase = (nb0 + wc) * kBrickRows;
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
                const f32x4 bv = *(const f32x4*)(bias + nbase + 8 * g + 4 * lh);
#pragma unroll
                for (int i = 0; i < 4; ++i) y[g][i] = acc[r][4 * g + i] + bv[i];
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
                    T* out = (T*)a.act_out + (size_t)seg0 * a.S + (size_t)(req / kBrickRows) * nKBp * 64 * EPC;
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
            out = (T*)a.act_out + (size_t)(seg0 + req) * a.S + (size_t)pix * L.N + nbase;
        }
        f32x4 y[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 bv = *(const f32x4*)(bias + nbase + 8 * g + 4 * lh);   // bias is padded to N_pad; re-read per block (L1) to keep registers free
#pragma unroll
            for (int i = 0; i < 4; ++i) y[g][i] = acc[r][4 * g + i] + bv[i];
        }
        __builtin_amdgcn_sched_barrier(0);
        activate_block<4>(y, L.act);
        store_unit_nhwc<T>(y, out, min((uint32_t)kBrickRows, L.N - nbase), scratch);
    }
}

// ---- global average pool: one workgroup per packed row, NHWC row in, brick slice out ------
constexpr uint32_t kGapThreads = 128;
template <typename T>
__device__ void gap_row(const GapArgs& a, const LayerDev& L, uint32_t p, uint32_t seg0)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const T* in = (const T*)a.act_in + (size_t)p * a.S;
    const uint32_t C = L.cin, HW = L.in_h * L.in_w;
    const uint32_t m = p - seg0, rb = m / kBrickRows, i = m % kBrickRows;
    const uint32_t nKB = L.out_fill / KB;
    T* out = (T*)a.act_out + (size_t)seg0 * a.S + (size_t)rb * nKB * 64 * EPC;
    const float inv = 1.0f / (float)HW;
    const uint32_t CPP = C / EPC;                              // 16-byte chunks per pixel (C is a multiple of 8)
    if (C % EPC == 0 && CPP <= kGapThreads && kGapThreads % CPP == 0) {
        // 16 bytes per load: thread (pg, cg) sums chunk cg of pixels pg, pg + G, ...; the G partial
        // sums of a channel are then added in a fixed order through LDS
        __shared__ float part[kGapThreads * EPC];
        const uint32_t G = kGapThreads / CPP, cg = threadIdx.x % CPP, pg = threadIdx.x / CPP;
        float s[EPC];
#pragma unroll
        for (uint32_t e = 0; e < EPC; ++e) s[e] = 0.0f;
        const u32x4* src = (const u32x4*)in + cg;
#pragma unroll 4
        for (uint32_t q = pg; q < HW; q += G) {
            const u32x4 v = src[(size_t)q * CPP];
            const T* ve = (const T*)&v;
#pragma unroll
            for (uint32_t e = 0; e < EPC; ++e) s[e] += (float)ve[e];
        }
#pragma unroll
        for (uint32_t e = 0; e < EPC; ++e) part[(pg * CPP + cg) * EPC + e] = s[e];
        __syncthreads();
        for (uint32_t c = threadIdx.x; c < L.out_fill; c += kGapThreads) {
            float t = 0.0f;
            if (c < C) for (uint32_t g = 0; g < G; ++g) t += part[g * C + c];
            const uint32_t kb = c / KB, h = (c % KB) / EPC, e = c % EPC;
            out[((size_t)kb * 64 + i + 32 * h) * EPC + e] = (T)(t * inv);
        }
        return;
    }
    for (uint32_t c = threadIdx.x; c < L.out_fill; c += blockDim.x) {
        float s = 0.0f;
        if (c < C) for (uint32_t q = 0; q < HW; ++q) s += (float)in[(size_t)q * C + c];
        const uint32_t kb = c / KB, h = (c % KB) / EPC, e = c % EPC;
        out[((size_t)kb * 64 + i + 32 * h) * EPC + e] = (T)(s * inv);
    }
}

__global__ __launch_bounds__(kGapThreads) void gap_kernel(GapArgs a)
{
    const uint32_t p = blockIdx.x;
    if (p >= a.off[a.T]) return;
    const int32_t r = a.perm[p];
    if (r < 0) return;
    const uint32_t t = (uint32_t)a.row_tenant[r];
    if (a.tenants[t].n_layers <= a.layer) return;
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    if (L.kind != MT_GAP) return;
    if (a.elem_size == 2) gap_row<__bf16>(a, L, p, a.off[t]); else gap_row<float>(a, L, p, a.off[t]);
}

// ---- head: one wave per submitted row --------------------------------------------------
__global__ __launch_bounds__(256) void head_kernel(HeadArgs a)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= a.R) return;
    const int32_t pos = a.pos_of[r];
    uint32_t C = 0;
    int32_t label = -1;
    float mx = -INFINITY, sum = 0.0f;
    const float* z = nullptr;
    if (pos < 0) return;                                    // rejected rows were answered by the batcher
    C = a.tenants[a.row_tenant[r]].n_classes;
    if (C < a.min_classes) return;                          // finished by the FC kernel
    z = a.logits + (size_t)pos * a.C_pad;
    if (a.vec_ok && C <= 1024) {
        // the row lives in registers: 16 logits per lane (four 16-byte loads), read once
        f32x4 v[4];
        int32_t best = 0x7fffffff;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            const uint32_t c = (q * 64 + lane) * 4;
            v[q] = c < a.C_pad ? *(const f32x4*)(z + c) : f32x4{0, 0, 0, 0};   // C_pad is a multiple of 32
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i) {
                if (c + i >= C) v[q][i] = -INFINITY;
                if (v[q][i] > mx) { mx = v[q][i]; best = (int32_t)(c + i); }      // increasing index: the first hit is this lane's lowest
            }
        }
        for (int d = 32; d >= 1; d >>= 1) {
            const float omx = __shfl_xor(mx, d);
            const int32_t ob = __shfl_xor(best, d);
            if (omx > mx || (omx == mx && ob < best)) { mx = omx; best = ob; }
        }
        label = best;
        f32x4 e[4];
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q)
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i) { e[q][i] = __expf(v[q][i] - mx); sum += e[q][i]; }   // exp(-inf) = 0 past the last class
        for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
        const float inv = 1.0f / sum;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            const uint32_t c = (q * 64 + lane) * 4;
            if (c < a.out.row_stride) {
                f32x4 pr, lg;
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) { const bool in = c + i < C; pr[i] = in ? e[q][i] * inv : 0.0f; lg[i] = in ? v[q][i] : 0.0f; }
                if (a.out.probs) *(f32x4*)(a.out.probs + (size_t)r * a.out.row_stride + c) = pr;
                if (a.out.logits) *(f32x4*)(a.out.logits + (size_t)r * a.out.row_stride + c) = lg;
            }
        }
        // rows wider than 1024 entries: zero the rest
        for (uint32_t c = 1024 + lane; c < a.out.row_stride; c += 64) {
            if (a.out.probs) a.out.probs[(size_t)r * a.out.row_stride + c] = 0.0f;
            if (a.out.logits) a.out.logits[(size_t)r * a.out.row_stride + c] = 0.0f;
        }
    } else {
        int32_t best = 0x7fffffff;
        for (uint32_t c = lane; c < C; c += 64) {
            const float v = z[c];
            if (v > mx) { mx = v; best = (int32_t)c; }      // strided: first hit is the lowest index of this lane
        }
        for (int d = 32; d >= 1; d >>= 1) {
            const float omx = __shfl_xor(mx, d);
            const int32_t ob = __shfl_xor(best, d);
            if (omx > mx || (omx == mx && ob < best)) { mx = omx; best = ob; }
        }
        label = best;
        for (uint32_t c = lane; c < C; c += 64) sum += __expf(z[c] - mx);
        for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
        const float inv = 1.0f / sum;
        for (uint32_t c = lane; c < a.out.row_stride; c += 64) {
            const bool in = c < C;
            if (a.out.probs) a.out.probs[(size_t)r * a.out.row_stride + c] = in ? __expf(z[c] - mx) * inv : 0.0f;
            if (a.out.logits) a.out.logits[(size_t)r * a.out.row_stride + c] = in ? z[c] : 0.0f;
        }
    }
    if (lane == 0) {
        a.out.labels[r] = label;
        if (a.out.n_classes) a.out.n_classes[r] = (int32_t)C;
    }
}

// ---- launchers ------------------------------------------------------------------------------
hipError_t launch_batcher(const BatchArgs& a, hipStream_t s)
{
    const bool one = a.n_segs == 1, wide = a.T > kBatchThreads;
    // rows per lane of the register path, as the kernel derives them
    uint32_t Tp = 64;
    while (Tp < a.T) Tp <<= 1;
    const uint32_t nw = std::min<uint32_t>(kBatchThreads / 64, kHistEntries / Tp);
    const uint32_t iters = (((a.R + nw - 1) / nw) + 63) / 64;
    if (a.n_rank_groups) {                  // large batch: ranked across the chip first
        if (a.T > (uint32_t)kRankMaxTenants || (uint64_t)a.n_rank_groups * Tp > (uint64_t)kHistEntries ||
            (uint64_t)a.n_rank_groups * kRankRows < a.R) return hipErrorInvalidValue;
        if (one) hipLaunchKernelGGL(rank_kernel<true>, dim3(a.n_rank_groups), dim3(kBatchThreads), 0, s, a);
        else hipLaunchKernelGGL(rank_kernel<false>, dim3(a.n_rank_groups), dim3(kBatchThreads), 0, s, a);
        hipLaunchKernelGGL((batcher_kernel<false, 1, 4, true>), dim3(1), dim3(kBatchThreads), 0, s, a);
        hipLaunchKernelGGL(place_kernel, dim3(a.n_rank_groups), dim3(kBatchThreads), 0, s, a);
        return hipGetLastError();
    }
#define MT_BATCHER(SEG, NS, IT) hipLaunchKernelGGL((batcher_kernel<SEG, NS, IT>), dim3(1), dim3(kBatchThreads), 0, s, a)
    if (!one) { if (wide) MT_BATCHER(false, 2, 4); else MT_BATCHER(false, 1, 4); }      // many submissions: no register path
    else if (wide) MT_BATCHER(true, 2, 16);
    else if (iters <= 4) MT_BATCHER(true, 1, 4);
    else if (iters <= 8) MT_BATCHER(true, 1, 8);
    else if (iters <= 16) MT_BATCHER(true, 1, 16);
    else MT_BATCHER(true, 1, 32);
#undef MT_BATCHER
    return hipGetLastError();
}
hipError_t launch_gather(const GatherArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(gather_kernel, dim3(a.P / kBrickRows), dim3(256), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_gather_image(const GatherArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(gather_image_kernel, dim3(a.P), dim3(256), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_fc(const GemmArgs& a, uint32_t dtype, uint32_t grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 7) / 8 * 8;
    if (dtype == MT_BF16) hipLaunchKernelGGL(fc_kernel<__bf16>, dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(fc_kernel<float>, dim3(grid), dim3(256), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_fc_big(const GemmArgs& a, uint32_t dtype, uint32_t grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 8 * kXcdChunk - 1) / (8 * kXcdChunk) * (8 * kXcdChunk);
    // (the 4-wave shape, 128x128 per wave at one wave per SIMD, reads a third less from LDS per
    // MFMA but was measured 1.5x slower: a single wave per SIMD leaves the MFMA pipe idle at every wait)
    if (dtype == MT_BF16) hipLaunchKernelGGL((fc_big_kernel<__bf16, 8>), dim3(grid), dim3(512), 0, s, a);
    else hipLaunchKernelGGL((fc_big_kernel<float, 8>), dim3(grid), dim3(512), 0, s, a);
    return hipGetLastError();
}
// ---- plain copy: the yardstick for byte counters and streaming bandwidth -------------------
__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, uint64_t bytes, hipStream_t s)
{
    const uint64_t n = bytes / 16;
    if (n == 0) return hipSuccess;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((n + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, s, (u32x4*)dst, (const u32x4*)src, n);
    return hipGetLastError();
}

template <typename T>
static void launch_conv_t(const GemmArgs& a, uint32_t max_cb, bool quad, uint32_t grid, hipStream_t s)
{
    if (max_cb <= 1) hipLaunchKernelGGL((conv_kernel<T, 1>), dim3(grid), dim3(256), 0, s, a);
    else if (max_cb == 2 && quad) hipLaunchKernelGGL((conv_lds_kernel<T, 2, true>), dim3(grid), dim3(256), 0, s, a);
    else if (max_cb == 2) hipLaunchKernelGGL((conv_lds_kernel<T, 2, false>), dim3(grid), dim3(256), 0, s, a);
    else if (quad) hipLaunchKernelGGL((conv_lds_kernel<T, 4, true>), dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((conv_lds_kernel<T, 4, false>), dim3(grid), dim3(256), 0, s, a);
}

hipError_t launch_conv(const GemmArgs& a, uint32_t dtype, uint32_t max_cb, bool quad, uint32_t grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 7) / 8 * 8;
    if (dtype == MT_BF16) launch_conv_t<__bf16>(a, max_cb, quad, grid, s);
    else launch_conv_t<float>(a, max_cb, quad, grid, s);
    return hipGetLastError();
}
hipError_t launch_gap(const GapArgs& a, hipStream_t s)
{
    // grid covers every packed row; rows of other layer kinds return at once
    hipLaunchKernelGGL(gap_kernel, dim3(a.P), dim3(kGapThreads), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_head(const HeadArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(head_kernel, dim3((a.R + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace mt
