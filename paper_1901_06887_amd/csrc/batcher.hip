// Tenant segmentation and grouped-work descriptors (see mt_device.h for the overview).
#include "mt_device.h"

namespace mt {

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

constexpr uint32_t kLists = kListKinds * kLayerGroup;     // FC, conv and big-FC tile-count arrays of the layer indices of one pass

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
    __shared__ uint32_t big_total[kLayerGroup];
    __shared__ uint32_t carry_l[kLists];

    const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t T = a.T, R = a.R;
    if (tid < kLayerGroup) big_total[tid] = 0;         // first read is several barriers away
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
    // layer facts the host keeps per tenant and group of kLayerGroup layer indices.  The tile
    // lists are built one such group at a time (models deeper than a group: further passes at the
    // end of the kernel); the facts of the first group are fetched here, ahead of everything.
    uint32_t grp[NSLOT][kLayerGroup], rpr[NSLOT][kLayerGroup], npad[NSLOT][kLayerGroup];
    uint32_t regd[NSLOT];
    static_assert(kLayerGroup == 8 && MT_MAX_LAYERS % kLayerGroup == 0, "a group's layer facts are four 16-byte loads");
    auto load_facts = [&](uint32_t group) {
#pragma unroll
        for (uint32_t slot = 0; slot < nslots; ++slot) {
            const uint32_t t = tid + slot * kBatchThreads;
            const bool live = t < T;
            u32x4 q[4] = {};
            if (group == 0) regd[slot] = 0;
            if (live) {
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) q[i] = ((const u32x4*)a.facts)[(size_t)t * (MT_MAX_LAYERS / 2) + group * 4 + i];
                if (group == 0) regd[slot] = a.tenants[t].registered;
            }
            if (group == 0 && t < Tp) regl[t] = live && regd[slot];
#pragma unroll
            for (uint32_t l = 0; l < kLayerGroup; ++l) {
                const uint32_t w0 = regd[slot] ? q[l / 2][2 * (l % 2)] : 0, w1 = q[l / 2][2 * (l % 2) + 1];
                const bool conv = w0 >> 31;
                const bool sk = a.fc_split_k && !conv && w0;    // this run's FC tiles: one column block each, 32 rows
                grp[slot][l] = sk ? w1 / kBrickRows : w0 & 0x3fffffffu;
                rpr[slot][l] = conv ? (w1 | 0x80000000u) : sk ? 2u : 1u + ((w0 >> 30) & 1);
                npad[slot][l] = conv ? 0 : w1;
            }
        }
    };
    load_facts(0);

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
    for (uint32_t group = 0; group * kLayerGroup < a.n_layer_slots; ++group) {
        const uint32_t l0 = group * kLayerGroup, lmask = a.list_mask[group];
        if (group > 0) {                       // deeper models: the next eight layer indices (uniform: every thread takes the same passes)
            load_facts(group);
            if (tid < kLayerGroup) big_total[tid] = 0;
            __syncthreads();
        }
        uint32_t big_here = 0;
        if (a.big_enabled && l0 < (uint32_t)kBigMaxLayer) {
            uint32_t bt[kLayerGroup];
#pragma unroll
            for (uint32_t l = 0; l < kLayerGroup; ++l) bt[l] = 0;
#pragma unroll
            for (uint32_t slot = 0; slot < nslots; ++slot) {
                const uint32_t t = tid + slot * kBatchThreads;
                const uint32_t Mt = t < Tp ? Ml[t] : 0;
#pragma unroll
                for (uint32_t l = 0; l < kLayerGroup; ++l) {
                    const uint32_t rr = rpr[slot][l], np = npad[slot][l];
                    const uint32_t g = grp[slot][l];
                    if (g && !(rr >> 31) && fc_is_big(Mt, np)) bt[l] += ceil_div(big_rows(Mt), kBigTile) * ceil_div(np, kBigTile);
                }
            }
#pragma unroll
            for (uint32_t l = 0; l < kLayerGroup; ++l) {
                uint32_t v = bt[l];
                if (__any(v != 0)) {
                    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
                    if (lane == 0) atomicAdd(&big_total[l], v);
                }
            }
            __syncthreads();
#pragma unroll
            for (uint32_t l = 0; l < kLayerGroup; ++l) big_here |= (big_total[l] >= a.big_min_tiles ? 1u : 0u) << l;
            big_layers |= big_here << l0;
        }

        // pass 4: tile counts of every (kind, layer) list of the group, scanned over tenants in one
        // vector scan.  Only the exclusive in-wave prefix of each list stays in registers across the
        // barriers; the running total over slots lives in LDS.
        if (tid < kLists) carry_l[tid] = 0;
#pragma unroll
        for (uint32_t slot = 0; slot < nslots; ++slot) {
            const uint32_t t = tid + slot * kBatchThreads;
            const uint32_t Mt = t < Tp ? Ml[t] : 0;
            uint32_t excl[kLists];
            auto wave_scan = [&](uint32_t i, uint32_t c) {
                uint32_t v = c;
                if ((lmask >> i) & 1) v = wave_inclusive_scan(c);             // lists no registered model contributes to are skipped
                excl[i] = v - c;
                if (lane == 63) wtot[w][i] = v;
            };
#pragma unroll
            for (uint32_t l = 0; l < kLayerGroup; ++l) {
                const uint32_t g = grp[slot][l], rr = rpr[slot][l], np = npad[slot][l];
                const bool conv = rr >> 31;
                const bool big = !conv && ((big_here >> l) & 1) && fc_is_big(Mt, np);
                // conv: rows = requests * output pixels per tile; FC: rr = 1 (64-row tiles) or 2 (32-row tiles),
                // over the rows that big tiles leave
                const uint32_t Mb = big ? big_rows(Mt) : 0;
                static_assert(kTileRows == 64, "FC tiles have 64 >> (rr - 1) rows");
                const uint32_t fc_shift = 7 - rr;                           // log2 of the FC tile's rows (rr is 1 or 2 there)
                // (the few rows that big tiles leave in a narrow layer are tiled one column block and 32 rows at a time,
                // with K split among the waves: see big_remainder_split_k)
                const bool rem_sk = big && big_remainder_split_k(np);
                const uint32_t sh = rem_sk ? 5 : fc_shift, gq = rem_sk ? np / kBrickRows : g;
                const uint32_t tiles = (g && Mt) ? (conv ? ceil_div(Mt * (rr & 0x7fffffffu), kConvTileRows) * g
                                                         : ((Mt - Mb + (1u << sh) - 1) >> sh) * gq) : 0;
                wave_scan(l, conv ? 0 : tiles);
                wave_scan(kLayerGroup + l, conv ? tiles : 0);
                wave_scan(2 * kLayerGroup + l, ceil_div(Mb, kBigTile) * ceil_div(np, kBigTile));
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
                if (((lmask >> i) & 1) && t < T)
                    a.tile_base[((size_t)(i / kLayerGroup) * MT_MAX_LAYERS + l0 + i % kLayerGroup) * (T + 1) + t] = wtot[w][i] + excl[i];
            __syncthreads();
        }
        if (tid < kLists && ((lmask >> tid) & 1))
            a.tile_base[((size_t)(tid / kLayerGroup) * MT_MAX_LAYERS + l0 + tid % kLayerGroup) * (T + 1) + T] = carry_l[tid];
        __syncthreads();                               // carry_l and wtot are reused by the next group
    }
    if (tid == 0) *a.big_layers = big_layers;   // the FC kernels split a qualifying tenant's rows by it
}

// ---- launcher ------------------------------------------------------------
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

}  // namespace mt
