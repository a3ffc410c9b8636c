// Grouped FC layer, compute-bound 256x256 tiles (see mt_device.h for the overview).
#include "mt_device.h"

namespace mt {

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
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the wave index as a scalar: staging addresses and LDS offsets become scalar arithmetic
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

    // staging: the first half of the waves copies the 8 activation row blocks, the second half the
    // 8 weight column blocks, BPW blocks each (blocks past the tile or the layer repeat the last valid one)
    const uint8_t* lp[BPW];                                 // uniform: the lane's 16 bytes are added as a 32-bit offset
    const uint32_t lane_off = lane * 16;
    {
        const uint8_t* xbase = (const uint8_t*)((const T*)act_of(a.act, L.in_buf) + (size_t)seg0 * a.S);
        const uint8_t* wbase = a.arena + L.w_off;
#pragma unroll
        for (uint32_t i = 0; i < BPW; ++i) {
            if (wave < WV / 2) lp[i] = xbase + (size_t)(m0 / kBrickRows + min(wave * BPW + i, nrb - 1)) * nKB * kBrickBytes;
            else lp[i] = wbase + (size_t)(n0 / kBrickRows + min((wave - WV / 2) * BPW + i, ncb - 1)) * nKB * kBrickBytes;
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
    auto issue_one = [&](uint32_t slot, uint32_t s, uint32_t q) {   // load q (of LPS) of stage s into ring slot `slot`
        uint8_t* dst = stages + (slot % kBigNS) * kBigStageBytes + (wave * BPW) * kBigKS * kBrickBytes;
        const uint32_t i = q / kBigKS, kk = q % kBigKS;
        uint32_t lo = lane_off;
        asm("" : "+v"(lo));                                   // keeps base and lane offset apart: scalar base + 32-bit lane offset is one addressing mode
        __builtin_amdgcn_global_load_lds((gvoid_t)(lp[i] + (size_t)(s * kBigKS + kk) * kBrickBytes + lo),
                                         (lvoid_t)(dst + (i * kBigKS + kk) * kBrickBytes), 16, 0, 0);
    };
    auto issue_stage = [&](uint32_t slot, uint32_t s) {
#pragma unroll
        for (uint32_t q = 0; q < LPS; ++q) issue_one(slot, s, q);
    };
    // MFMA operands of one k step: 4 activation bricks and 2 weight bricks of this wave
    auto read_a = [&](const uint8_t* buf, uint32_t kk, u32x4 (&a4)[4], int i0, int i1) {
        const uint8_t* ab = buf + (wm * 4 * kBigKS) * kBrickBytes + lane * 16;
#pragma unroll
        for (int i = i0; i < i1; ++i) a4[i] = *(const u32x4*)(ab + (i * kBigKS + kk) * kBrickBytes);
    };
    auto read_b = [&](const uint8_t* buf, uint32_t kk, u32x4 (&b2)[CJ]) {
        const uint8_t* bb = buf + ((kBigBlocks + wn * CJ) * kBigKS) * kBrickBytes + lane * 16;
#pragma unroll
        for (int j = 0; j < (int)CJ; ++j) b2[j] = *(const u32x4*)(bb + (j * kBigKS + kk) * kBrickBytes);
    };
    auto read_ops = [&](const uint8_t* buf, uint32_t kk, u32x4 (&a4)[4], u32x4 (&b2)[CJ]) {
        read_a(buf, kk, a4, 0, 4);
        read_b(buf, kk, b2);
    };
    auto mma_rows = [&](const u32x4 (&a4)[4], const u32x4 (&b2)[CJ], int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < (int)CJ; ++j) Mma<T>::run(acc[i][j], b2[j], a4[i]);   // weights as the row operand: see the epilogue
    };
    auto mma_all = [&](const u32x4 (&a4)[4], const u32x4 (&b2)[CJ]) { mma_rows(a4, b2, 0, 4); };
    static_assert(kBigKS == 2, "the loop below is written for two k steps per stage");

    // The two k steps of a stage use two operand register sets, X and Y; the second k step of a
    // stage is multiplied after the next stage's barrier, so the MFMA pipe has work the moment the
    // barrier opens.  Between the barriers the 16 MFMAs of a wave are issued in pairs and the
    // stage's four global->LDS loads and twelve LDS reads are dealt out between the pairs, in the
    // shadow of an MFMA already in the pipe.  Issued as one burst behind the barrier (all eight
    // waves at once: 32 KiB, which the L2 -> LDS path takes ~250 ns to accept) the loads held every
    // wave at its load instructions while the pipes ran dry: 16 % more clocks per tile.
    static_assert(LPS == 4, "the schedule below deals out four loads per wave and stage");
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
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
            const uint8_t* buf = stages + (s % kBigNS) * kBigStageBytes;
            const uint32_t slot = s + kBigNS - 1, nxt = min(slot, last);   // past the end: a harmless repeat keeps the count uniform
            fence();
            mma_rows(ya, yb, 0, 1);                                   // second k step of stage s - 1: the pipe has work the moment the barrier opens
            fence();
            issue_one(slot, nxt, 0);
            fence();
            mma_rows(ya, yb, 1, 2);
            fence();
            read_a(buf, 0, xa, 0, 1); read_b(buf, 0, xb);             // first k step of stage s
            fence();
            mma_rows(ya, yb, 2, 3);
            fence();
            issue_one(slot, nxt, 1); read_a(buf, 0, xa, 1, 4);
            fence();
            mma_rows(ya, yb, 3, 4);
            fence();
            issue_one(slot, nxt, 2);
            fence();
            mma_rows(xa, xb, 0, 1);
            fence();
            read_a(buf, 1, ya, 0, 1); read_b(buf, 1, yb); issue_one(slot, nxt, 3);   // Y is free: its last MFMA has been issued
            fence();
            mma_rows(xa, xb, 1, 2);
            fence();
            read_a(buf, 1, ya, 1, 4);
            fence();
            mma_rows(xa, xb, 2, 4);
            fence();
        }
        mma_all(ya, yb);
    } else {
        for (uint32_t s = 1; s < n_stages; ++s) {
            ring_barrier(true);
            issue_stage(s + kBigNS - 1, min(s + kBigNS - 1, last));
        }
    }
    // the bias values of this wave's column blocks (the same for all its row blocks), fetched
    // here so that the wait below covers them: loading them block by block in the epilogue put
    // eight dependent L2 round trips on every tile's critical path
    const float* bias = (const float*)(a.arena + L.b_off);
    f32x4 bias_q[CJ][4];
#pragma unroll
    for (uint32_t j = 0; j < CJ; ++j) {
        const uint32_t nb = n0 / kBrickRows + min(wn * CJ + j, ncb - 1);          // blocks past the layer repeat the last one (unused)
#pragma unroll
        for (int g = 0; g < 4; ++g) bias_q[j][g] = *(const f32x4*)(bias + nb * kBrickRows + 4 * lh + 8 * g);   // bias is padded to N_pad
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
    const uint32_t nKB_out = L.out_fill / KB;
    auto block = [&](const f32x16& blk, uint32_t i, uint32_t j) {
        const uint32_t rb = wm * 4 + i;
        if (rb < nrb && wn * CJ + j < ncb) {
            const uint32_t nb = n0 / kBrickRows + wn * CJ + j, nl = nb * kBrickRows + 4 * lh;   // first output of this lane's runs
            const uint32_t mb = m0 + rb * kBrickRows;          // first row of the block inside the tenant
            f32x4 y[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) y[g][e] = blk[4 * g + e] + bias_q[j][g][e];
            }
            if (L.is_last) {
                if (mb + li < Mt) {
                    float* row = a.logits + (size_t)(seg0 + mb + li) * a.C_pad;
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        if (nl + 8 * g < L.N) *(f32x4*)(row + nl + 8 * g) = y[g];                 // starts below N at a multiple of 4, so it ends inside the row's C_pad = round_up(classes, 4) floats
                }
            } else {
                u32x4* out = (u32x4*)((T*)act_of(a.act, L.out_buf) + (size_t)seg0 * a.S) +
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

// ---- the same tiles, one workgroup per CU walking several of them ------------------------------
// A tile of fc_big_kernel spends ~5 us outside its K loop and its epilogue: the copy of the tile list, the
// search for its tenant, the tenant's facts, the first stages' way from memory.  Here a workgroup takes
// tiles b, b + G, b + 2G, ... of the same order (G = the grid, one workgroup per CU), copies the list once
// and lets the ring run on: the three stages that the loop of a tile issues past its own end are the first
// three stages of the next tile, and the barrier that opens the next tile is passed before the epilogue of
// this one, so the epilogue's stores and the next tile's loads are both in flight while the other proceeds.
// What a tile needs besides its operands comes through global->LDS loads too (the next tile's facts at the
// head of a tile, its bias values, from which its sums start, before the last three stages): the kernel issues no load into registers after its first
// tile, and "how many of my loads are outstanding" keeps meaning what the ring needs it to mean.  The
// epilogue's stores count as well, which only makes the waits stricter by the stores of the tile before.
// Tiles need at least seven stages (the host checks K): the facts are read after the barrier of stage 3.
struct BigTile {                                   // what a workgroup knows of one tile; all wave-uniform
    uint32_t Mt, seg0, m0, n0, nrb, ncb, n_stages, N, N_pad, act, is_last, out_fill, out_buf;
    uint64_t b_off;
    const uint8_t* xrow;                           // first activation row block of the tile
    const uint8_t* wcol;                           // first weight column block of the tile
    uint32_t blk_bytes;                            // bytes of one row / column block (all of K)
};

template <typename T>
__global__ __launch_bounds__(512) void fc_big_walk_kernel(GemmArgs a)
{
    constexpr uint32_t WV = 8, WN = 4, CJ = 2, BPW = 2, LPS = 4;
    static_assert(kBigKS == 2 && kBigNS == 4 && kBigBlocks == 8, "written for the 256x256 tile, two k steps per stage, four stages");
    // The ring, and behind it, in the same array (the compiler's wait counts stay exact only while all global->LDS
    // loads of a kernel go to one object): per wave 1 KiB for the bias values of the next tile and 256 bytes for
    // its facts, which every wave fetches for itself; then the copy of the tile list.
    constexpr uint32_t kRing = kBigNS * kBigStageBytes, kBiasBytes = WV * kBigTile * 4, kFactBytes = WV * 256;
    constexpr uint32_t kFactWords = sizeof(LayerDev) / 4;    // lanes 0..: the layer's row; then the tenant's row count and first row
    static_assert(sizeof(LayerDev) % 4 == 0 && kFactWords + 2 <= 64, "one dword per lane");
    __shared__ __attribute__((aligned(16))) uint8_t stages[kRing + kBiasBytes + kFactBytes + (kMaxTenantsPadded + 1) * 4];
    float* const bias_l = (float*)(stages + kRing);
    uint32_t* const fact_l = (uint32_t*)(stages + kRing + kBiasBytes);
    uint32_t* const base_l = (uint32_t*)(stages + kRing + kBiasBytes + kFactBytes);
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t li = lane & 31, lh = lane >> 5, wm = wave / WN, wn = wave % WN;
    const uint32_t lane_off = lane * 16;

    const uint32_t n_tiles = a.tile_base[a.T];
    for (uint32_t i = tid; i <= a.T; i += WV * 64) base_l[i] = a.tile_base[i];
    __syncthreads();
    auto logical = [&](uint32_t v) {                         // the order of logical_tile_chunked, for a block index of the one-tile-per-workgroup grid
        const uint32_t xcd = v & 7, i = v >> 3;
        return ((i / kXcdChunk) * 8 + xcd) * kXcdChunk + (i % kXcdChunk);
    };
    auto next_valid = [&](uint32_t v) { while (v < a.big_vgrid && logical(v) >= n_tiles) v += gridDim.x; return v; };
    // the tile with block index v of the one-tile-per-workgroup grid, given its tenant t, the tenant's row count and
    // first row, and the layer's row; everything is wave-uniform
    auto make_tile = [&](uint32_t v, uint32_t t, uint32_t Mt, uint32_t seg0, const LayerDev& L) {
        BigTile q;
        const uint32_t local = logical(v) - base_l[t];
        q.Mt = Mt; q.seg0 = seg0;
        const uint32_t nKB = L.K / KB;
        const uint32_t Mb = big_rows(q.Mt);
        const uint32_t mt_ = ceil_div(Mb, kBigTile), nt_ = ceil_div(L.N_pad, kBigTile);
        const uint32_t per_group = kBigGroup * nt_, grp = local / per_group, first_m = grp * kBigGroup;
        const uint32_t gsz = min(mt_ - first_m, kBigGroup), in_grp = local - grp * per_group;
        q.m0 = (first_m + in_grp % gsz) * kBigTile; q.n0 = (in_grp / gsz) * kBigTile;
        q.nrb = ceil_div(min((uint32_t)kBigTile, Mb - q.m0), kBrickRows);
        q.ncb = min(kBigBlocks, L.N_pad / kBrickRows - q.n0 / kBrickRows);
        q.n_stages = nKB / kBigKS; q.N = L.N; q.N_pad = L.N_pad; q.act = L.act; q.is_last = L.is_last; q.out_fill = L.out_fill; q.out_buf = L.out_buf;
        q.blk_bytes = nKB * kBrickBytes;
        const uint8_t* xrow = (const uint8_t*)((const T*)act_of(a.act, L.in_buf) + (size_t)q.seg0 * a.S) + (size_t)(q.m0 / kBrickRows) * q.blk_bytes;
        const uint8_t* wcol = a.arena + L.w_off + (size_t)(q.n0 / kBrickRows) * q.blk_bytes;
        // everything here is the same in every lane; saying so keeps the facts in scalar registers from tile to tile
        // (loaded values travel in vector registers otherwise, and so would every address derived from them)
        auto uni = [](uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane(x); };
        auto uni64 = [&](uint64_t x) { return (uint64_t)uni((uint32_t)x) | ((uint64_t)uni((uint32_t)(x >> 32)) << 32); };
        q.Mt = uni(q.Mt); q.seg0 = uni(q.seg0); q.m0 = uni(q.m0); q.n0 = uni(q.n0); q.nrb = uni(q.nrb); q.ncb = uni(q.ncb);
        q.n_stages = uni(q.n_stages); q.N = uni(q.N); q.N_pad = uni(q.N_pad); q.act = uni(q.act); q.is_last = uni(q.is_last);
        q.out_fill = uni(q.out_fill); q.out_buf = uni(q.out_buf); q.blk_bytes = uni(q.blk_bytes);
        q.b_off = uni64(L.b_off);
        q.xrow = (const uint8_t*)uni64((uint64_t)xrow); q.wcol = (const uint8_t*)uni64((uint64_t)wcol);
        return q;
    };
    auto tenant_of = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane(find_tenant(base_l, a.T, logical(v))); };
    // block i (of BPW) that this wave stages of a tile: the first half of the waves copies the 8 activation row
    // blocks, the second half the 8 weight column blocks (blocks past the tile or the layer repeat the last valid one)
    auto feed = [&](const BigTile& q, uint32_t i) -> const uint8_t* {
        return wave < WV / 2 ? q.xrow + (size_t)min(wave * BPW + i, q.nrb - 1) * q.blk_bytes
                             : q.wcol + (size_t)min((wave - WV / 2) * BPW + i, q.ncb - 1) * q.blk_bytes;
    };

    typedef const __attribute__((address_space(1))) void* gvoid_t;
    typedef __attribute__((address_space(3))) void* lvoid_t;
    auto load_brick = [&](const uint8_t* src, uint32_t ring_stage, uint32_t i, uint32_t kk) {      // brick (block i, k step kk) of a stage into the ring
        uint8_t* dst = stages + (ring_stage % kBigNS) * kBigStageBytes + ((wave * BPW + i) * kBigKS + kk) * kBrickBytes;
        uint32_t lo = lane_off;
        uint64_t base = (uint64_t)src;
        asm("" : "+v"(lo));                                   // scalar base + 32-bit lane offset is one addressing mode;
        asm("" : "+s"(base));                                 // kept apart, or the sums get regrouped into 64-bit vector additions
        __builtin_amdgcn_global_load_lds((gvoid_t)((const uint8_t*)base + lo), (lvoid_t)dst, 16, 0, 0);
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    constexpr uint32_t kOut = 2 * LPS;                       // loads of the two younger stages may stay in flight (one more, the bias load, only makes the wait stricter)
    constexpr int kWaitVm = (int)((kOut & 15) | ((kOut >> 4) << 14) | 0x0070 | 0x0F00), kWaitVmLgkm0 = kWaitVm & ~0x0F00;
    auto ring_barrier = [&](bool lds_too) {
        if (lds_too) __builtin_amdgcn_s_waitcnt(kWaitVmLgkm0); else __builtin_amdgcn_s_waitcnt(kWaitVm);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // a tile's 256 bias values into this wave's bias area, 16 bytes per lane (the last lanes of a narrow
    // last tile repeat its last four)
    auto issue_bias = [&](const BigTile& q) {
        uint32_t off = min(q.n0 + 4 * lane, q.N_pad - 4) * 4;
        uint64_t base = (uint64_t)(a.arena + q.b_off);
        asm("" : "+v"(off));
        asm("" : "+s"(base));
        __builtin_amdgcn_global_load_lds((gvoid_t)((const uint8_t*)base + off), (lvoid_t)(bias_l + wave * kBigTile), 16, 0, 0);
    };
    // the facts of the tile with block index vt, one dword per lane, into this wave's fact area
    auto issue_facts = [&](uint32_t vt) {
        const uint32_t t = tenant_of(vt);
        const uint32_t* row = (const uint32_t*)(a.layers + (size_t)t * MT_MAX_LAYERS + a.layer);
        const uint32_t* src = lane < kFactWords ? row + lane : lane == kFactWords ? a.M + t : lane == kFactWords + 1 ? a.off + t : row;
        __builtin_amdgcn_global_load_lds((gvoid_t)src, (lvoid_t)(fact_l + wave * 64), 4, 0, 0);
        return t;
    };
    auto read_facts = [&](uint32_t vt, uint32_t t) {
        const uint32_t w = fact_l[wave * 64 + lane];
        uint32_t words[kFactWords];
#pragma unroll
        for (uint32_t j = 0; j < kFactWords; ++j) words[j] = __builtin_amdgcn_readlane(w, j);
        const LayerDev L = __builtin_bit_cast(LayerDev, words);
        return make_tile(vt, t, __builtin_amdgcn_readlane(w, kFactWords), __builtin_amdgcn_readlane(w, kFactWords + 1), L);
    };

    uint32_t v = next_valid(blockIdx.x);
    if (v >= a.big_vgrid) return;
    BigTile cur;
    {
        const uint32_t t = tenant_of(v);
        cur = make_tile(v, t, a.M[t], a.off[t], a.layers[t * MT_MAX_LAYERS + a.layer]);
    }
    uint32_t g0 = 0;                                         // ring stage of the current tile's stage 0: the ring runs on from tile to tile
    {
        const uint8_t* f0 = feed(cur, 0); const uint8_t* f1 = feed(cur, 1);
        issue_bias(cur);                                     // first, so that it has landed when stage 0 has
#pragma unroll
        for (uint32_t s = 0; s < kBigNS; ++s) {              // the first tile's first four stages (tiles have more)
            if (s == kBigNS - 1) ring_barrier(false);        // the bias values and stage 0 are complete for every wave
#pragma unroll
            for (uint32_t q = 0; q < LPS; ++q) load_brick((q / kBigKS ? f1 : f0) + (size_t)(s * kBigKS + q % kBigKS) * kBrickBytes, s, q / kBigKS, q % kBigKS);
        }
    }
    // Per tile, from here: its bias values and its stage 0 are complete for every wave, its stages 1..3 are on their way.
    for (;;) {
        const uint32_t vn = next_valid(v + gridDim.x);
        const bool has_next = vn < a.big_vgrid;
        uint32_t tn = 0;
        if (has_next) tn = issue_facts(vn);                  // read once stage 3's barrier has passed: two stages' loads are younger by then
        const uint32_t n = cur.n_stages;
        const uint8_t* cf[BPW] = {feed(cur, 0), feed(cur, 1)};
        // what follows this tile's own stages: the next tile's first stages, or, behind the last tile, repeats of
        // its last stage, which keep the count of loads uniform
        BigTile nxt = cur;
        const uint8_t* nf[BPW] = {cf[0] + (size_t)(n - 1) * kBigKS * kBrickBytes, cf[1] + (size_t)(n - 1) * kBigKS * kBrickBytes};
        uint32_t nstep = 0;
        // load q (of LPS) of the stage three ahead of stage s of this tile; `own`: that stage is this tile's
        auto issue_ahead = [&](uint32_t s, uint32_t q, bool own) {
            const uint32_t sa = s + kBigNS - 1, i = q / kBigKS, kk = q % kBigKS;
            const uint8_t* src = own ? cf[i] + (size_t)sa * (kBigKS * kBrickBytes) : nf[i] + (size_t)(sa - n) * nstep;
            load_brick(src + kk * kBrickBytes, g0 + sa, i, kk);
        };
        // The sums start from the bias: a lane's sixteen values of a block are four runs of four output columns (see
        // the epilogue of fc_big_kernel), the same columns in each of the wave's four row blocks.
        f32x16 acc[4][CJ];
        {
            const float* bias_w = bias_l + wave * kBigTile;
#pragma unroll
            for (int j = 0; j < (int)CJ; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 bq = *(const f32x4*)(bias_w + (wn * CJ + j) * kBrickRows + 4 * lh + 8 * g);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = bq[e];
                }
        }
        auto read_a = [&](const uint8_t* buf, uint32_t kk, u32x4 (&a4)[4], int i0, int i1) {
            const uint8_t* ab = buf + (wm * 4 * kBigKS) * kBrickBytes + lane * 16;
#pragma unroll
            for (int i = i0; i < i1; ++i) a4[i] = *(const u32x4*)(ab + (i * kBigKS + kk) * kBrickBytes);
        };
        auto read_b = [&](const uint8_t* buf, uint32_t kk, u32x4 (&b2)[CJ]) {
            const uint8_t* bb = buf + ((kBigBlocks + wn * CJ) * kBigKS) * kBrickBytes + lane * 16;
#pragma unroll
            for (int j = 0; j < (int)CJ; ++j) b2[j] = *(const u32x4*)(bb + (j * kBigKS + kk) * kBrickBytes);
        };
        auto mma_rows = [&](const u32x4 (&a4)[4], const u32x4 (&b2)[CJ], int i0, int i1) {
#pragma unroll
            for (int i = i0; i < i1; ++i)
#pragma unroll
                for (int j = 0; j < (int)CJ; ++j) Mma<T>::run(acc[i][j], b2[j], a4[i]);
        };
        u32x4 xa[4], xb[CJ], ya[4], yb[CJ];
        auto step = [&](uint32_t s, bool own) {              // the schedule of fc_big_kernel
            ring_barrier(true);
            const uint8_t* buf = stages + ((g0 + s) % kBigNS) * kBigStageBytes;
            fence();
            mma_rows(ya, yb, 0, 1);
            fence();
            issue_ahead(s, 0, own);
            fence();
            mma_rows(ya, yb, 1, 2);
            fence();
            read_a(buf, 0, xa, 0, 1); read_b(buf, 0, xb);
            fence();
            mma_rows(ya, yb, 2, 3);
            fence();
            issue_ahead(s, 1, own); read_a(buf, 0, xa, 1, 4);
            fence();
            mma_rows(ya, yb, 3, 4);
            fence();
            issue_ahead(s, 2, own);
            fence();
            mma_rows(xa, xb, 0, 1);
            fence();
            read_a(buf, 1, ya, 0, 1); read_b(buf, 1, yb); issue_ahead(s, 3, own);
            fence();
            mma_rows(xa, xb, 1, 2);
            fence();
            read_a(buf, 1, ya, 1, 4);
            fence();
            mma_rows(xa, xb, 2, 4);
            fence();
        };
        auto idle_step = [&](uint32_t s, bool own) {         // a wave without rows only helps with staging and barriers
            ring_barrier(true);
#pragma unroll
            for (uint32_t q = 0; q < LPS; ++q) issue_ahead(s, q, own);
        };
        // Two loops, so that neither chooses its source per load: the stages three ahead are this tile's own up to
        // stage n - 4, the next tile's first three after that.  Between the loops the next tile's facts, which
        // landed long ago, turn into addresses.
        const bool rows = __builtin_amdgcn_readfirstlane(wm * 4 < cur.nrb);
        if (rows) {
            const uint8_t* b0 = stages + (g0 % kBigNS) * kBigStageBytes;
            read_a(b0, 0, xa, 0, 4); read_b(b0, 0, xb);
            read_a(b0, 1, ya, 0, 4); read_b(b0, 1, yb);
            fence();
            mma_rows(xa, xb, 0, 4);
            for (uint32_t s = 1; s + kBigNS - 1 < n; ++s) step(s, true);
        } else {
            for (uint32_t s = 1; s + kBigNS - 1 < n; ++s) idle_step(s, true);
        }
        if (has_next) {
            nxt = read_facts(vn, tn);
#pragma unroll
            for (uint32_t i = 0; i < BPW; ++i) nf[i] = feed(nxt, i);
            nstep = kBigKS * kBrickBytes;
            issue_bias(nxt);                                 // this tile took its own at its head; older than the twelve loads that follow, so it
                                                             // has landed when the barrier that opens the next tile is passed
        }
        if (rows) {
            for (uint32_t s = n - (kBigNS - 1); s < n; ++s) step(s, false);
            mma_rows(ya, yb, 0, 4);
        } else {
            for (uint32_t s = n - (kBigNS - 1); s < n; ++s) idle_step(s, false);
        }
        // The next tile starts before this one's epilogue: once every wave has the last stage in registers and the
        // next tile's stage 0 has landed, its stage 3 can go into the slot of the stage just read.  The epilogue's
        // stores then drain under the next tile's K loop instead of in front of a barrier.
        if (has_next) {
            ring_barrier(true);
#pragma unroll
            for (uint32_t q = 0; q < LPS; ++q) load_brick(feed(nxt, q / kBigKS) + (size_t)((kBigNS - 1) * kBigKS + q % kBigKS) * kBrickBytes, g0 + n + kBigNS - 1, q / kBigKS, q % kBigKS);
        }

        // epilogue (see fc_big_kernel; the bias is in the sums already): no LDS
        const uint32_t nKB_out = cur.out_fill / KB;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < (int)CJ; ++j) {
                const uint32_t rb = wm * 4 + i, cb = wn * CJ + j;
                if (rb < cur.nrb && cb < cur.ncb) {
                    const uint32_t nb = cur.n0 / kBrickRows + cb, nl = nb * kBrickRows + 4 * lh;
                    const uint32_t mb = cur.m0 + rb * kBrickRows;
                    f32x4 y[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g)
#pragma unroll
                        for (int e = 0; e < 4; ++e) y[g][e] = acc[i][j][4 * g + e];
                    if (cur.is_last) {
                        if (mb + li < cur.Mt) {
                            float* row = a.logits + (size_t)(cur.seg0 + mb + li) * a.C_pad;
#pragma unroll
                            for (int g = 0; g < 4; ++g)
                                if (nl + 8 * g < cur.N) *(f32x4*)(row + nl + 8 * g) = y[g];
                        }
                    } else {
                        u32x4* out = (u32x4*)((T*)act_of(a.act, cur.out_buf) + (size_t)cur.seg0 * a.S) +
                                     ((size_t)(mb / kBrickRows) * nKB_out + nb * (kBrickRows / KB)) * 64 + lane;
                        activate_block<4>(y, cur.act);
                        if constexpr (sizeof(T) == 4) {
#pragma unroll
                            for (int g = 0; g < 4; ++g) out[g * 64] = __builtin_bit_cast(u32x4, y[g]);
                        } else {
                            uint32_t pk[4][2];
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                T o[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) o[e] = (T)y[g][e];
                                const uint64_t qq = __builtin_bit_cast(uint64_t, o);
                                pk[g][0] = (uint32_t)qq; pk[g][1] = (uint32_t)(qq >> 32);
                            }
#pragma unroll
                            for (int h = 0; h < 2; ++h) {
                                const auto s0 = __builtin_amdgcn_permlane32_swap(pk[2 * h][0], pk[2 * h + 1][0], false, false);
                                const auto s1 = __builtin_amdgcn_permlane32_swap(pk[2 * h][1], pk[2 * h + 1][1], false, false);
                                out[h * 64] = u32x4{s0[0], s1[0], s0[1], s1[1]};
                            }
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        if (!has_next) break;
        g0 += n; cur = nxt; v = vn;
    }
    __builtin_amdgcn_s_waitcnt(0);                           // the repeats behind the last tile have landed before the workgroup gives its LDS back
}

// ---- launcher ------------------------------------------------------------
hipError_t launch_fc_big(const GemmArgs& a, uint32_t dtype, uint32_t grid, uint32_t walk_grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 8 * kXcdChunk - 1) / (8 * kXcdChunk) * (8 * kXcdChunk);
    // (the 4-wave shape, 128x128 per wave at one wave per SIMD, reads a third less from LDS per
    // MFMA but was measured 1.5x slower: a single wave per SIMD leaves the MFMA pipe idle at every wait)
    if (walk_grid) {                                         // one workgroup per CU walks the tiles of the same grid
        GemmArgs b = a;
        b.big_vgrid = grid;
        if (dtype == MT_BF16) hipLaunchKernelGGL((fc_big_walk_kernel<__bf16>), dim3(std::min(grid, walk_grid)), dim3(512), 0, s, b);
        else hipLaunchKernelGGL((fc_big_walk_kernel<float>), dim3(std::min(grid, walk_grid)), dim3(512), 0, s, b);
        return hipGetLastError();
    }
    if (dtype == MT_BF16) hipLaunchKernelGGL((fc_big_kernel<__bf16, 8>), dim3(grid), dim3(512), 0, s, a);
    else hipLaunchKernelGGL((fc_big_kernel<float, 8>), dim3(grid), dim3(512), 0, s, a);
    return hipGetLastError();
}

}  // namespace mt
