// Grouped FC layer, weight-streaming tiles (see mt_device.h for the overview).
#include "mt_device.h"

namespace mt {

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
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nKB = L.K / KB;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    const uint32_t nb_eff = active ? nb : 0;                 // idle waves still help staging; they stream block 0 and drop it
    const u32x4* wp = (const u32x4*)(a.arena + L.w_off) + (size_t)nb_eff * nKB * 64 + lane;
    const u32x4* xbase = (const u32x4*)((const T*)act_of(a.act, L.in_buf) + (size_t)seg0 * a.S) + lane;

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
    const u32x4* xbase = (const u32x4*)((const T*)act_of(a.act, L.in_buf) + (size_t)seg0 * a.S) + lane;
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
__device__ __forceinline__ void fc_tile(const GemmArgs& a, const Tile& tl, const LayerDev& L, uint32_t Mt, uint32_t seg0, uint8_t* smem)
{
    const uint32_t split = tl.split;
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t li = lane & 31, lh = lane >> 5;
    const uint32_t ks = 4 / split;
    const uint32_t nb = tl.n0 / kBrickRows + (wave % split), kq = wave / split;
    const bool active = nb < L.N_pad / kBrickRows;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
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
    if (L.is_last && a.fuse_head && L.N <= kBrickRows) {
        // at most 32 classes (one column block, so split == 1): the writer wave holds whole rows of logits.  Transpose them
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
    if (L.is_last && a.fuse_head && L.N <= a.fuse_head_max && L.N_pad <= split * kBrickRows) {
        // 33 .. 128 classes, all of them inside this tile (one column group): the waves put their
        // 32x32 blocks of logits side by side in LDS as [row][class], then eight threads share a
        // row: softmax, argmax (lowest index on ties) and the outputs in submission order.
        constexpr uint32_t LRS = kTileCols + 4;                 // floats per row of the logits tile (16-byte aligned rows)
        static_assert(kBrickRows * LRS * 4 <= kFcLdsBytes, "the logits tile of one row block must fit the kernel's LDS");
        float* lt = (float*)smem;
        const uint32_t C = L.N, tid = threadIdx.x, row = tid >> 3, part = tid & 7;
        const bool vec = a.out_vec_ok;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            __syncthreads();
            if (writer && (uint32_t)r < nrb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) lt[(8 * (v >> 2) + 4 * lh + (v & 3)) * LRS + n] = acc[r][v] + bv;
            }
            __syncthreads();
            const uint32_t m = tl.m0 + r * kBrickRows + row;
            if ((uint32_t)r < nrb && m < Mt) {                   // the eight threads of a row are neighbours in one wave
                f32x4 z[4];
                float mx = -INFINITY; int32_t best = 0x7fffffff;
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    z[q] = *(const f32x4*)(lt + row * LRS + part * 16 + q * 4);
#pragma unroll
                    for (uint32_t i = 0; i < 4; ++i) {
                        const uint32_t c = part * 16 + q * 4 + i;
                        if (c >= C) z[q][i] = -INFINITY;       // also hides what idle waves did not write
                        if (z[q][i] > mx) { mx = z[q][i]; best = (int32_t)c; }      // increasing index: the first hit is the lowest
                    }
                }
#pragma unroll
                for (int d = 4; d >= 1; d >>= 1) {
                    const float omx = __shfl_xor(mx, d);
                    const int32_t ob = __shfl_xor(best, d);
                    if (omx > mx || (omx == mx && ob < best)) { mx = omx; best = ob; }
                }
                f32x4 e[4];
                float sum = 0.0f;
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q)
#pragma unroll
                    for (uint32_t i = 0; i < 4; ++i) { e[q][i] = __expf(z[q][i] - mx); sum += e[q][i]; }   // exp(-inf) = 0 past the last class
#pragma unroll
                for (int d = 4; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
                const float inv = 1.0f / sum;
                const uint32_t sub = (uint32_t)a.perm[seg0 + m];
                if (part == 0) {
                    a.out.labels[sub] = best;
                    if (a.out.n_classes) a.out.n_classes[sub] = (int32_t)C;
                }
                float* pr = a.out.probs ? a.out.probs + (size_t)sub * a.out.row_stride : nullptr;
                float* lg = a.out.logits ? a.out.logits + (size_t)sub * a.out.row_stride : nullptr;
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const uint32_t c0 = part * 16 + q * 4;
                    f32x4 pv, lv;
#pragma unroll
                    for (uint32_t i = 0; i < 4; ++i) { const bool in = c0 + i < C; pv[i] = in ? e[q][i] * inv : 0.0f; lv[i] = in ? z[q][i] : 0.0f; }
                    if (vec) {
                        if (c0 < a.out.row_stride) { if (pr) *(f32x4*)(pr + c0) = pv; if (lg) *(f32x4*)(lg + c0) = lv; }
                    } else {
#pragma unroll
                        for (uint32_t i = 0; i < 4; ++i)
                            if (c0 + i < a.out.row_stride) { if (pr) pr[c0 + i] = pv[i]; if (lg) lg[c0 + i] = lv[i]; }
                    }
                }
                for (uint32_t c = kTileCols + part; c < a.out.row_stride; c += 8) {      // wider output rows: zeros past the tile
                    if (pr) pr[c] = 0.0f;
                    if (lg) lg[c] = 0.0f;
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
    u32x4* obase = (u32x4*)((T*)act_of(a.act, L.out_buf) + (size_t)seg0 * a.S) + lane;
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
    __shared__ __attribute__((aligned(16))) uint8_t smem[kFcLdsBytes];
    __shared__ uint32_t owner_part[4];
    TileOwner<256> lookup;
    lookup.fetch(a.tile_base, a.T);
    const uint32_t n_tiles = a.tile_base[a.T];
    uint32_t idx;
    if (!logical_tile(n_tiles, &idx)) return;
    Tile tl;
    tl.tenant = lookup.owner(a.T, idx, owner_part);           // uniform: the tenant's facts come through scalar loads
    // everything the tile needs to know about its tenant, fetched in one go
    const LayerDev L = a.layers[tl.tenant * MT_MAX_LAYERS + a.layer];
    const uint32_t Mt = a.M[tl.tenant], seg0 = a.off[tl.tenant];
    const uint32_t local = idx - a.tile_base[tl.tenant];
    asm volatile("" :: "s"(seg0), "s"(local));                // keeps those loads here, next to the others, instead of at their first use
    // where big tiles serve this tenant-layer, only the rows they leave are tiled here (in the shape that
    // big_remainder_split_k says: the batcher counted the tiles by the same rule)
    const bool big = ((*a.big_layers >> a.layer) & 1) && fc_is_big(Mt, L.N_pad);
    uint32_t groups, trows;
    fc_shape(L.N_pad, a.fc_split_k || (big && big_remainder_split_k(L.N_pad)), &tl.split, &groups, &trows);
    const uint32_t first = big ? big_rows(Mt) : 0;
    const uint32_t mt_ = ceil_div(Mt - first, trows);
    tl.m0 = first + (local % mt_) * trows;
    tl.rows = min(trows, Mt - tl.m0);
    tl.n0 = (local / mt_) * tl.split * kBrickRows;
    const uint32_t nrb = (tl.rows + kBrickRows - 1) / kBrickRows;
    if (a.gather) {
        if (nrb <= 1) fc_tile<T, 1, 8, true>(a, tl, L, Mt, seg0, smem);
        else fc_tile<T, 2, 4, true>(a, tl, L, Mt, seg0, smem);
    } else {
        if (nrb <= 1) fc_tile<T, 1, 8, false>(a, tl, L, Mt, seg0, smem);
        else fc_tile<T, 2, 4, false>(a, tl, L, Mt, seg0, smem);
    }
}

// ---- launcher ------------------------------------------------------------
hipError_t launch_fc(const GemmArgs& a, uint32_t dtype, uint32_t grid, hipStream_t s)
{
    if (grid == 0) return hipSuccess;
    grid = (grid + 7) / 8 * 8;
    if (dtype == MT_BF16) hipLaunchKernelGGL(fc_kernel<__bf16>, dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(fc_kernel<float>, dim3(grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace mt
