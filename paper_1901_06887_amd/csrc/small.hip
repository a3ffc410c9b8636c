// Gather, pooling, head and copy kernels (see mt_device.h for the overview).
#include "mt_device.h"

namespace mt {

// ---- gather ------------------------------------------------------------------------------
// Images (first layer is a convolution): gridDim.y workgroups per packed row, which deal the
// row's pixels out among themselves (a 224x224 image is 50176 pixels), one thread per pixel;
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
    if (sizeof(T) == 2 && ci == 3 && cp == 8 && npix % 2 == 0 && ((uintptr_t)src & 3) == 0) {
        // three-channel bf16 images, the usual case: two pixels are three aligned dwords; a thread
        // reads them, issues all its loads first, and writes two padded pixels of 16 bytes
        const uint32_t* s32 = (const uint32_t*)src;
        u32x4* d16 = (u32x4*)dst;
        constexpr uint32_t kPairs = 4;                       // pixel pairs in flight per thread
        for (uint32_t base = blockIdx.y * kPairs * blockDim.x; base < npix / 2; base += gridDim.y * kPairs * blockDim.x) {
            uint32_t w[kPairs][3];
#pragma unroll
            for (uint32_t i = 0; i < kPairs; ++i) {
                const uint32_t pp = min(base + i * blockDim.x + threadIdx.x, npix / 2 - 1);
#pragma unroll
                for (uint32_t j = 0; j < 3; ++j) w[i][j] = s32[(size_t)pp * 3 + j];
            }
#pragma unroll
            for (uint32_t i = 0; i < kPairs; ++i) {
                const uint32_t pp = base + i * blockDim.x + threadIdx.x;
                if (pp < npix / 2) {
                    d16[2 * pp] = u32x4{w[i][0], w[i][1] & 0xffffu, 0, 0};
                    d16[2 * pp + 1] = u32x4{(w[i][1] >> 16) | (w[i][2] << 16), w[i][2] >> 16, 0, 0};
                }
            }
        }
        for (uint32_t e = npix * cp + blockIdx.y * blockDim.x + threadIdx.x; e < td.in_fill; e += gridDim.y * blockDim.x) dst[e] = (T)0.0f;
        return;
    }
    for (uint32_t pix = blockIdx.y * blockDim.x + threadIdx.x; pix < npix; pix += gridDim.y * blockDim.x) {
        for (uint32_t g = 0; g < cp; g += EPC) {
            alignas(16) T tmp[EPC];
#pragma unroll
            for (uint32_t c = 0; c < EPC; ++c) tmp[c] = g + c < ci ? src[(size_t)pix * ci + g + c] : (T)0.0f;
            *(u32x4*)(dst + (size_t)pix * cp + g) = *(const u32x4*)tmp;
        }
    }
    for (uint32_t e = npix * cp + blockIdx.y * blockDim.x + threadIdx.x; e < td.in_fill; e += gridDim.y * blockDim.x) dst[e] = (T)0.0f;
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
        for (uint32_t kb0 = wave + 16 * blockIdx.y; kb0 < nKB; kb0 += 16 * gridDim.y) {
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
    for (uint32_t kb = wave + 4 * blockIdx.y; kb < nKB; kb += 4 * gridDim.y) {
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

// ---- global average pool: one workgroup per packed row, NHWC row in, brick slice out ------
constexpr uint32_t kGapThreads = 128;
template <typename T>
__device__ void gap_row(const GapArgs& a, const LayerDev& L, uint32_t p, uint32_t seg0)
{
    constexpr uint32_t EPC = 16 / sizeof(T), KB = 2 * EPC;
    const T* in = (const T*)act_of(a.act, L.in_buf) + (size_t)p * a.S;
    const uint32_t C = L.cin, HW = L.in_h * L.in_w;
    const uint32_t m = p - seg0, rb = m / kBrickRows, i = m % kBrickRows;
    const uint32_t nKB = L.out_fill / KB;
    T* out = (T*)act_of(a.act, L.out_buf) + (size_t)seg0 * a.S + (size_t)rb * nKB * 64 * EPC;
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

// ---- max-pool and residual add: gridDim.y workgroups per packed row, NHWC rows in and out ----
// 16 bytes per thread and step: a chunk of channels of one output pixel.  The window's taps
// outside the image are skipped, so they never win; an addition is followed by the layer's
// activation and the rounding to the element type.
constexpr uint32_t kImageOpThreads = 256;
template <typename T>
__device__ void maxpool_row(const GapArgs& a, const LayerDev& L, uint32_t p)
{
    constexpr uint32_t EPC = 16 / sizeof(T);
    const u32x4* in = (const u32x4*)((const T*)act_of(a.act, L.in_buf) + (size_t)p * a.S);
    u32x4* out = (u32x4*)((T*)act_of(a.act, L.out_buf) + (size_t)p * a.S);
    const uint32_t cpp = L.cin / EPC, n = L.rows_per_req * cpp;          // chunks per pixel (channels are a multiple of 8), chunks of the output
    for (uint32_t q = blockIdx.y * kImageOpThreads + threadIdx.x; q < n; q += gridDim.y * kImageOpThreads) {
        const uint32_t pix = q / cpp, ch = q - pix * cpp, oh = pix / L.out_w, ow = pix - oh * L.out_w;
        float best[EPC];
#pragma unroll
        for (uint32_t e = 0; e < EPC; ++e) best[e] = -INFINITY;
        for (uint32_t kh = 0; kh < L.ksize; ++kh) {
            const int32_t ih = (int32_t)(oh * L.stride + kh) - (int32_t)L.pad;
            if (ih < 0 || ih >= (int32_t)L.in_h) continue;
            for (uint32_t kw = 0; kw < L.ksize; ++kw) {
                const int32_t iw = (int32_t)(ow * L.stride + kw) - (int32_t)L.pad;
                if (iw < 0 || iw >= (int32_t)L.in_w) continue;
                const u32x4 v = in[((size_t)ih * L.in_w + iw) * cpp + ch];
                const T* ve = (const T*)&v;
#pragma unroll
                for (uint32_t e = 0; e < EPC; ++e) best[e] = fmaxf(best[e], (float)ve[e]);
            }
        }
        T o[EPC];
#pragma unroll
        for (uint32_t e = 0; e < EPC; ++e) o[e] = (T)best[e];             // a maximum of representable values: exact
        out[q] = __builtin_bit_cast(u32x4, o);
    }
    for (uint32_t q = n + blockIdx.y * kImageOpThreads + threadIdx.x; q < L.out_fill / EPC; q += gridDim.y * kImageOpThreads) out[q] = u32x4{0, 0, 0, 0};
}

template <typename T>
__device__ void add_row(const GapArgs& a, const LayerDev& L, uint32_t p)
{
    constexpr uint32_t EPC = 16 / sizeof(T);
    const u32x4* x = (const u32x4*)((const T*)act_of(a.act, L.in_buf) + (size_t)p * a.S);
    const u32x4* y = (const u32x4*)((const T*)act_of(a.act, L.in2_buf) + (size_t)p * a.S);
    u32x4* out = (u32x4*)((T*)act_of(a.act, L.out_buf) + (size_t)p * a.S);
    const uint32_t n = L.out_len / EPC;                                   // whole chunks: channels are a multiple of 8
    for (uint32_t q = blockIdx.y * kImageOpThreads + threadIdx.x; q < n; q += gridDim.y * kImageOpThreads) {
        const u32x4 xv = x[q], yv = y[q];
        const T* xe = (const T*)&xv;
        const T* ye = (const T*)&yv;
        T o[EPC];
#pragma unroll
        for (uint32_t e = 0; e < EPC; ++e) o[e] = (T)activate((float)xe[e] + (float)ye[e], L.act);
        out[q] = __builtin_bit_cast(u32x4, o);
    }
    for (uint32_t q = n + blockIdx.y * kImageOpThreads + threadIdx.x; q < L.out_fill / EPC; q += gridDim.y * kImageOpThreads) out[q] = u32x4{0, 0, 0, 0};
}

__global__ __launch_bounds__(kImageOpThreads) void image_ops_kernel(GapArgs a)
{
    const uint32_t p = blockIdx.x;
    if (p >= a.off[a.T]) return;
    const int32_t r = a.perm[p];
    if (r < 0) return;
    const uint32_t t = (uint32_t)a.row_tenant[r];
    if (a.tenants[t].n_layers <= a.layer) return;
    const LayerDev L = a.layers[t * MT_MAX_LAYERS + a.layer];
    if (L.kind == MT_MAXPOOL) {
        if (a.elem_size == 2) maxpool_row<__bf16>(a, L, p); else maxpool_row<float>(a, L, p);
    } else if (L.kind == MT_ADD) {
        if (a.elem_size == 2) add_row<__bf16>(a, L, p); else add_row<float>(a, L, p);
    }
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
            v[q] = c < a.C_pad ? *(const f32x4*)(z + c) : f32x4{0, 0, 0, 0};   // C_pad is a multiple of 4 and c too: a 16-byte read stays inside the row
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

// ---- matrix-instruction rate: what a loop of nothing but MFMAs sustains --------------------------
// Every wave keeps eight independent 32x32 accumulators going over pseudo-random bf16 operands
// (values of both signs and many exponents, like activations and weights: the clock the chip
// holds under matrix load depends on how much the operands toggle).  No memory traffic in the loop.
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* out, uint32_t iters)
{
    constexpr int NACC = 8;
    auto rnd = [](uint32_t x) {                    // integer hash -> roughly bell-shaped value in (-2, 2)
        x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
        return ((float)(x & 0xffff) + (float)(x >> 16)) * (1.0f / 32768.0f) - 2.0f;
    };
    bf16x8 a[NACC], b[NACC];
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 8; ++i) {
            a[j][i] = (__bf16)rnd((threadIdx.x * 8 + i) * 16 + j);
            b[j][i] = (__bf16)(rnd((threadIdx.x * 8 + i) * 16 + j + 0x9e3779b9u) * 0.015625f);
        }
    f32x16 acc[NACC];
    for (int j = 0; j < NACC; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < NACC; ++r)
#pragma unroll
            for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + r) % NACC], acc[j], 0, 0, 0);
    }
    float sum = 0.0f;
    for (int j = 0; j < NACC; ++j)
        for (int v = 0; v < 16; ++v) sum += acc[j][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

// `out` holds grid * 512 floats; flops of the launch = grid * 8 waves * iters * 64 MFMAs * 32768
hipError_t launch_mfma_rate(float* out, uint32_t iters, uint32_t grid, hipStream_t s)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(512), 0, s, out, iters);
    return hipGetLastError();
}

// ---- launchers ------------------------------------------------------------
hipError_t launch_gather(const GatherArgs& a, uint32_t slices, hipStream_t s)
{
    hipLaunchKernelGGL(gather_kernel, dim3(a.P / kBrickRows, slices), dim3(256), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_gather_image(const GatherArgs& a, uint32_t slices, hipStream_t s)
{
    hipLaunchKernelGGL(gather_image_kernel, dim3(a.P, slices), dim3(256), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_gap(const GapArgs& a, hipStream_t s)
{
    // grid covers every packed row; rows of other layer kinds return at once
    hipLaunchKernelGGL(gap_kernel, dim3(a.P), dim3(kGapThreads), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_image_ops(const GapArgs& a, uint32_t slices, hipStream_t s)
{
    hipLaunchKernelGGL(image_ops_kernel, dim3(a.P, slices), dim3(kImageOpThreads), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_head(const HeadArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(head_kernel, dim3((a.R + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace mt
