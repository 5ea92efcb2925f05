// Per-pair preprocessing (paper: "Input Preprocessing"; pooled target features
// per level, Sec. "Implementation Details"): one pass over a dense NCHW fp32
// map that emits every pyramid level in the layouts the lookup kernels read.
//
// A workgroup owns 32 channels x (8 rows x 32 columns) of level 0.  The tile is
// read once (128 B runs along x; 16-byte loads when the rows allow it), pooled 2x2 in LDS level after level
// (0.25f * (a + b + c + d), the order of the definition, in fp32) and written as
//   split : [D/32][P][32 x bf16 hi | 32 x bf16 lo] with P = every pixel of every level and batch
//           item (level-major, then batch, then row-major), so a 32-channel chunk of a window row
//           is one contiguous run and all levels share one chunk stride
//   hi    : [D/32][P][32 x bf16]: the hi parts alone, same pixel order (bf16 mode reads half the bytes)
//   nhwc  : [B][pixel][D] fp32
// A level-l pixel is written iff it lies inside the floor-halved level size, so
// a trailing odd row or column is dropped exactly as the definition says.
#include "corr_internal.h"

namespace {

constexpr int TILE_H = 8, TILE_W = 32, CH = CORR_CHUNK;

// LDS tile index of (channel c, row, col): rows padded by one float, and every group of 8 channels
// skewed by 16 floats so that the four 8-channel parts of one pixel fall in different banks
template <int ROWS, int COLS>
__device__ __forceinline__ int tix(int c, int row, int col) { return (c * ROWS + row) * (COLS + 1) + col + (c >> 3) * 16; }
template <int ROWS, int COLS>
constexpr int tile_floats() { return CH * ROWS * (COLS + 1) + (CH / 8 - 1) * 16; }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

struct LevelOut {
    uint16_t* split;   // may be null; base of the whole split buffer
    uint16_t* hi;      // may be null; base of the whole hi-only buffer
    size_t ptotal, pbase;   // pixels per chunk plane, first pixel of this level in a plane
    float* nhwc;       // may be null
    int H, W;
};
struct BuildArgs {
    const float* src;
    int B, D, H, W, nlev;
    int vec4;          // rows can be read with aligned 16-byte loads (W % 4 == 0 and a 16-byte aligned base)
    LevelOut lv[CORR_MAX_L];
};

// Write one level's part of the tile.  `t` holds [CH][rows][cols (+pad)] fp32.
template <int ROWS, int COLS>
__device__ __forceinline__ void emit_level(const float* t, const LevelOut& lo, int b, int kc, int D,
                                           int y0, int x0) {
    // one thread = one pixel x 8 channels (16 B of hi, 16 B of lo, 32 B of fp32)
    for (int w = threadIdx.x; w < ROWS * COLS * 4; w += blockDim.x) {
        const int part = w & 3, pix = w >> 2;
        const int row = pix / COLS, col = pix % COLS;
        const int y = y0 + row, x = x0 + col;
        if (y >= lo.H || x >= lo.W) continue;
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = t[tix<ROWS, COLS>(part * 8 + k, row, col)];
        const size_t p = (size_t)y * lo.W + x;
        const size_t npix = (size_t)lo.H * lo.W;
        if (lo.hi && !lo.split) {
            uint32_t hi[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) hi[k] = f32_to_bf16_rne(v[k]);
            uint16_t* dst = lo.hi + ((size_t)kc * lo.ptotal + lo.pbase + (size_t)b * npix + p) * CH + part * 8;
            *reinterpret_cast<uint4*>(dst) = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16),
                                                        hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
        }
        if (lo.split) {
            uint32_t hi[8], lw[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                hi[k] = f32_to_bf16_rne(v[k]);
                lw[k] = f32_to_bf16_rne(v[k] - bf16_bits_to_f32(hi[k]));
            }
            uint16_t* dst = lo.split + ((size_t)kc * lo.ptotal + lo.pbase + (size_t)b * npix + p) * (2 * CH) + part * 8;
            uint4 h4 = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16),
                                  hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
            uint4 l4 = make_uint4(lw[0] | (lw[1] << 16), lw[2] | (lw[3] << 16),
                                  lw[4] | (lw[5] << 16), lw[6] | (lw[7] << 16));
            *reinterpret_cast<uint4*>(dst) = h4;
            *reinterpret_cast<uint4*>(dst + CH) = l4;
            if (lo.hi)
                *reinterpret_cast<uint4*>(lo.hi + ((size_t)kc * lo.ptotal + lo.pbase + (size_t)b * npix + p) * CH + part * 8) = h4;
        }
        if (lo.nhwc) {
            float* dst = lo.nhwc + ((size_t)b * npix + p) * D + kc * CH + part * 8;
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
}

// dst[c][r][q] = 0.25f * (src[c][2r][2q] + src[c][2r][2q+1] + src[c][2r+1][2q] + src[c][2r+1][2q+1])
template <int ROWS, int COLS>   // ROWS, COLS of the destination
__device__ __forceinline__ void pool_level(const float* src, float* dst) {
    constexpr int SP = 2 * COLS + 1;
    for (int w = threadIdx.x; w < CH * ROWS * COLS; w += blockDim.x) {
        const int c = w / (ROWS * COLS), rq = w % (ROWS * COLS);
        const int r = rq / COLS, q = rq % COLS;
        const float* s = src + tix<2 * ROWS, 2 * COLS>(c, 2 * r, 2 * q);
        const float a = s[0], bb = s[1], cc = s[SP], dd = s[SP + 1];
        dst[tix<ROWS, COLS>(c, r, q)] = 0.25f * (((a + bb) + cc) + dd);
    }
}

__global__ __launch_bounds__(256) void build_features_kernel(BuildArgs a) {
    __shared__ float t0[tile_floats<TILE_H, TILE_W>()];
    __shared__ float t1[tile_floats<TILE_H / 2, TILE_W / 2>()];
    __shared__ float t2[tile_floats<TILE_H / 4, TILE_W / 4>()];
    __shared__ float t3[tile_floats<TILE_H / 8, TILE_W / 8>()];
    const int NC = a.D / CH;
    const int b = blockIdx.z / NC, kc = blockIdx.z % NC;
    const int y0 = blockIdx.y * TILE_H, x0 = blockIdx.x * TILE_W;
    if (a.vec4) {
        // 16-byte loads: a wave reads the 8 rows x 128 B of one channel, the four waves four channels
        const int col = (threadIdx.x & 7) * 4, row = (threadIdx.x >> 3) & 7, c0 = threadIdx.x >> 6;
        const int y = y0 + row, x = x0 + col;
        const bool ok = (y < a.H) && (x < a.W);              // a float4 is inside or outside as a whole
        const float* src = a.src + (((size_t)b * a.D + kc * CH + c0) * a.H + (ok ? y : 0)) * a.W + (ok ? x : 0);
        const size_t cstride = (size_t)a.H * a.W;
        float4 v[CH / 4];
#pragma unroll
        for (int i = 0; i < CH / 4; ++i)
            v[i] = ok ? *reinterpret_cast<const float4*>(src + (size_t)(4 * i) * cstride) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < CH / 4; ++i) {
            float* d = t0 + tix<TILE_H, TILE_W>(c0 + 4 * i, row, col);
            d[0] = v[i].x; d[1] = v[i].y; d[2] = v[i].z; d[3] = v[i].w;
        }
    } else {
        const int col = threadIdx.x % TILE_W, row = threadIdx.x / TILE_W;
        const int y = y0 + row, x = x0 + col;
        const bool ok = (y < a.H) && (x < a.W);
        const float* src = a.src + (((size_t)b * a.D + kc * CH) * a.H + (ok ? y : 0)) * a.W + (ok ? x : 0);
        const size_t cstride = (size_t)a.H * a.W;
#pragma unroll 8
        for (int c = 0; c < CH; ++c)
            t0[tix<TILE_H, TILE_W>(c, row, col)] = ok ? src[c * cstride] : 0.0f;
    }
    __syncthreads();
    emit_level<TILE_H, TILE_W>(t0, a.lv[0], b, kc, a.D, y0, x0);
    if (a.nlev > 1) {
        pool_level<TILE_H / 2, TILE_W / 2>(t0, t1);
        __syncthreads();
        emit_level<TILE_H / 2, TILE_W / 2>(t1, a.lv[1], b, kc, a.D, y0 / 2, x0 / 2);
    }
    if (a.nlev > 2) {
        pool_level<TILE_H / 4, TILE_W / 4>(t1, t2);
        __syncthreads();
        emit_level<TILE_H / 4, TILE_W / 4>(t2, a.lv[2], b, kc, a.D, y0 / 4, x0 / 4);
    }
    if (a.nlev > 3) {
        pool_level<TILE_H / 8, TILE_W / 8>(t2, t3);
        __syncthreads();
        emit_level<TILE_H / 8, TILE_W / 8>(t3, a.lv[3], b, kc, a.D, y0 / 8, x0 / 8);
    }
}

__global__ __launch_bounds__(256) void copy_f32_kernel(float4* __restrict__ dst, const float4* __restrict__ src, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

}  // namespace

hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t s) {
    // whole float4s only; the measurement buffers are multiples of 4 floats
    hipLaunchKernelGGL(copy_f32_kernel, dim3(256 * 16), dim3(256), 0, s, reinterpret_cast<float4*>(dst),
                       reinterpret_cast<const float4*>(src), n / 4);
    return hipGetLastError();
}

hipError_t launch_build_features(const float* nchw, int B, int D, int H, int W, int nlev,
                                 uint16_t* split, uint16_t* hi, float* const* nhwc, hipStream_t s) {
    BuildArgs a;
    a.src = nchw; a.B = B; a.D = D; a.H = H; a.W = W; a.nlev = nlev;
    a.vec4 = (W % 4 == 0) && (reinterpret_cast<uintptr_t>(nchw) % 16 == 0);
    size_t ptotal = 0;
    for (int l = 0; l < nlev; ++l) ptotal += (size_t)B * (H >> l) * (W >> l);
    size_t pbase = 0;
    for (int l = 0; l < CORR_MAX_L; ++l) {
        a.lv[l].split = l < nlev ? split : nullptr;
        a.lv[l].hi = l < nlev ? hi : nullptr;
        a.lv[l].ptotal = ptotal; a.lv[l].pbase = pbase;
        if (l < nlev) pbase += (size_t)B * (H >> l) * (W >> l);
        a.lv[l].nhwc = (l < nlev && nhwc) ? nhwc[l] : nullptr;
        a.lv[l].H = H >> l; a.lv[l].W = W >> l;
    }
    dim3 grid((W + TILE_W - 1) / TILE_W, (H + TILE_H - 1) / TILE_H, B * (D / CH));
    hipLaunchKernelGGL(build_features_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}
