// Full-volume reference mode (paper: Eq. 2 and the paragraph after it, the
// "default implementation"): the dense volume C = F1 . F2^T / sqrt(D) for all
// pixel pairs, a pyramid made by 2x2 average pooling of the volume's last two
// dimensions, then bilinear sampling of the pooled volumes with zero padding.
// fp32, vector ALU.  Memory is quadratic in pixels; the caller checks the size.
#include "corr_internal.h"

namespace {

constexpr size_t MAX_BLOCKS = 1u << 22;     // of 256 threads: 2^30 threads per launch, the kernels stride over the rest

// C[p][q] = scale * sum_d A[p][d] * B[q][d]; 64x64 tile per workgroup, 4x4 per thread.
__global__ __launch_bounds__(256) void vol_gemm_kernel(const float* __restrict__ A, const float* __restrict__ Bm,
                                                       float* __restrict__ C, int N, int D, float scale) {
    __shared__ float sa[16][65], sb[16][65];
    const int b = blockIdx.z;
    A += (size_t)b * N * D; Bm += (size_t)b * N * D; C += (size_t)b * N * N;
    const int p0 = blockIdx.y * 64, q0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < D; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int row = i >> 4, kk = i & 15;
            sa[kk][row] = (p0 + row < N) ? A[(size_t)(p0 + row) * D + k0 + kk] : 0.f;
            sb[kk][row] = (q0 + row < N) ? Bm[(size_t)(q0 + row) * D + k0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = sa[kk][ty * 4 + i]; bv[i] = sb[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            const int p = p0 + ty * 4 + i, q = q0 + tx * 4 + j;
            if (p < N && q < N) C[(size_t)p * N + q] = acc[i][j] * scale;
        }
}

// dst[bp][v][u] = 0.25 * (src[bp][2v][2u] + src[bp][2v][2u+1] + src[bp][2v+1][2u] + src[bp][2v+1][2u+1])
__global__ __launch_bounds__(256) void vol_pool_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                       size_t rows, int Hs, int Ws, int Hd, int Wd) {
    // grid-stride: a launch holds fewer than 2^32 threads, a pooled volume can hold more elements than that
    const size_t per = (size_t)Hd * Wd, total = rows * per, step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const size_t bp = i / per;
        const int vu = (int)(i - bp * per), v = vu / Wd, u = vu - v * Wd;
        const float* s = src + bp * (size_t)Hs * Ws + (size_t)(2 * v) * Ws + 2 * u;
        dst[i] = 0.25f * (((s[0] + s[1]) + s[Ws]) + s[Ws + 1]);
    }
}

struct FvArgs {
    const float* vol[CORR_MAX_L];
    const float* coords;
    float* out;
    int B, HW, L, r;
    int tap_stride, pix_stride;      // layout of out
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
};

__device__ __forceinline__ float vol_at(const float* v, int H, int W, int y, int x) {
    return (y >= 0 && y < H && x >= 0 && x < W) ? v[(size_t)y * W + x] : 0.f;
}

__global__ __launch_bounds__(256) void vol_sample_kernel(FvArgs a) {
    const int K = 2 * a.r + 1, KK = K * K;
    const size_t total = (size_t)a.B * a.L * KK * a.HW, step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
    const int pix = (int)(i % a.HW);
    size_t rest = i / a.HW;
    const int t = (int)(rest % KK); rest /= KK;
    const int l = (int)(rest % a.L);
    const int b = (int)(rest / a.L);
    const float cx0 = a.coords[((size_t)b * 2 + 0) * a.HW + pix];
    const float cy0 = a.coords[((size_t)b * 2 + 1) * a.HW + pix];
    float v = 0.f;
    if (fabsf(cx0) <= CORR_COORD_LIMIT && fabsf(cy0) <= CORR_COORD_LIMIT) {
        const float inv = __uint_as_float((uint32_t)(127 - l) << 23);
        const float cx = cx0 * inv, cy = cy0 * inv;
        const float flx = floorf(cx), fly = floorf(cy);
        const float fx = cx - flx, fy = cy - fly;
        const int ti = t / K, tj = t - ti * K;            // ti: x offset, tj: y offset
        const int x0 = (int)flx - a.r + ti, y0 = (int)fly - a.r + tj;
        const int H = a.Hl[l], W = a.Wl[l];
        const float* vp = a.vol[l] + ((size_t)b * a.HW + pix) * (size_t)H * W;
        v = (1.f - fx) * (1.f - fy) * vol_at(vp, H, W, y0, x0) + fx * (1.f - fy) * vol_at(vp, H, W, y0, x0 + 1)
          + (1.f - fx) * fy * vol_at(vp, H, W, y0 + 1, x0) + fx * fy * vol_at(vp, H, W, y0 + 1, x0 + 1);
    }
    a.out[(size_t)b * a.L * KK * a.HW + (size_t)(l * KK + t) * a.tap_stride + (size_t)pix * a.pix_stride] = v;
    }
}

}  // namespace

hipError_t launch_fullvol_build(const corr_pyramid* p, hipStream_t s) {
    const int N = p->H * p->W;
    dim3 grid((N + 63) / 64, (N + 63) / 64, p->B);
    hipLaunchKernelGGL(vol_gemm_kernel, grid, dim3(256), 0, s, p->f1_nhwc, p->f2_nhwc[0], p->vol[0], N, p->D,
                       1.0f / sqrtf((float)p->D));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int l = 1; l < p->L; ++l) {
        const size_t rows = (size_t)p->B * N;
        const size_t total = rows * p->Hl[l] * p->Wl[l];
        const size_t blocks = (total + 255) / 256;
        hipLaunchKernelGGL(vol_pool_kernel, dim3((unsigned)(blocks < MAX_BLOCKS ? blocks : MAX_BLOCKS)), dim3(256), 0, s,
                           p->vol[l - 1], p->vol[l], rows, p->Hl[l - 1], p->Wl[l - 1], p->Hl[l], p->Wl[l]);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_fullvol_sample(const corr_pyramid* p, const LookupArgs& q, hipStream_t s) {
    FvArgs a;
    for (int l = 0; l < CORR_MAX_L; ++l) {
        a.vol[l] = l < p->L ? p->vol[l] : nullptr;
        a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l];
    }
    a.coords = q.coords; a.out = q.out; a.B = p->B; a.HW = p->H * p->W; a.L = p->L; a.r = q.r;
    a.tap_stride = corr_tap_stride(p, q); a.pix_stride = corr_pix_stride(p, q);
    const int K = 2 * q.r + 1;
    const size_t total = (size_t)p->B * p->L * K * K * a.HW;
    const size_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(vol_sample_kernel, dim3((unsigned)(blocks < MAX_BLOCKS ? blocks : MAX_BLOCKS)), dim3(256), 0, s, a);
    return hipGetLastError();
}
