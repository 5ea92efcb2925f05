// Gradient of the lookup with respect to the two feature maps (the paper leaves the backward pass as future
// work, Sec. "Conclusion"; what it computes follows from Eq. 1).  Coordinates are constants.
//
// For one query p and level l the 81 tap gradients fold into a (K+1) x (K+1) footprint of weights
//     G[v][u] = sum over the up to four taps whose bilinear stencil touches footprint point (u, v) of
//               d_out[tap] * (corner weight),
// because all taps of a query share one fractional part.  Then
//     d f1(p)       += G[v][u] / sqrt(D) * f2_l(origin + (u, v))
//     d f2_l(q)     += G[v][u] / sqrt(D) * f1(p)          (q = origin + (u, v), inside the level)
// and the levels' gradients go down the pyramid by the adjoint of the 2x2 mean.
//
// This is the on-demand form: one wave per query, fp32 vector ALU, channels across lanes, hardware float
// atomics for d f2_l (its footprints overlap between queries).  fp32 channels-last representation of the
// pyramid (CORR_REP_F32), gradients accumulated channels-last in a caller-provided workspace and transposed
// to NCHW at the end.  Summation order of the atomics is not fixed: results agree to rounding, not bit for bit.
#include "corr_internal.h"

namespace {

constexpr int BQ = 4;                       // queries (waves) per workgroup
constexpr int MAXK = 2 * CORR_R + 1;
constexpr int MAX_NK = 1024 / 64;           // channel slots per lane at the largest D

struct BwdArgs {
    const float* f1;                        // [B*HW][D]
    const float* f2[CORR_MAX_L];            // [B*Hl*Wl][D]
    float* d_f1;                            // [B*HW][D], written
    float* d_f2[CORR_MAX_L];                // [B*Hl*Wl][D], zero on entry, accumulated
    const float* coords;                    // [B][2][HW]
    const float* d_out;                     // [B][L*K*K][HW]
    int B, HW, D, L, r;
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    float scale;
};

__global__ __launch_bounds__(64 * BQ) void bwd_query_kernel(BwdArgs a) {
    __shared__ float s_taps[BQ][MAXK * MAXK];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = 2 * a.r + 1, KK = K * K, NK = (a.D + 63) / 64;
    const long long q = (long long)blockIdx.x * BQ + wave;
    const bool real = q < (long long)a.B * a.HW;          // waves past the end stay for the barriers
    const int b = real ? (int)(q / a.HW) : 0, p = real ? (int)(q - (long long)b * a.HW) : 0;
    const float cx = a.coords[((size_t)b * 2 + 0) * a.HW + p], cy = a.coords[((size_t)b * 2 + 1) * a.HW + p];
    // comparisons are false for NaN: non-finite or huge coordinates give the constant 0, no gradient
    const bool live = real && fabsf(cx) <= CORR_COORD_LIMIT && fabsf(cy) <= CORR_COORD_LIMIT;
    float f1r[MAX_NK], acc[MAX_NK];
#pragma unroll
    for (int k = 0; k < MAX_NK; ++k) {
        const int ch = lane + 64 * k;
        f1r[k] = (k < NK && ch < a.D && real) ? a.f1[(size_t)q * a.D + ch] : 0.f;
        acc[k] = 0.f;
    }
    for (int l = 0; l < a.L; ++l) {
        __syncthreads();                                   // the previous level's taps are no longer read
        for (int t = lane; t < KK; t += 64)
            s_taps[wave][t] = live ? a.d_out[((size_t)b * a.L * KK + (size_t)l * KK + t) * a.HW + p] : 0.f;
        __syncthreads();
        if (!live) continue;                               // uniform per wave; the barriers above are outside
        const float inv = __uint_as_float((uint32_t)(127 - l) << 23);
        const float cxl = cx * inv, cyl = cy * inv;
        const float flx = floorf(cxl), fly = floorf(cyl);
        const float fx = cxl - flx, fy = cyl - fly;
        const int x0 = (int)flx - a.r, y0 = (int)fly - a.r;
        const int Hl = a.Hl[l], Wl = a.Wl[l];
        for (int pv = 0; pv <= K; ++pv) {
            const int v = y0 + pv;
            if (v < 0 || v >= Hl) continue;
            for (int pu = 0; pu <= K; ++pu) {
                const int u = x0 + pu;
                if (u < 0 || u >= Wl) continue;
                // taps (i, j) = (pu - du, pv - dv), du, dv in {0, 1}; tap channel = i*K + j, i the x offset
                float g = 0.f;
#pragma unroll
                for (int dv = 0; dv < 2; ++dv)
#pragma unroll
                    for (int du = 0; du < 2; ++du) {
                        const int i = pu - du, j = pv - dv;
                        if (i >= 0 && i < K && j >= 0 && j < K)
                            g += s_taps[wave][i * K + j] * (du ? fx : 1.f - fx) * (dv ? fy : 1.f - fy);
                    }
                g *= a.scale;
                const size_t row = ((size_t)b * Hl * Wl + (size_t)v * Wl + u) * a.D;
                const float* f2p = a.f2[l] + row;
                float* dp = a.d_f2[l] + row;
#pragma unroll
                for (int k = 0; k < MAX_NK; ++k) {
                    const int ch = lane + 64 * k;
                    if (k < NK && ch < a.D) {
                        acc[k] += g * f2p[ch];
                        unsafeAtomicAdd(dp + ch, g * f1r[k]);
                    }
                }
            }
        }
    }
    if (real) {
#pragma unroll
        for (int k = 0; k < MAX_NK; ++k) {
            const int ch = lane + 64 * k;
            if (k < NK && ch < a.D) a.d_f1[(size_t)q * a.D + ch] = acc[k];
        }
    }
}

// adjoint of the 2x2 mean: every pixel of the coarse level adds a quarter of its gradient to its four children
__global__ __launch_bounds__(256) void bwd_unpool_kernel(const float* __restrict__ coarse, float* __restrict__ fine,
                                                         size_t n, int D, int Hc, int Wc, int Hf, int Wf) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int ch = (int)(i % D);
        size_t pix = i / D;
        const int u = (int)(pix % Wc); pix /= Wc;
        const int v = (int)(pix % Hc);
        const size_t b = pix / Hc;
        const float t = 0.25f * coarse[i];
        float* f = fine + ((b * Hf + 2 * v) * (size_t)Wf + 2 * u) * D + ch;
        f[0] += t; f[D] += t; f[(size_t)Wf * D] += t; f[(size_t)Wf * D + D] += t;
    }
}

// [B][HW][D] -> [B][D][HW] through a 32 x 32 LDS tile
__global__ __launch_bounds__(256) void bwd_to_nchw_kernel(const float* __restrict__ src, float* __restrict__ dst, int HW, int D) {
    __shared__ float tile[32][33];
    const int b = blockIdx.z, p0 = blockIdx.x * 32, d0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8
    for (int r = ty; r < 32; r += 8)
        if (p0 + r < HW && d0 + tx < D) tile[r][tx] = src[((size_t)b * HW + p0 + r) * D + d0 + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8)
        if (d0 + r < D && p0 + tx < HW) dst[((size_t)b * D + d0 + r) * HW + p0 + tx] = tile[tx][r];
}

}  // namespace

size_t corr_backward_workspace_floats(int B, int H, int W, int D, int L) {
    size_t px = 0;
    for (int l = 0; l < L; ++l) px += (size_t)(H >> l) * (W >> l);
    return ((size_t)B * H * W + (size_t)B * px) * D;
}

hipError_t launch_backward(const corr_pyramid* p, const float* coords, const float* d_out, int r,
                           float* d_fmap1, float* d_fmap2, float* ws, hipStream_t s) {
    BwdArgs a;
    const int HW = p->H * p->W;
    a.f1 = p->f1_nhwc; a.coords = coords; a.d_out = d_out;
    a.B = p->B; a.HW = HW; a.D = p->D; a.L = p->L; a.r = r;
    a.scale = 1.0f / sqrtf((float)p->D);
    float* cur = ws;
    a.d_f1 = cur; cur += (size_t)p->B * HW * p->D;
    size_t lev_floats = 0;
    for (int l = 0; l < CORR_MAX_L; ++l) {
        a.f2[l] = l < p->L ? p->f2_nhwc[l] : nullptr;
        a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l];
        a.d_f2[l] = nullptr;
        if (l < p->L) {
            a.d_f2[l] = cur;
            const size_t n = (size_t)p->B * p->Hl[l] * p->Wl[l] * p->D;
            cur += n; lev_floats += n;
        }
    }
    // the level gradients accumulate: they start at zero (a fill kernel, so the call can be graph-captured)
    hipError_t e = launch_fill_i32(reinterpret_cast<int*>(a.d_f2[0]), 0, lev_floats, s);
    if (e != hipSuccess) return e;
    const long long BN = (long long)p->B * HW;
    hipLaunchKernelGGL(bwd_query_kernel, dim3((unsigned)((BN + BQ - 1) / BQ)), dim3(64 * BQ), 0, s, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    for (int l = p->L - 1; l >= 1; --l) {
        const size_t n = (size_t)p->B * p->Hl[l] * p->Wl[l] * p->D;
        const size_t blocks = (n + 255) / 256;
        hipLaunchKernelGGL(bwd_unpool_kernel, dim3((unsigned)(blocks < (1u << 20) ? blocks : (1u << 20))), dim3(256), 0, s,
                           a.d_f2[l], a.d_f2[l - 1], n, p->D, p->Hl[l], p->Wl[l], p->Hl[l - 1], p->Wl[l - 1]);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    dim3 tg((HW + 31) / 32, (p->D + 31) / 32, p->B);
    hipLaunchKernelGGL(bwd_to_nchw_kernel, tg, dim3(256), 0, s, a.d_f1, d_fmap1, HW, p->D);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_to_nchw_kernel, tg, dim3(256), 0, s, a.d_f2[0], d_fmap2, HW, p->D);
    return hipGetLastError();
}
