// On-demand reference mode (paper: Sec. "Problem and Baseline Implementation",
// the memory-efficient alternative that evaluates Eq. 1 directly for each source
// pixel and stores nothing).  fp32 throughout, vector ALU only.
//
// One wave per query.  The query's feature vector stays in registers (lanes
// split the channels); for each level the (2r+2)^2 integer-grid dot products
// are reduced across the wave into LDS, then lanes turn them into the
// (2r+1)^2 bilinear taps.
#include "corr_internal.h"

namespace {

struct OdArgs {
    const float* f1;                 // [B][HW][D]
    const float* f2[CORR_MAX_L];     // [B][HlWl][D]
    const float* coords;
    float* out;
    int B, HW, D, L, r;
    int tap_stride, pix_stride;      // layout of out
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    float scale;
};

constexpr int MAXD4 = 4;    // D <= 1024: up to 4 float4 per lane
constexpr int MAXG = 10;    // 2r+2 <= 10

__global__ __launch_bounds__(256) void ondemand_kernel(OdArgs a) {
    __shared__ float s_all[4][MAXG * MAXG];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = blockIdx.x * 4 + wave;
    if (q >= a.B * a.HW) return;                 // whole wave leaves together
    float* S = s_all[wave];
    const int b = q / a.HW, pix = q - b * a.HW;
    const int D4 = a.D >> 2;
    float4 f1v[MAXD4];
    const float4* f1p = reinterpret_cast<const float4*>(a.f1 + ((size_t)b * a.HW + pix) * a.D);
#pragma unroll
    for (int k = 0; k < MAXD4; ++k) {
        const int c4 = lane + 64 * k;
        f1v[k] = c4 < D4 ? f1p[c4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const float cx0 = a.coords[((size_t)b * 2 + 0) * a.HW + pix];
    const float cy0 = a.coords[((size_t)b * 2 + 1) * a.HW + pix];
    const bool finite_ok = (fabsf(cx0) <= CORR_COORD_LIMIT) && (fabsf(cy0) <= CORR_COORD_LIMIT);
    const int K = 2 * a.r + 1, Gs = K + 1, KK = K * K;
    for (int l = 0; l < a.L; ++l) {
        float* o = a.out + (size_t)b * a.L * KK * a.HW + (size_t)(l * KK) * a.tap_stride + (size_t)pix * a.pix_stride;
        const float inv = __uint_as_float((uint32_t)(127 - l) << 23);
        float fx = 0.f, fy = 0.f;
        int ox = 0, oy = 0;
        bool live = finite_ok;
        if (live) {
            const float cx = cx0 * inv, cy = cy0 * inv;
            const float flx = floorf(cx), fly = floorf(cy);
            fx = cx - flx; fy = cy - fly;
            ox = (int)flx - a.r; oy = (int)fly - a.r;
            live = (ox + K >= 0) && (ox <= a.Wl[l] - 1) && (oy + K >= 0) && (oy <= a.Hl[l] - 1);
        }
        if (!live) {
            for (int t = lane; t < KK; t += 64) o[(size_t)t * a.tap_stride] = 0.f;
            continue;
        }
        const float* f2b = a.f2[l] + (size_t)b * a.Hl[l] * a.Wl[l] * a.D;
        for (int pt = 0; pt < Gs * Gs; ++pt) {
            const int wy = pt / Gs, wx = pt - wy * Gs;
            const int y = oy + wy, x = ox + wx;
            float sum = 0.f;
            if (y >= 0 && y < a.Hl[l] && x >= 0 && x < a.Wl[l]) {
                const float4* f2p = reinterpret_cast<const float4*>(f2b + ((size_t)y * a.Wl[l] + x) * a.D);
#pragma unroll
                for (int k = 0; k < MAXD4; ++k) {
                    const int c4 = lane + 64 * k;
                    if (c4 < D4) {
                        const float4 v = f2p[c4];
                        sum += f1v[k].x * v.x + f1v[k].y * v.y + f1v[k].z * v.z + f1v[k].w * v.w;
                    }
                }
#pragma unroll
                for (int m = 32; m > 0; m >>= 1) sum += __shfl_xor(sum, m, 64);
            }
            if (lane == 0) S[pt] = sum * a.scale;
        }
        // lane 0's LDS writes must be visible to the other lanes of this wave
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const float w00 = (1.f - fx) * (1.f - fy), w01 = fx * (1.f - fy);
        const float w10 = (1.f - fx) * fy, w11 = fx * fy;
        for (int t = lane; t < KK; t += 64) {
            const int i = t / K, j = t - i * K;   // i: x offset, j: y offset
            const float* s = S + j * Gs + i;
            o[(size_t)t * a.tap_stride] = w00 * s[0] + w01 * s[1] + w10 * s[Gs] + w11 * s[Gs + 1];
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace

hipError_t launch_ondemand(const corr_pyramid* p, const LookupArgs& q, hipStream_t s) {
    OdArgs a;
    a.f1 = p->f1_nhwc; a.coords = q.coords; a.out = q.out;
    a.B = p->B; a.HW = p->H * p->W; a.D = p->D; a.L = p->L; a.r = q.r;
    a.tap_stride = corr_tap_stride(p, q); a.pix_stride = corr_pix_stride(p, q);
    for (int l = 0; l < CORR_MAX_L; ++l) {
        a.f2[l] = l < p->L ? p->f2_nhwc[l] : nullptr;
        a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l];
    }
    a.scale = 1.0f / sqrtf((float)p->D);
    const int BN = p->B * p->H * p->W;
    hipLaunchKernelGGL(ondemand_kernel, dim3((BN + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}
