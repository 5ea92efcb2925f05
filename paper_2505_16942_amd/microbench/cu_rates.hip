// Microbenchmarks behind the block kernel's design figures, one workgroup of four waves per compute unit
// (the block kernel's shape).  Not part of the library.
//   hipcc --offload-arch=gfx950 -O3 -w -o cu_rates paper_2505_16942_amd/microbench/cu_rates.hip && ./cu_rates
//  1. LDS read bandwidth of ds_read_b128 with the kernel's fragment addressing (rows of 128 bytes, the
//     16-byte piece XOR-swizzled by the row), with and without the swizzle, and from one wave alone.
//  2. MFMA issue rate of v_mfma_f32_16x16x32_bf16 as a function of how many accumulators rotate, and with
//     two LDS fragment reads per six MFMAs (the chunk loop's mix).
//  3. Bandwidth of buffer_load_dwordx4 ... lds (loads that land in LDS without passing registers) when
//     every workgroup streams a private window of 16 KiB (stays in the vector L1), 64 KiB (32 workgroups
//     per XCD: stays in that XCD's 4 MiB L2) or 256 KiB (does not), on 64 and on 256 compute units.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

// ---- 1. LDS reads
template <int PAT, int WAVES>
__global__ __launch_bounds__(256, 1) void lds_kernel(unsigned* out, int iters) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 65536 / 4; i += 256) reinterpret_cast<unsigned*>(smem)[i] = i * 2654435761u;
    __syncthreads();
    const int r = lane & 15, p = lane >> 4;
    const unsigned off = PAT == 0 ? lane * 16 : PAT == 1 ? r * 128 + ((p ^ (r & 7)) * 16) : r * 128 + p * 16;
    u32x4 acc = {0, 0, 0, 0};
    if (wave < WAVES)
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int u = 0; u < 16; ++u)
                acc ^= *reinterpret_cast<const u32x4*>(smem + off + (unsigned)(u * 2048) + (unsigned)(it & 1) * 32768u);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) out[tid] = acc.x;
}
template <int PAT, int WAVES> int run_lds(unsigned* d, const char* name) {
    const int iters = 4000;
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    lds_kernel<PAT, WAVES><<<256, 256, 65536>>>(d, 10);
    CHECK(hipEventRecord(e0));
    lds_kernel<PAT, WAVES><<<256, 256, 65536>>>(d, iters);
    CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double bytes = (double)iters * 16 * 1024 * WAVES;
    printf("lds  %-26s %d wave(s): %6.1f B/ns per CU\n", name, WAVES, bytes / (ms * 1e6));
    return 0;
}

// ---- 2. MFMA rate
template <int R, int M, int NACC>
__global__ __launch_bounds__(256, 1) void mfma_kernel(float* out, long long* clk, int iters) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < 65536 / 4; i += 256) reinterpret_cast<unsigned*>(smem)[i] = 0x3c003c00u + (i & 7);
    __syncthreads();
    const int r = lane & 15, p = lane >> 4;
    const unsigned off = r * 128 + ((p ^ (r & 7)) * 16);
    f32x4 acc[NACC];
    for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0, 0, 0, 0};
    bf16x8 q[4];
    for (int i = 0; i < 4; ++i) q[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(smem + lane * 16 + i * 1024));
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            bf16x8 a[R > 0 ? R : 1];
#pragma unroll
            for (int x = 0; x < R; ++x)
                a[x] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(smem + off + (unsigned)((u * R + x) * 2048) % 32768u + (unsigned)(it & 1) * 32768u));
            if (R == 0) a[0] = q[u & 3];
#pragma unroll
            for (int m = 0; m < M; ++m)
                acc[(u * M + m) % NACC] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[R > 0 ? m % R : 0], q[m & 3], acc[(u * M + m) % NACC], 0, 0, 0);
        }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0;
    for (int i = 0; i < NACC; ++i) s += acc[i].x + acc[i].y + acc[i].z + acc[i].w;
    if (s == 12345.f) out[tid] = s;
    if (tid == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}
template <int R, int M, int NACC> int run_mfma(float* d, long long* clk, const char* name) {
    const int iters = 4000;
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    mfma_kernel<R, M, NACC><<<256, 256, 65536>>>(d, clk, 10);
    CHECK(hipEventRecord(e0));
    mfma_kernel<R, M, NACC><<<256, 256, 65536>>>(d, clk, iters);
    CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    long long h[2]; CHECK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
    printf("mfma %-12s %d reads + %2d MFMAs per step, %2d accumulators: %5.2f ns per MFMA per wave; shader clock %.2f GHz\n",
           name, R, M, NACC, ms * 1e6 / ((double)iters * 8 * M), (double)h[0] / h[1] / 10.0);
    return 0;
}

// ---- 3. loads into LDS
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned lds_base, int voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory");
}
template <unsigned WIN>
__global__ __launch_bounds__(256, 1) void dma_kernel(const unsigned char* src, unsigned region, unsigned* out, int iters) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem) + wave * 1024;
    const uint64_t base = (uint64_t)src;
    i32x4 rs;
    rs[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)base);
    rs[1] = __builtin_amdgcn_readfirstlane((int)((base >> 32) & 0xffff));
    rs[2] = __builtin_amdgcn_readfirstlane((int)region); rs[3] = 0x00020000;
    const unsigned wg_off = (blockIdx.x * WIN) % region;      // offsets stay below `region`: every load is in bounds
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
            dma16(rs, lds + (u & 7) * 4096, (int)((wg_off + (unsigned)(((it & 3) * 16 + u) * 4096u % WIN) + tid * 16u) % region));
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (reinterpret_cast<unsigned*>(smem)[tid] == 0x12345u) out[tid] = 1;
}
template <unsigned WIN> int run_dma(const unsigned char* src, unsigned region, unsigned* out, int grid) {
    const int iters = 2000;
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    dma_kernel<WIN><<<grid, 256, 65536>>>(src, region, out, 50);
    CHECK(hipEventRecord(e0));
    dma_kernel<WIN><<<grid, 256, 65536>>>(src, region, out, iters);
    CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double bytes = (double)iters * 16 * 4096;
    printf("load-to-LDS, %3u KiB per workgroup, %3d workgroups: %6.1f B/ns per CU, %5.2f TB/s in all\n", WIN >> 10, grid,
           bytes / (ms * 1e6), bytes * grid / (ms * 1e9));
    return 0;
}

int main() {
    unsigned* d; long long* clk; unsigned char* src;
    const unsigned region = 64u << 20;
    CHECK(hipMalloc(&d, 4096)); CHECK(hipMalloc(&clk, 64)); CHECK(hipMalloc(&src, region)); CHECK(hipMemset(src, 1, region));
    if (run_lds<0, 4>(d, "linear") || run_lds<0, 1>(d, "linear") || run_lds<1, 4>(d, "rows of 128 B, swizzled") ||
        run_lds<1, 1>(d, "rows of 128 B, swizzled") || run_lds<2, 4>(d, "rows of 128 B, plain")) return 1;
    float* f = reinterpret_cast<float*>(d);
    if (run_mfma<0, 6, 1>(f, clk, "MFMA only") || run_mfma<0, 6, 2>(f, clk, "MFMA only") || run_mfma<0, 6, 6>(f, clk, "MFMA only") ||
        run_mfma<0, 6, 12>(f, clk, "MFMA only") || run_mfma<2, 6, 2>(f, clk, "with reads") || run_mfma<2, 6, 12>(f, clk, "with reads")) return 1;
    for (int grid : {64, 256})
        if (run_dma<16384>(src, region, d, grid) || run_dma<65536>(src, region, d, grid) || run_dma<262144>(src, region, d, grid)) return 1;
    CHECK(hipDeviceSynchronize());
    printf("done\n");
    return 0;
}
