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
// Both forms below read the fp32 channels-last representation of the pyramid (CORR_REP_F32), accumulate the
// gradients channels-last in a caller-provided workspace and bring them to NCHW at the end.  Summation order of
// the atomics on d f2_l is not fixed: d_fmap2 agrees between calls to rounding, not bit for bit.
//
// The first form is the plain one: one wave per query, fp32 vector ALU, channels across lanes, a hardware float
// atomic per (footprint point, channel) for d f2_l.  The second, further down, is what the entry point runs.
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

// ---------------------------------------------------------------------------------------------------------
// The item form: the same work items as the forward block kernel (a target cell and up to 128 of its queries,
// one fixed window of level-l points per level), and both gradients as dense contractions on the matrix cores.
// For one item and level, with G[point][query] the footprint weights of every query scattered over the window
// (zero outside the query's footprint) and 1/sqrt(D) folded in:
//     d f1[query][:]       += sum over points  G[point][query] * f2_l[point][:]       (M = queries, K = points)
//     d f2_l[point][:]     += sum over queries G[point][query] * f1[query][:]         (M = points,  K = queries)
// fp32 throughout: v_mfma_f32_16x16x4_f32 takes one fp32 element of A and of B per lane, so G (in LDS, one
// column per query) and the channels-last fp32 feature rows feed it without any transposition.  G is built
// CH points at a time from the tap gradients (a footprint point collects up to four taps); d f1 stays in
// accumulators over all levels and is stored once (a query belongs to one item); the window's d f2_l rows go
// out through float atomics once per item and pass, instead of once per query and footprint point.
// Eight waves, two per SIMD: a wave owns 32 channels of a 256-channel group (16 of a 128-channel group for
// D <= 128); lane = (K index lane/16, M or N index lane%16).  Feature rows come through buffer resources: an offset past the end reads zero and an atomic
// there is dropped, so rows outside the level and empty query slots need no branch inside the loops.
constexpr int NTI = 512;
constexpr int GST = CORR_GROUP + 4;         // floats between G rows (bank shift 4 per row: a 16-row x 4-query read is conflict-free)
constexpr int CH = 144;                     // window points per pass: level 2's window in one pass, level 0's in three
constexpr int MTC = CH / 16;
constexpr int TAB_PAD = 16;                 // the operand loads run three k-steps ahead: the tables end in invalid entries
constexpr int MAXKK = MAXK * MAXK;
constexpr int ITEM_LDS = CH * GST * 4 + (CH + TAB_PAD) * 4 + (CORR_GROUP + TAB_PAD) * 4 + CORR_GROUP * 8 + MAXKK * CORR_GROUP * 4;
constexpr unsigned BAD_OFF = 0x80000000u;   // beyond every buffer here (each is below 2 GiB)

struct BwdItemArgs {
    const float* f1;
    const float* f2[CORR_MAX_L];
    float* d_f1;                            // zero on entry (queries without an item keep the zero)
    float* d_f2[CORR_MAX_L];                // zero on entry, accumulated
    const float* d_out;
    const int* perm;
    const float2* sorted_c;
    const int4* items;
    const int* n_items;
    int* queue;                             // [8] next queue position per XCD, zero on entry
    int parts;                              // 1, 2 or L: small inputs run an item's levels in workgroups of their own, each with
                                            // a d_f1 array of its own (part p at d_f1 + p * B*HW*D), summed in order at the end
    int B, HW, D, L, r;
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    CellGrid g;
    float scale;
#ifdef CORR_TRACE
    long long* trace;
#endif
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 mma4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const float* base, size_t floats) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)(unsigned)(floats * 4), 0x00020000);
}
typedef int i32x4 __attribute__((ext_vector_type(4)));
// 4 bytes per lane from a buffer straight into LDS at lds_base + lane * 4 (lds_base, the resource and soff uniform).
// A lane whose offset lies beyond the resource's size writes zero.
__device__ __forceinline__ void dma4(i32x4 rsrc, unsigned lds_base, unsigned voff, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, unsigned off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}

// d f2_l rows of one pass = G x f1 for MT 16-point tiles (rows past the window are zero in G), then out through
// atomics.  k-step ks takes queries 4*ks + lg.  Software pipeline, pinned by the scheduling barriers: the f1 values
// of step ks + 3, the table entry of step ks + 4 and the G fragments of step ks + 1 are on their way while the
// matrix cores work on step ks.
template <int NMT, int MT, int NTW>
__device__ __forceinline__ void rows_gradient(const float* G, const unsigned* rowoff, const unsigned* q_off,
                                              __amdgpu_buffer_rsrc_t r_f1, __amdgpu_buffer_rsrc_t r_d2,
                                              unsigned ch4, int lr, int lg) {
    f32x4 acc2[MT][NTW];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) acc2[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float bq[4][NTW], af[2][MT];
    auto load_b = [&](unsigned off, float (&dst)[NTW]) {
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) dst[nt] = buf_load(r_f1, off + ch4 + 64u * nt);
    };
    // The point tiles' fragments are 16 rows of G apart (33 * 256 bytes): from a base the compiler has to take as it
    // is (the empty asm), with constant offsets, two of them leave in one LDS instruction.  Left to itself the loop
    // optimiser rebases the reads on the end of the range and spends an address addition on every one of them.
    typedef const __attribute__((address_space(3))) float* lds_cfp;
    lds_cfp gbase = (lds_cfp)G + lr * GST + lg;
    auto read_a = [&](lds_cfp gc, float (&dst)[MT]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) dst[mt] = gc[16 * mt * GST];
    };
    load_b(q_off[lg], bq[0]); load_b(q_off[4 + lg], bq[1]); load_b(q_off[8 + lg], bq[2]);
    unsigned off_next = q_off[12 + lg];
    read_a(gbase, af[0]);
#pragma unroll 1
    for (int ks0 = 0; ks0 < NMT * 4; ks0 += 4) {
        lds_cfp gstep = gbase + 4 * ks0;
        asm volatile("" : "+v"(gstep));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int ks = ks0 + s;
            load_b(off_next, bq[(s + 3) & 3]);
            off_next = q_off[4 * (ks + 4) + lg];
            read_a(gstep + 4 * (s + 1), af[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) acc2[mt][nt] = mma4(af[s & 1][mt], bq[s][nt], acc2[mt][nt]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned off = rowoff[16 * mt + 4 * lg + e] + ch4;
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt)
                __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(acc2[mt][nt][e], r_d2, (int)(off + 64u * nt), 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);                   // one tile's table reads at a time (left alone, all are hoisted)
    }
}

#ifdef CORR_TRACE
// trace builds: thread 0 adds up the 100 MHz wall clock per phase (a barrier in front of every reading, so a phase's
// time is that of its slowest wave) and leaves the item's seven sums and its tile count in trace[item][8]
#define BT(slot) do { __builtin_amdgcn_s_barrier(); if (tid == 0) { long long now = (long long)wall_clock64(); tacc[slot] += now - tlast; tlast = now; } } while (0)
#else
#define BT(slot) do {} while (0)
#endif
// One item, levels lv_lo .. lv_hi - 1, d f1 into share `part` (whole items: all levels, share 0).
// NMT: 16-query tiles the item fills (1..8)
// KT: the window side 2r + 1 as a constant (the largest radius, the usual one), or 0: taken from the arguments
// NTW: 16-channel tiles per wave: 2 (a workgroup covers 256 channels at a time), or 1 for D <= 128, so that all
// eight waves have channels to work on
template <int NMT, int KT, int NTW>
__device__ __forceinline__ void bwd_item_body(const BwdItemArgs& a, unsigned char* smem, const int4 item, const int k,
                                              const int lv_lo, const int lv_hi, const int part) {
    float* G = reinterpret_cast<float*>(smem);                   // [CH][GST]
    // byte offset of the feature row (pixel * D * 4) of each point of the pass / of each query slot; BAD_OFF: outside the level / empty
    unsigned* rowoff = reinterpret_cast<unsigned*>(smem + CH * GST * 4);   // [CH + pad]
    unsigned* q_off = rowoff + CH + TAB_PAD;                                // [128 + pad]
    float* q_cx = reinterpret_cast<float*>(q_off + CORR_GROUP + TAB_PAD);
    float* q_cy = q_cx + CORR_GROUP;
    float* taps = q_cy + CORR_GROUP;                             // [K*K][128] tap gradients of the level in work, one column per query
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lg = lane >> 4;
    const int n = item.z;
#ifdef CORR_TRACE
    long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long tlast = (long long)wall_clock64();
#endif
    int b, u, v;
    corr_cell_coords(a.g, item.x, &b, &u, &v);
    u += a.g.u_min; v += a.g.v_min;
    const int K = KT ? KT : 2 * a.r + 1, KK = K * K, D = a.D;
    const int R = (K - 1) / 2;
    if (tid < CORR_GROUP + TAB_PAD) {
        int pix = -1;
        float2 xy = make_float2(0.f, 0.f);
        if (tid < n) { pix = a.perm[item.y + tid] - b * a.HW; xy = a.sorted_c[item.y + tid]; }
        q_off[tid] = pix >= 0 ? (unsigned)pix * (unsigned)D * 4u : BAD_OFF;
        if (tid < CORR_GROUP) { q_cx[tid] = xy.x; q_cy[tid] = xy.y; }
    }
    if (tid < TAB_PAD) rowoff[CH + tid] = BAD_OFF;
    __syncthreads();
    BT(0);
    const __amdgpu_buffer_rsrc_t r_f1 = rsrc_of(a.f1 + (size_t)b * a.HW * D, (size_t)a.HW * D);
    const __amdgpu_buffer_rsrc_t r_d1 = rsrc_of(a.d_f1 + ((size_t)part * a.B + b) * a.HW * D, (size_t)a.HW * D);

    for (int cg = 0; cg < D; cg += 128 * NTW) {                  // channel groups of 128 * NTW: 16 * NTW per wave
        const int ch = cg + wave * (16 * NTW) + lr;              // this lane's channel of tile nt: ch + 16 * nt
        const bool wave_on = cg + wave * (16 * NTW) < D;         // uniform; D is a multiple of 32
        f32x4 acc1[NMT][NTW];
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) acc1[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

        // Tap gradients of one level, from d_out straight into LDS (no registers in between, so the loads can fly
        // under a contraction): wave = (half of the queries, every fourth tap), lane = query.  The level's K*K
        // planes of this batch item are one buffer: the lane's pixel is the vector offset (an empty slot's lies
        // past the end and lands as zero), the tap's plane a scalar offset; a wave's 64 values land at
        // taps[t][64 * half + lane].
        const unsigned tq_off = (tid & (CORR_GROUP - 1)) < n ? q_off[tid & (CORR_GROUP - 1)] / (unsigned)D : BAD_OFF;   // pixel * 4
        int tv_level = -1;
        auto load_taps = [&](int lv) {
            const uint64_t base = reinterpret_cast<uint64_t>(a.d_out + ((size_t)(b * a.L + lv) * KK) * a.HW);
            i32x4 rs;
            rs[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)base);
            rs[1] = __builtin_amdgcn_readfirstlane((int)((base >> 32) & 0xffffu));
            rs[2] = __builtin_amdgcn_readfirstlane(KK * a.HW * 4);
            rs[3] = __builtin_amdgcn_readfirstlane(0x00020000);
            const unsigned lds0 = __builtin_amdgcn_readfirstlane(
                (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)taps + (unsigned)(wave & 1) * 256u);
            for (int t = wave >> 1; t < KK; t += NTI / CORR_GROUP)
                dma4(rs, __builtin_amdgcn_readfirstlane(lds0 + (unsigned)t * (CORR_GROUP * 4)), tq_off,
                     __builtin_amdgcn_readfirstlane(t * a.HW * 4));
            tv_level = lv;
        };
        for (int l = lv_lo; l < lv_hi; ++l) {
            const int Hl = a.Hl[l], Wl = a.Wl[l];
            const int CXL = max((1 << CORR_LOG_CX) >> l, 1), CYL = max((1 << CORR_LOG_CY) >> l, 1);
            const int WSX = CXL + K, WSY = CYL + K, NPTS = WSX * WSY;
            const int xs = ((u << CORR_LOG_CX) >> l) - R, ys = ((v << CORR_LOG_CY) >> l) - R;
            if (!(xs + WSX - 1 >= 0 && xs <= Wl - 1 && ys + WSY - 1 >= 0 && ys <= Hl - 1)) continue;   // all padding (uniform)
            const __amdgpu_buffer_rsrc_t r_f2 = rsrc_of(a.f2[l] + (size_t)b * Hl * Wl * D, (size_t)Hl * Wl * D);
            const __amdgpu_buffer_rsrc_t r_d2 = rsrc_of(a.d_f2[l] + (size_t)b * Hl * Wl * D, (size_t)Hl * Wl * D);
            // this level's tap gradients: on their way into LDS since the previous level's last pass, or loaded now
            // (the first level, or one after a level that was all padding)
            if (tv_level != l) {
                __syncthreads();                                 // the previous level's last pass no longer reads taps
                load_taps(l);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's part has landed; the passes' barriers cover the others'
            BT(1);
            for (int r0 = 0; r0 < NPTS; r0 += CH) {
                __syncthreads();                                 // the previous pass no longer reads G or rowoff
                {
                    float4* g4 = reinterpret_cast<float4*>(G);
                    for (int i = tid; i < CH * GST / 4; i += NTI) g4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (tid < CH) {
                        const int row = r0 + tid, wy = row / WSX, wx = row - wy * WSX;
                        const int y = ys + wy, x = xs + wx;
                        rowoff[tid] = (row < NPTS && y >= 0 && y < Hl && x >= 0 && x < Wl) ? (unsigned)(y * Wl + x) * (unsigned)D * 4u : BAD_OFF;
                    }
                }
                __syncthreads();
                BT(2);
                {
                    // footprint weights into G: thread = (query, quarter of the footprint columns).  Point (pu, pv)
                    // collects the taps (pu - du, pv - dv), du, dv in {0, 1}, with their corner weights; every
                    // element of G has one writer, so G (and with it d f1) is the same bits on every call.
                    const int q = tid & (CORR_GROUP - 1), part = tid >> 7;
                    if (q < n) {
                        const float inv = __uint_as_float((uint32_t)(127 - l) << 23);
                        const float cxl = q_cx[q] * inv, cyl = q_cy[q] * inv;
                        const float flx = floorf(cxl), fly = floorf(cyl);
                        const float fx = cxl - flx, fy = cyl - fly;
                        const int rx = (int)flx - R - xs, ry = (int)fly - R - ys;
                        const float wx1 = fx * a.scale, wx0 = a.scale - wx1;
                        const int p0 = part * (K + 1) / 4, p1 = (part + 1) * (K + 1) / 4;
                        const float* dp = taps + q;
                        float* gq = G + q;
                        for (int pu = p0; pu < p1; ++pu) {
                            // the column's horizontally weighted taps first (all LDS reads in flight at once), then its K + 1 points
                            const float w0 = pu < K ? wx0 : 0.f, w1 = pu >= 1 ? wx1 : 0.f;
                            const float* c0 = dp + min(pu, K - 1) * K * CORR_GROUP;
                            const float* c1 = dp + max(pu - 1, 0) * K * CORR_GROUP;
                            float t[MAXK + 1];
#pragma unroll
                            for (int j = 0; j < MAXK; ++j) {
                                const int jj = min(j, K - 1);
                                t[j] = j < K ? c0[jj * CORR_GROUP] * w0 + c1[jj * CORR_GROUP] * w1 : 0.f;
                            }
                            t[MAXK] = 0.f;
                            int rr = ry * WSX + rx + pu - r0;
#pragma unroll
                            for (int pv = 0; pv <= MAXK; ++pv) {
                                const float tprev = pv >= 1 ? t[pv - 1] : 0.f;
                                if (pv <= K && (unsigned)rr < (unsigned)CH) gq[rr * GST] = t[pv] + fy * (tprev - t[pv]);
                                rr += WSX;
                            }
                        }
                    }
                }
                __syncthreads();
                BT(3);
                if (wave_on) {
                    const int rows = min(CH, NPTS - r0);
                    const unsigned ch4 = (unsigned)ch * 4u;
                    float bq[4][NTW];
                    // d f1 += G^T x f2 rows.  k-step ks takes points 4*ks + lg.  Software pipeline, pinned by the
                    // scheduling barriers: the f2 values of step ks + 3, the table entry of step ks + 4 and the G
                    // fragments of step ks + 1 are on their way while the matrix cores work on step ks.  Steps
                    // past the last one find BAD_OFF in the table (zeros) and rows of zeros in G.
                    const int nks = (rows + 3) >> 2;
                    {
                        float af[2][NMT];
                        auto load_b = [&](unsigned off, float (&dst)[NTW]) {
#pragma unroll
                            for (int nt = 0; nt < NTW; ++nt) dst[nt] = buf_load(r_f2, off + ch4 + 64u * nt);
                        };
                        auto read_a = [&](int ks, float (&dst)[NMT]) {
                            const float* gr = G + (4 * ks + lg) * GST + lr;
#pragma unroll
                            for (int mt = 0; mt < NMT; ++mt) dst[mt] = gr[16 * mt];
                        };
                        load_b(rowoff[lg], bq[0]); load_b(rowoff[4 + lg], bq[1]); load_b(rowoff[8 + lg], bq[2]);
                        unsigned off_next = rowoff[12 + lg];
                        read_a(0, af[0]);
#pragma unroll 1
                        for (int ks0 = 0; ks0 < nks; ks0 += 4) {
#pragma unroll
                            for (int s = 0; s < 4; ++s) {
                                const int ks = ks0 + s;
                                load_b(off_next, bq[(s + 3) & 3]);
                                off_next = rowoff[4 * (ks + 4) + lg];
                                read_a(ks + 1, af[(s + 1) & 1]);
                                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                                for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
                                    for (int nt = 0; nt < NTW; ++nt) acc1[mt][nt] = mma4(af[s & 1][mt], bq[s][nt], acc1[mt][nt]);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
                }
                BT(4);
                // the next level's tap gradients start to move under the second contraction of this level's last
                // pass (every wave is past the pass's scatter, the last reader of the current ones)
                if (r0 + CH >= NPTS && l + 1 < lv_hi) load_taps(l + 1);
                if (wave_on) {
                    const int rows = min(CH, NPTS - r0);
                    const unsigned ch4 = (unsigned)ch * 4u;
                    // d f2_l rows of this pass = G x f1, over as many 16-point tiles as the pass has rows (rounded up to odd)
                    const int tiles = (rows + 15) >> 4;
                    if (tiles <= 3) rows_gradient<NMT, 3, NTW>(G, rowoff, q_off, r_f1, r_d2, ch4, lr, lg);
                    else if (tiles <= 5) rows_gradient<NMT, 5, NTW>(G, rowoff, q_off, r_f1, r_d2, ch4, lr, lg);
                    else if (tiles <= 7) rows_gradient<NMT, 7, NTW>(G, rowoff, q_off, r_f1, r_d2, ch4, lr, lg);
                    else rows_gradient<NMT, MTC, NTW>(G, rowoff, q_off, r_f1, r_d2, ch4, lr, lg);
                }
                BT(5);
            }
        }
        if (wave_on) {
#pragma unroll
            for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned off = q_off[16 * mt + 4 * lg + e] + (unsigned)ch * 4u;
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt)
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc1[mt][nt][e]), r_d1, (int)(off + 64u * nt), 0, 0);
                }
        }
    }
    // a prefetch for a level that turned out to be all padding may still be in flight: nothing may land in LDS after the end
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#ifdef CORR_TRACE
    BT(6);
    if (tid == 0 && a.trace) { for (int i = 0; i < 7; ++i) a.trace[(size_t)k * 8 + i] = tacc[i]; a.trace[(size_t)k * 8 + 7] = NMT; }
#endif
}

// One workgroup per compute unit, each taking items from a queue until it is empty.  Workgroup w runs on XCD
// w % 8 and serves that XCD's share of the item list in list order (runs of CORR_XCD_RUN consecutive items, as in
// the forward kernel: neighbouring cells share window rows, so they should share an L2 and run at about the same
// time); a workgroup whose queue has run out goes on with the next XCD's.  So no compute unit spends time on
// workgroups that find nothing to do (one of this kernel's workgroups needs most of a unit's LDS, so even an empty
// one waits for a unit of its own), and the end of the launch is shared out item by item.  Handing out the full
// items first and the small ones last was measured too: it costs more in L2 misses than it gains at the end.
__global__ __launch_bounds__(NTI, 2) void bwd_item_kernel(BwdItemArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_next;
    int xcd = (int)blockIdx.x & 7, tried = 0;
    const int n_items = *a.n_items;
    const int share = (n_items + 8 * CORR_XCD_RUN - 1) / (8 * CORR_XCD_RUN) * CORR_XCD_RUN;   // item positions per queue
    for (;;) {
        __syncthreads();                                   // the previous item's last LDS reads; s_next has been read
        if (threadIdx.x == 0) s_next = atomicAdd(a.queue + xcd, 1);
        __syncthreads();
        const int pos = s_next;                            // uniform
        if (pos >= share * a.parts) {                  // this queue is empty: help the next XCD's, until all eight are
            if (++tried == 8) break;
            xcd = (xcd + 1) & 7;
            continue;
        }
        // with parts > 1 consecutive positions are the levels of one item
        const int part = pos % a.parts, ipos = pos / a.parts;
        const int k = corr_item_of_workgroup(ipos * 8 + xcd);
        if (k >= n_items) continue;
        const int4 item = a.items[k];
        const int tiles = (item.z + 15) >> 4;
        // parts = L: one level each; parts = 2 (and L > 2): level 0, and the rest
        const int lv_lo = a.parts > 1 ? part : 0;
        const int lv_hi = a.parts == 1 || (a.parts == 2 && part == 1) ? a.L : part + 1;
#define CORR_BWD_CASE(N, KT, NTW) case N: bwd_item_body<N, KT, NTW>(a, smem, item, k, lv_lo, lv_hi, part); break;
#define CORR_BWD_SWITCH(KT, NTW)                                                                              \
        switch (tiles) {                                                                                      \
            CORR_BWD_CASE(1, KT, NTW) CORR_BWD_CASE(2, KT, NTW) CORR_BWD_CASE(3, KT, NTW) CORR_BWD_CASE(4, KT, NTW) \
            CORR_BWD_CASE(5, KT, NTW) CORR_BWD_CASE(6, KT, NTW) CORR_BWD_CASE(7, KT, NTW)                     \
            default: bwd_item_body<8, KT, NTW>(a, smem, item, k, lv_lo, lv_hi, part); break;                  \
        }
        if (a.D <= 128) {
            if (a.r == CORR_R) { CORR_BWD_SWITCH(MAXK, 1) } else { CORR_BWD_SWITCH(0, 1) }
        } else {
            if (a.r == CORR_R) { CORR_BWD_SWITCH(MAXK, 2) } else { CORR_BWD_SWITCH(0, 2) }
        }
#undef CORR_BWD_SWITCH
#undef CORR_BWD_CASE
    }
}

// Channels-last gradients to NCHW, and for fmap2 the levels' gradients down the pyramid in the same pass.
// Adjoint of the 2x2 mean: a pixel of level l - 1 receives a quarter of its parent's gradient at level l, if it
// has a parent (a trailing odd row or column that the pooling dropped has none, and then none at the deeper
// levels either).  For a level-0 pixel that is the nested sum d0 + (d1 + (d2 + d3 / 4) / 4) / 4 along its chain
// of parents, evaluated from the deepest level.  With L = 1 this is a plain transposition (d_fmap1).
// A workgroup moves 64 pixels x 64 channels through LDS: 16-byte loads along the channels (a wave reads four
// pixels' 256 bytes), 256-byte runs along the pixels on the way out.
struct GatherOne {
    const float* d[CORR_MAX_L];
    float* dst;
    int L;                      // levels to fold (1: a plain transposition)
    int parts;                  // d[0] is the sum of this many arrays, part_stride floats apart (d_fmap1 of a small input)
    size_t part_stride;
};
struct GatherArgs {
    GatherOne out[2];           // blockIdx.z = which * B + batch item
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    int B, D, W, HW;
};
constexpr int TP = 64, TC = 64;
__global__ __launch_bounds__(256) void bwd_gather_nchw_kernel(GatherArgs g) {
    __shared__ float tile[TC][TP + 1];
    const int which = (int)blockIdx.z / g.B, b = (int)blockIdx.z - which * g.B;
    const GatherOne& o = g.out[which];
    const int p0 = blockIdx.x * TP, d0 = blockIdx.y * TC;
#pragma unroll
    for (int k = 0; k < TP * TC / 4 / 256; ++k) {
        const int idx = threadIdx.x + 256 * k, c4 = idx & (TC / 4 - 1), pr = idx / (TC / 4);
        const int p = p0 + pr, ch = d0 + 4 * c4;
        if (p < g.HW && ch < g.D) {                        // D is a multiple of 4
            const int y = p / g.W, x = p - y * g.W;
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int l = o.L - 1; l >= 1; --l) {
                const int yy = y >> l, xx = x >> l;
                if (yy < g.Hl[l] && xx < g.Wl[l]) {
                    const float4 v = *reinterpret_cast<const float4*>(o.d[l] + (((size_t)b * g.Hl[l] + yy) * g.Wl[l] + xx) * g.D + ch);
                    t = make_float4(v.x + 0.25f * t.x, v.y + 0.25f * t.y, v.z + 0.25f * t.z, v.w + 0.25f * t.w);
                }
            }
            const float* src = o.d[0] + ((size_t)b * g.HW + p) * g.D + ch;
            float4 v = *reinterpret_cast<const float4*>(src);
            for (int part = 1; part < o.parts; ++part) {
                const float4 w = *reinterpret_cast<const float4*>(src + part * o.part_stride);
                v = make_float4(v.x + w.x, v.y + w.y, v.z + w.z, v.w + w.w);
            }
            tile[4 * c4 + 0][pr] = v.x + 0.25f * t.x;
            tile[4 * c4 + 1][pr] = v.y + 0.25f * t.y;
            tile[4 * c4 + 2][pr] = v.z + 0.25f * t.z;
            tile[4 * c4 + 3][pr] = v.w + 0.25f * t.w;
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TP * TC / 256; ++k) {
        const int idx = threadIdx.x + 256 * k, px = idx & (TP - 1), chn = idx / TP;
        if (d0 + chn < g.D && p0 + px < g.HW) o.dst[((size_t)b * g.D + d0 + chn) * g.HW + p0 + px] = tile[chn][px];
    }
}

}  // namespace

// Small inputs run an item's levels in workgroups of their own (a map of a few thousand queries has fewer items
// than the chip has compute units, and the call's time is one item's latency); each level then adds into a d f1
// array of its own and the final gather sums them in level order, so the result stays the same bits on every call.
#ifndef CORR_BACKWARD_SPLIT_MAX_QUERIES
#define CORR_BACKWARD_SPLIT_MAX_QUERIES 32000   // measured: the split gains up to about 28000 queries and costs 8 % at 45000
#endif
#ifndef CORR_BACKWARD_HALVE_MAX_QUERIES
#define CORR_BACKWARD_HALVE_MAX_QUERIES 40000   // up to here an item is two pieces: level 0 (three passes) and the other levels (four); measured: -7 % at 32400 queries, nothing from 45000 on
#endif
static int backward_parts(int B, int H, int W, int L) {
    const long long BN = (long long)B * H * W;
    return BN <= CORR_BACKWARD_SPLIT_MAX_QUERIES ? L : (BN <= CORR_BACKWARD_HALVE_MAX_QUERIES && L > 1) ? 2 : 1;
}
size_t corr_backward_workspace_floats(int B, int H, int W, int D, int L) {
    size_t px = 0;
    for (int l = 0; l < L; ++l) px += (size_t)(H >> l) * (W >> l);
    return ((size_t)backward_parts(B, H, W, L) * B * H * W + (size_t)B * px) * D;
}

// gradient arrays (rounded up to 256 bytes), then a planning workspace like the pyramid's (the call bins the
// queries itself and leaves the pyramid's own workspace alone)
static size_t grad_bytes(int B, int H, int W, int D, int L) {
    return (corr_backward_workspace_floats(B, H, W, D, L) * sizeof(float) + 255) & ~(size_t)255;
}
size_t corr_backward_workspace_bytes_internal(int B, int H, int W, int D, int L) {
    CellGrid g;
    corr_fill_grid(&g, H, W, L);
    return grad_bytes(B, H, W, D, L) + corr_ws_layout(B * H * W, corr_ncells(g, B)).total;
}

#ifdef CORR_TRACE
static long long* g_bwd_trace = nullptr;
extern "C" void corr_debug_set_backward_trace(long long* p) { g_bwd_trace = p; }
#endif
hipError_t launch_backward(const corr_pyramid* p, const float* coords, const float* d_out, int r,
                           float* d_fmap1, float* d_fmap2, float* ws, int form, int split_max, hipStream_t s) {
    const int HW = p->H * p->W;
    float* cur = ws;
    // the test hook can switch the splitting of levels off (a setting of 0; the workspace is laid out for the default)
    const bool split = split_max != 0;
    const int parts = form == CORR_BACKWARD_ITEMS && split ? backward_parts(p->B, p->H, p->W, p->L) : 1;
    float* d_f1 = cur; cur += (size_t)backward_parts(p->B, p->H, p->W, p->L) * p->B * HW * p->D;
    float* d_f2[CORR_MAX_L] = {nullptr, nullptr, nullptr, nullptr};
    size_t lev_floats = 0;
    for (int l = 0; l < p->L; ++l) {
        d_f2[l] = cur;
        const size_t n = (size_t)p->B * p->Hl[l] * p->Wl[l] * p->D;
        cur += n; lev_floats += n;
    }
    const float scale = 1.0f / sqrtf((float)p->D);
    const long long BN = (long long)p->B * HW;
    hipError_t e;
    if (form == CORR_BACKWARD_ITEMS) {
        // Everything accumulates or keeps its zero; in the planning workspace the bin counters, the item counters and
        // the item kernel's queues (kept in the statistics slots) start at zero, the rest is written before it is
        // read.  Fill kernels, so the call can be graph-captured.  A small input's whole workspace is cleared in one
        // launch: there the call's time is launches and one item's latency.
        const size_t gbytes = grad_bytes(p->B, p->H, p->W, p->D, p->L);
        const int ncells = corr_ncells(p->grid, p->B);
        const BinWs bws = corr_ws_carve(reinterpret_cast<char*>(ws) + gbytes, (int)BN, ncells);
        if (backward_parts(p->B, p->H, p->W, p->L) > 1) {
            const size_t all = gbytes + corr_ws_layout((int)BN, ncells).total;
            if ((e = launch_fill_i32(reinterpret_cast<int*>(ws), 0, all / 4, s)) != hipSuccess) return e;
        } else {
            if ((e = launch_fill_i32(reinterpret_cast<int*>(ws), 0, (size_t)(cur - ws), s)) != hipSuccess) return e;
            if ((e = launch_fill_i32(bws.bin_count, 0, (size_t)bws.nbins, s)) != hipSuccess) return e;
            // item counters and, right behind them, the statistics slots
            const size_t tail = (size_t)(reinterpret_cast<int*>(bws.stats) + 2 * CORR_NSTATS - bws.n_items);
            if ((e = launch_fill_i32(bws.n_items, 0, tail, s)) != hipSuccess) return e;
        }
        LookupArgs q{coords, nullptr, r, 0, 0, 0};
        if ((e = launch_binning(p, bws, q, s)) != hipSuccess) return e;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_item_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, ITEM_LDS);
        if (attr != hipSuccess) return attr;
        BwdItemArgs a;
#ifdef CORR_TRACE
        a.trace = g_bwd_trace;
#endif
        a.f1 = p->f1_nhwc; a.d_f1 = d_f1; a.d_out = d_out;
        a.perm = bws.perm; a.sorted_c = bws.sorted_c; a.items = bws.items; a.n_items = bws.n_items; a.queue = reinterpret_cast<int*>(bws.stats); a.parts = parts;
        a.B = p->B; a.HW = HW; a.D = p->D; a.L = p->L; a.r = r; a.g = p->grid; a.scale = scale;
        for (int l = 0; l < CORR_MAX_L; ++l) {
            a.f2[l] = l < p->L ? p->f2_nhwc[l] : nullptr; a.d_f2[l] = d_f2[l];
            a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l];
        }
        hipLaunchKernelGGL(bwd_item_kernel, dim3(CORR_NUM_CU), dim3(NTI), ITEM_LDS, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else {
        BwdArgs a;
        a.f1 = p->f1_nhwc; a.coords = coords; a.d_out = d_out;
        a.B = p->B; a.HW = HW; a.D = p->D; a.L = p->L; a.r = r; a.scale = scale;
        a.d_f1 = d_f1;
        for (int l = 0; l < CORR_MAX_L; ++l) {
            a.f2[l] = l < p->L ? p->f2_nhwc[l] : nullptr; a.d_f2[l] = d_f2[l];
            a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l];
        }
        if ((e = launch_fill_i32(reinterpret_cast<int*>(d_f2[0]), 0, lev_floats, s)) != hipSuccess) return e;
        hipLaunchKernelGGL(bwd_query_kernel, dim3((unsigned)((BN + BQ - 1) / BQ)), dim3(64 * BQ), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    // both gradients to NCHW in one launch: d_fmap1 (a small input's per-level shares summed), d_fmap2 (levels folded)
    GatherArgs ga;
    for (int l = 0; l < CORR_MAX_L; ++l) {
        ga.Hl[l] = p->Hl[l]; ga.Wl[l] = p->Wl[l];
        ga.out[0].d[l] = nullptr; ga.out[1].d[l] = d_f2[l];
    }
    ga.out[0].d[0] = d_f1; ga.out[0].dst = d_fmap1; ga.out[0].L = 1;
    ga.out[0].parts = parts; ga.out[0].part_stride = (size_t)p->B * HW * p->D;
    ga.out[1].dst = d_fmap2; ga.out[1].L = p->L; ga.out[1].parts = 1; ga.out[1].part_stride = 0;
    ga.B = p->B; ga.D = p->D; ga.W = p->W; ga.HW = HW;
    hipLaunchKernelGGL(bwd_gather_nchw_kernel, dim3((HW + TP - 1) / TP, (p->D + TC - 1) / TC, 2 * p->B), dim3(256), 0, s, ga);
    return hipGetLastError();
}
