// Per-lookup compute (paper: steps b and c, "Sparse Correlation Volume
// Computation" and "Sparse Volume Sampling"; fused as in "Fused Implementation":
// the computed block lives only in registers and LDS).
//
// One workgroup (4 waves, the only one on its CU) = one work item = (target cell of 16 x 8
// level-0 pixels, up to 128 of its queries), processed level after level.  Wave w owns queries
// 32w .. 32w+31 of the item as two MFMA column blocks of 16.
//   queries     : each wave loads the bf16 hi (and lo) fragments of its queries for 256 channels
//                 once per item, straight from global memory into the MFMA B-operand layout, and
//                 keeps them in registers for all levels (a larger D runs in groups of 256 channels
//                 with the fragments reloaded).
//   contraction : S_l[pt][q] = <f2_l(window point pt), f1(query q)> over D.  The window is
//                 streamed through LDS in units of (32-channel chunk, group of 16-point row blocks):
//                 every thread issues 16-byte buffer loads that write LDS directly (no registers
//                 in between), whole 128-byte pixel records per 8 lanes, the 16-byte pieces permuted
//                 on the global side so that the LDS rows come out XOR-swizzled and the fragment
//                 reads are conflict-free.  The units of a level go round a ring of LDS slots that
//                 keeps several of them in flight ahead of the one being multiplied; the waits are
//                 explicit vmcnt counts, one barrier per unit.  Every wave multiplies the row blocks
//                 with its own query fragments on v_mfma_f32_16x16x32_bf16 (rows = window points,
//                 columns = queries); fp32 features enter as bf16 hi + lo and the three significant
//                 partial products are accumulated in fp32 (hi*hi + hi*lo + lo*hi), or hi*hi alone
//                 in bf16 mode.  The accumulators (up to 27 blocks x 2 x 4 registers) live in the
//                 second half of the 512-register file a lone wave per SIMD has.
//   epilogue    : S_l goes to LDS as [pt][query], 64 queries at a time; each query reads the 2x2
//                 stencil of its own (2r+2)^2 sub-window and writes its (2r+1)^2 taps.  The first
//                 units of the next level are already loading into the LDS above S.
// Window points outside the level are staged as zeros, which is the zero
// padding of the sampling rule.
#include "corr_internal.h"

#ifdef CORR_TRACE
extern long long* g_corr_trace;
#endif

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// This file is compiled once per lookup radius (CORR_BLOCK_R = 1..4): window sizes, LDS sizes and
// the tap loops are compile-time functions of it.
#ifndef CORR_BLOCK_R
#define CORR_BLOCK_R CORR_R
#endif
#define CORR_CAT2(a, b) a##b
#define CORR_CAT(a, b) CORR_CAT2(a, b)
constexpr int R = CORR_BLOCK_R, K = 2 * R + 1, KK = K * K;
constexpr int CX = 1 << CORR_LOG_CX, CY = 1 << CORR_LOG_CY;
constexpr int NW = 4, NT = 64 * NW;
constexpr int QW = CORR_GROUP / NW;                    // queries per wave: two column blocks of 16
constexpr int XCD_RUN = 32;                            // consecutive items dealt to one XCD; a power of two
constexpr int NCMAX = CORR_BLOCK_MAX_D / CORR_CHUNK;   // chunks of query fragments a wave holds
constexpr int LDS_BYTES = 160 * 1024;
constexpr int META_BYTES = CORR_GROUP * 12;
constexpr int LDS_DATA = LDS_BYTES - META_BYTES;       // ring slots and S
constexpr int OOB = (int)0x80000000u;                  // a buffer offset beyond the whole pyramid (< 2 GiB): loads zeros
static_assert(QW == 32 && NW == 4, "a wave owns two 16-query column blocks");

struct BlockArgs {
    const uint16_t* f1s;                 // [NC][B*HW][rec]
    const uint16_t* f2s;                 // [NC][P][rec], P = pixels of all levels; level l starts at pix_base[l]
    const float* coords;                 // [B][2][HW]
    const int* perm;
    const int4* items;
    const int* n_items;
    float* out;
    int B, HW, NC, L;
    int tap_stride, pix_stride;          // layout of out
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L], pix_base[CORR_MAX_L];
    int f1_stride;                       // elements between chunk planes of f1s
    unsigned f2_plane_bytes;             // bytes of one chunk plane of f2s
    int rec;                             // elements per pixel record: 64 (hi + lo) or 32 (hi only)
    CellGrid g;
    float scale;
#ifdef CORR_TRACE
    long long* trace;                    // [items][16] timestamps (debug builds)
#endif
};

constexpr int cmax(int a, int b) { return a > b ? a : b; }
constexpr int cmin(int a, int b) { return a < b ? a : b; }

template <int LVL, bool THREE>
struct Geo {
    static constexpr int PPR = THREE ? 8 : 4;             // 16-byte pieces staged per row (hi, and lo if used)
    static constexpr int ROWB = PPR * 16;                 // LDS bytes per staged row (pieces swizzled, no padding)
    static constexpr int CXL = cmax(CX >> LVL, 1), CYL = cmax(CY >> LVL, 1);
    static constexpr int WSX = CXL + K, WSY = CYL + K;    // window sides
    static constexpr int NPTS = WSX * WSY;
    static constexpr int NB = (NPTS + 15) / 16;           // 16-point row blocks
    static constexpr int ROWS = NB * 16;
    static constexpr int NG = NB > 16 ? 2 : 1;            // row-block groups a chunk is streamed in (block b: group b % NG)
    static constexpr int BPS = (NB + NG - 1) / NG;        // blocks per unit
    static constexpr int ITERS = (BPS * 16 * ROWB + 4095) / 4096;   // 16-byte loads per thread and unit
    static constexpr int SLOT = ITERS * 4096;             // LDS bytes of a ring slot
    static constexpr int NU = NCMAX * NG;                 // units per group of NCMAX chunks
    static constexpr int S_BYTES = ROWS * 64 * 4;         // S of one epilogue round: [ROWS][64 queries] fp32
    // swizzle: the piece slot of a row is XORed with this, so that the 16 rows x 16 bytes a quarter
    // wave reads for one MFMA fragment fall in 16 different 4-bank groups
    __device__ static constexpr int swz(int r) { return PPR == 8 ? ((r >> 1) & 7) : ((r >> 2) & 3); }
};
// Ring of a level: the slots that lie above the previous level's S can be filled while that
// level's epilogue still reads S ("upper" slots, used first); the others reuse the space of S.
template <int LVL, bool THREE>
struct Ring {
    using G = Geo<LVL, THREE>;
    static constexpr int SPREV = LVL == 0 ? 0 : Geo<(LVL > 0 ? LVL - 1 : 0), THREE>::S_BYTES;
    static constexpr int UP = (LDS_DATA - SPREV) / G::SLOT;
    static constexpr int LOW = SPREV / G::SLOT;
    static constexpr int NS0 = cmin(G::NU, UP + LOW);
    static constexpr int NS = NS0 / G::NG * G::NG;        // a slot always holds the same group of row blocks
    static constexpr int PRE = cmin(UP, NS);              // units that can be issued before the previous epilogue
    static_assert(NS >= 2 && NS >= G::NG, "ring too small");
    static_assert(G::S_BYTES <= LDS_DATA, "S does not fit");
    __device__ static constexpr int slot_off(int i) { return i < PRE ? SPREV + i * G::SLOT : (i - PRE) * G::SLOT; }
    // loads that may still be in flight behind unit u when it is waited for
    __device__ static constexpr int younger(int u) { return cmin(G::NU - 1, NS - 1 + cmax(u - 1, 0)) - u; }
};

#ifdef CORR_TRACE
#define TRACE(slot) do { if (c.tid == 0 && a.trace) a.trace[(size_t)c.item * 16 + (slot)] = (long long)wall_clock64(); } while (0)
#else
#define TRACE(slot) do {} while (0)
#endif

struct ItemCtx {
    int item;
    int b, u, v, n;          // batch item, absolute cell coordinates, queries in the group
    int tid, lane, wave;
    const int* q_pix;        // LDS: pixel of each query slot or -1
    const float* q_cx;       // LDS: raw coordinates
    const float* q_cy;
    unsigned lds_wave;       // LDS byte address of smem + wave * 1024 (uniform)
#ifdef CORR_DEBUG_SYNC_STAGE
    unsigned char* dbg_smem;
#endif
    i32x4 rsrc, rsrc_null;   // buffer resources: all chunk planes of f2s; an empty buffer
};

// 16 bytes per lane from a buffer straight into LDS at lds_base + lane * 16.  A lane whose
// voffset + soffset lies beyond the resource's size writes zeros (measured on gfx950).
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned lds_base, int voff, unsigned soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit count");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int LVL>
__device__ __forceinline__ void window_origin(const ItemCtx& c, int& xs, int& ys) {
    xs = ((c.u << CORR_LOG_CX) >> LVL) - R;
    ys = ((c.v << CORR_LOG_CY) >> LVL) - R;
}

template <int LVL, bool THREE>
__device__ __forceinline__ bool window_touches(const BlockArgs& a, const ItemCtx& c) {
    using G = Geo<LVL, THREE>;
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    return xs + G::WSX - 1 >= 0 && xs <= a.Wl[LVL] - 1 && ys + G::WSY - 1 >= 0 && ys <= a.Hl[LVL] - 1;
}
// Byte offsets (within a chunk plane) of the 16-byte pieces this thread moves for every unit of
// level LVL: voff[g][it] feeds LDS position it * 256 + tid of a slot that holds group g.
template <int LVL, bool THREE>
__device__ __forceinline__ void plan(const BlockArgs& a, const ItemCtx& c, int (&voff)[Geo<LVL, THREE>::NG][Geo<LVL, THREE>::ITERS]) {
    using G = Geo<LVL, THREE>;
    const int Hl = a.Hl[LVL], Wl = a.Wl[LVL];
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    const int base = a.pix_base[LVL] + c.b * Hl * Wl;
#pragma unroll
    for (int g = 0; g < G::NG; ++g)
#pragma unroll
        for (int it = 0; it < G::ITERS; ++it) {
            const int idx = it * NT + c.tid;
            const int rs = idx / G::PPR, sp = idx % G::PPR;       // row of the slot, piece slot in the row
            const int r = rs & 15;
            const int row = ((rs >> 4) * G::NG + g) * 16 + r;     // window point
            const int piece = sp ^ G::swz(r);                     // pieces 0..3: hi record, 4..7: lo record
            const int wy = row / G::WSX, wx = row - wy * G::WSX;
            const int y = ys + wy, x = xs + wx;
            const bool ok = row < G::NPTS && y >= 0 && y < Hl && x >= 0 && x < Wl;
            voff[g][it] = ok ? (base + y * Wl + x) * (a.rec * 2) + piece * 16 : OOB;
        }
}

// issue the loads of unit u (chunk kc0 + u / NG, group u % NG) into its ring slot
template <int LVL, bool THREE, int U>
__device__ __forceinline__ void issue_unit(const BlockArgs& a, const ItemCtx& c,
                                           const int (&voff)[Geo<LVL, THREE>::NG][Geo<LVL, THREE>::ITERS], int kc0) {
    using G = Geo<LVL, THREE>;
    using RG = Ring<LVL, THREE>;
    constexpr int g = U % G::NG, slot = U % RG::NS;
    const int kc = kc0 + U / G::NG;
    const bool real = kc < a.NC;                                  // uniform
    const i32x4 rs = real ? c.rsrc : c.rsrc_null;
    const unsigned soff = real ? (unsigned)kc * a.f2_plane_bytes : 0u;
#pragma unroll
    for (int it = 0; it < G::ITERS; ++it) {
#ifdef CORR_DEBUG_SYNC_STAGE
        uint4 v = make_uint4(0, 0, 0, 0);
        if (real && voff[g][it] != OOB) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.f2s) + soff + voff[g][it]);
        *reinterpret_cast<uint4*>(c.dbg_smem + RG::slot_off(slot) + (it * NT + c.tid) * 16) = v;
#else
        dma16(rs, c.lds_wave + RG::slot_off(slot) + it * 4096, voff[g][it], soff);
#endif
    }
}

// Query fragments of this wave for chunks kc0 .. kc0+NCMAX-1: lane holds channels 8*(lane/16) .. +7 of
// every chunk of queries 32*wave + 16*h + lane%16 (the B operands of the MFMA).
template <bool THREE>
__device__ __forceinline__ void load_queries(const BlockArgs& a, const ItemCtx& c, int kc0,
                                             bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX]) {
    const char* base = reinterpret_cast<const char*>(a.f1s);          // uniform; byte offsets fit 32 bits
    const unsigned plane = (unsigned)a.f1_stride * 2u;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pix = c.q_pix[c.wave * QW + h * 16 + (c.lane & 15)];
        const unsigned off = ((unsigned)(c.b * a.HW + max(pix, 0)) * (unsigned)a.rec + (unsigned)(c.lane >> 4) * 8u) * 2u;
#pragma unroll
        for (int kk = 0; kk < NCMAX; ++kk) {
            // no predicates: an empty query slot reads pixel 0 and a chunk past the last one reads the
            // last; the products of those columns and chunks are never used
            const unsigned o = off + (unsigned)min(kc0 + kk, a.NC - 1) * plane;
            const uint4 hv = *reinterpret_cast<const uint4*>(base + o);
            uint4 lv = make_uint4(0, 0, 0, 0);
            if (THREE) lv = *reinterpret_cast<const uint4*>(base + (o + 64u));
            qhi[h][kk] = __builtin_bit_cast(bf16x8, hv);
            qlo[h][kk] = __builtin_bit_cast(bf16x8, lv);
        }
    }
    // The compiler's wait-count bookkeeping does not see the LDS loads issued from inline assembly.
    // A full wait here, on a path every wave takes, leaves it with nothing pending, so it never
    // puts a small vmcnt of its own (which would drain the ring) in front of the MFMAs.
    __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0), expcnt and lgkmcnt untouched
}

// the MFMAs of unit U: every row block of its group against this wave's two query column blocks.
// The fragment reads run two row blocks ahead of the MFMAs that use them; sched_group_barrier
// pins that order (left alone, the scheduler hoists every read of the unit and spills).
template <int LVL, bool THREE, int U>
__device__ __forceinline__ void mfma_unit(const ItemCtx& c, const unsigned char* smem,
                                          const bf16x8 (&qhi)[2][NCMAX], const bf16x8 (&qlo)[2][NCMAX],
                                          f32x4 (&acc)[Geo<LVL, THREE>::NB][2], int frag_hi, int frag_lo) {
    using G = Geo<LVL, THREE>;
    using RG = Ring<LVL, THREE>;
    constexpr int g = U % G::NG, slot = U % RG::NS, kc = U / G::NG;
    constexpr int NJ = (G::NB - g + G::NG - 1) / G::NG;      // row blocks of this group
    constexpr int PF = 2;
    const unsigned char* rows = smem + RG::slot_off(slot);
    bf16x8 wh[NJ + PF], wl[NJ + PF];
#pragma unroll
    for (int j = 0; j < PF; ++j) {
        if (j < NJ) {
            wh[j] = *reinterpret_cast<const bf16x8*>(rows + j * 16 * G::ROWB + frag_hi);
            if (THREE) wl[j] = *reinterpret_cast<const bf16x8*>(rows + j * 16 * G::ROWB + frag_lo);
        }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, (THREE ? 2 : 1) * cmin(PF, NJ), 0);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int b = j * G::NG + g;
        if (j + PF < NJ) {
            wh[j + PF] = *reinterpret_cast<const bf16x8*>(rows + (j + PF) * 16 * G::ROWB + frag_hi);
            if (THREE) wl[j + PF] = *reinterpret_cast<const bf16x8*>(rows + (j + PF) * 16 * G::ROWB + frag_lo);
        }
        if (THREE) {
            acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[j], qhi[0][kc], acc[b][0], 0, 0, 0);
            acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[j], qhi[1][kc], acc[b][1], 0, 0, 0);
            acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qlo[0][kc], acc[b][0], 0, 0, 0);
            acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qlo[1][kc], acc[b][1], 0, 0, 0);
        }
        acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qhi[0][kc], acc[b][0], 0, 0, 0);
        acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qhi[1][kc], acc[b][1], 0, 0, 0);
        // keep this order in the schedule: the reads for block j + PF, then the MFMAs of block j
        if (j + PF < NJ) __builtin_amdgcn_sched_group_barrier(0x100, THREE ? 2 : 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, THREE ? 6 : 2, 0);
    }
}

// The chunk loop of one level over NCMAX chunks starting at kc0.  Units 0 .. pre-1 were issued
// by the caller (before the previous level's epilogue); the rest of the ring is filled here.
template <int LVL, bool THREE, int U>
struct KSteps {
    using G = Geo<LVL, THREE>;
    using RG = Ring<LVL, THREE>;
    __device__ static __forceinline__ void fill(const BlockArgs& a, const ItemCtx& c,
                                                const int (&voff)[G::NG][G::ITERS], int kc0, int pre) {
        if constexpr (U < RG::NS) {
            if (U >= pre) issue_unit<LVL, THREE, U>(a, c, voff, kc0);
            KSteps<LVL, THREE, U + 1>::fill(a, c, voff, kc0, pre);
        }
    }
    __device__ static __forceinline__ void run(const BlockArgs& a, const ItemCtx& c, const unsigned char* smem,
                                               const int (&voff)[G::NG][G::ITERS], int kc0,
                                               const bf16x8 (&qhi)[2][NCMAX], const bf16x8 (&qlo)[2][NCMAX],
                                               f32x4 (&acc)[G::NB][2], int frag_hi, int frag_lo, bool active) {
        if constexpr (U < G::NU) {
            wait_vm<G::ITERS * RG::younger(U)>();
            __syncthreads();                     // unit U is in LDS for everyone; everyone is done with unit U - 1
            if constexpr (U >= 1 && U - 1 + RG::NS < G::NU) issue_unit<LVL, THREE, U - 1 + RG::NS>(a, c, voff, kc0);
            if (active && kc0 + U / G::NG < a.NC)
                mfma_unit<LVL, THREE, U>(c, smem, qhi, qlo, acc, frag_hi, frag_lo);
            KSteps<LVL, THREE, U + 1>::run(a, c, smem, voff, kc0, qhi, qlo, acc, frag_hi, frag_lo, active);
        }
    }
};

// The taps of level LVL for column block h of every wave (64 queries of the item), from that
// level's S rows in LDS ([point][64 columns]).  lane = column; wave 0 takes tap columns (x offsets) 0..2, waves 1..3 two
// columns each.  A footprint column is read from LDS once (all 2r+2 rows at once, so the reads
// overlap) and serves as the right neighbour of one tap column and the left neighbour of the next.
template <int LVL, bool THREE, bool NHWC>
__device__ __forceinline__ void write_taps(const BlockArgs& a, const ItemCtx& c, const float* S, int h) {
    using G = Geo<LVL, THREE>;
    // channels-last output: the tap stride is the constant 1, so that the compiler can merge a
    // query's consecutive taps into wide stores
    const size_t tap_stride = NHWC ? 1 : (size_t)a.tap_stride;
    float* o_lvl = a.out + (size_t)c.b * a.L * KK * a.HW + (size_t)(LVL * KK) * tap_stride;
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    const int q = (c.lane >> 4) * QW + h * 16 + (c.lane & 15), wave = c.wave;   // S column lane -> query slot
    if (q < c.n) {
        const float inv = __uint_as_float((uint32_t)(127 - LVL) << 23);   // 2^-LVL
        const float cxl = c.q_cx[q] * inv, cyl = c.q_cy[q] * inv;
        const float flx = floorf(cxl), fly = floorf(cyl);
        const float fx = cxl - flx, fy = cyl - fly;
        const int rx = (int)flx - R - xs, ry = (int)fly - R - ys;         // in [0, CXL) x [0, CYL)
        // K = 9: columns 0..3, 3..5, 5..7, 7..9; otherwise an even split
        const int i0 = K == 9 ? (wave == 0 ? 0 : 2 * wave + 1) : wave * K / NW;
        const int i1 = K == 9 ? 2 * wave + 3 : (wave + 1) * K / NW;
        const float* s = S + (ry * G::WSX + rx + i0) * 64 + c.lane;
        float* o = o_lvl + (size_t)c.q_pix[q] * a.pix_stride + (size_t)(i0 * K) * tap_stride;
        float left[K + 1], right[K + 1];
#pragma unroll
        for (int j = 0; j <= K; ++j) left[j] = s[j * G::WSX * 64];
        for (int i = i0; i < i1; ++i) {
            s += 64;
#pragma unroll
            for (int j = 0; j <= K; ++j) right[j] = s[j * G::WSX * 64];
            float hprev = left[0] + fx * (right[0] - left[0]);
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const float hcur = left[j + 1] + fx * (right[j + 1] - left[j + 1]);
                o[(size_t)j * tap_stride] = (hprev + fy * (hcur - hprev)) * a.scale;    // 1/sqrt(D), once per tap
                hprev = hcur;
            }
#pragma unroll
            for (int j = 0; j <= K; ++j) left[j] = right[j];
            o += (size_t)K * tap_stride;
        }
    }
}

// All taps of level LVL are zero for this item (its window is all padding).
template <int LVL, bool NHWC>
__device__ __forceinline__ void write_zero_taps(const BlockArgs& a, const ItemCtx& c) {
    const size_t tap_stride = NHWC ? 1 : (size_t)a.tap_stride;
    float* o_lvl = a.out + (size_t)c.b * a.L * KK * a.HW + (size_t)(LVL * KK) * tap_stride;
    for (int q = c.lane; q < c.n; q += 64) {
        float* o = o_lvl + (size_t)c.q_pix[q] * a.pix_stride;
        for (int t = c.wave; t < KK; t += NW) o[(size_t)t * tap_stride] = 0.f;
    }
}

// Per-level staging plan; the next level's is made (and its first units issued) before the
// current level's epilogue.
template <int LVL, bool THREE>
struct Plan {
    int voff[Geo<LVL, THREE>::NG][Geo<LVL, THREE>::ITERS];
    bool touches;       // the window reaches into the level (uniform); otherwise all taps are zero
    int pre;            // units already issued
};

// issue units 0 .. PRE-1 of level LVL (the slots above the running epilogue's S)
template <int LVL, bool THREE, int U = 0>
__device__ __forceinline__ void prefetch_units(const BlockArgs& a, const ItemCtx& c, Plan<LVL, THREE>& pl) {
    using RG = Ring<LVL, THREE>;
    if constexpr (U < RG::PRE) {
        issue_unit<LVL, THREE, U>(a, c, pl.voff, 0);
        prefetch_units<LVL, THREE, U + 1>(a, c, pl);
    }
}

template <int LVL, bool THREE>
__device__ __forceinline__ void begin_level(const BlockArgs& a, const ItemCtx& c, Plan<LVL, THREE>& pl) {
    pl.pre = 0;
    pl.touches = LVL < a.L && window_touches<LVL, THREE>(a, c);
    if (pl.touches) {
        plan<LVL, THREE>(a, c, pl.voff);
        prefetch_units<LVL, THREE>(a, c, pl);
        pl.pre = Ring<LVL, THREE>::PRE;
    }
}

// One level of one work item.  On entry `pl` holds the staging plan and units 0 .. pl.pre-1 are
// in flight; before its own epilogue the level plans the next one and issues its first units.
template <int LVL, bool THREE, bool BIGD, bool NHWC, class NextPlan>
__device__ __forceinline__ void level_pass(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                           bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX],
                                           Plan<LVL, THREE>& pl, NextPlan& nx) {
    using G = Geo<LVL, THREE>;
    float* S = reinterpret_cast<float*>(smem);               // [ROWS][64], aliases the ring
    const int lane = c.lane, wave = c.wave;
    auto begin_next = [&]() {
        if constexpr (LVL + 1 < CORR_MAX_L) begin_level<LVL + 1, THREE>(a, c, nx);
    };
    if (!pl.touches) {                                       // uniform: a window that is all padding gives zero taps
        begin_next();
        write_zero_taps<LVL, NHWC>(a, c);
        return;
    }

    f32x4 acc[G::NB][2];
#pragma unroll
    for (int i = 0; i < G::NB; ++i) { acc[i][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[i][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }

    const bool active = wave * QW < c.n;                     // this wave has queries
    // fragment read: lane holds channels 8*(lane/16)..+7 of row 16*j + lane%16 of a slot
    const int fr = lane & 15, fk = lane >> 4;
    const int frag_hi = fr * G::ROWB + ((fk ^ G::swz(fr)) << 4);
    const int frag_lo = fr * G::ROWB + (((4 + fk) ^ G::swz(fr)) << 4);

    for (int kc0 = 0; kc0 < (BIGD ? a.NC : 1); kc0 += NCMAX) {
        if (BIGD && (kc0 > 0 || LVL > 0)) load_queries<THREE>(a, c, kc0, qhi, qlo);
        KSteps<LVL, THREE, 0>::fill(a, c, pl.voff, kc0, kc0 == 0 ? pl.pre : 0);
        KSteps<LVL, THREE, 0>::run(a, c, smem, pl.voff, kc0, qhi, qlo, acc, frag_hi, frag_lo, active);
        __syncthreads();                                     // every wave is done with the ring
    }
    TRACE(2 + 2 * LVL);
    begin_next();                                            // loads into the slots above S fly under the tap writes

    // lane holds queries 32*wave + 16*h + lane % 16, points 4*(lane/16)+v of every row block.
    // Round h of the epilogue takes column block h of every wave: S column 16*wave + lane%16.
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h * 16 < c.n) {                                  // uniform
            if (active) {
#pragma unroll
                for (int b = 0; b < G::NB; ++b)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        S[(b * 16 + 4 * (lane >> 4) + v) * 64 + wave * 16 + (lane & 15)] = acc[b][h][v];
            }
            __syncthreads();
            write_taps<LVL, THREE, NHWC>(a, c, S, h);
            __syncthreads();                                 // S is dead
        }
    }
    TRACE(3 + 2 * LVL);
}

template <bool THREE, bool BIGD, bool NHWC>
__global__ __launch_bounds__(NT, 1) void block_kernel(BlockArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    int* q_pix = reinterpret_cast<int*>(smem + LDS_DATA);
    float* q_cx = reinterpret_cast<float*>(q_pix + CORR_GROUP);
    float* q_cy = q_cx + CORR_GROUP;

    // XCD-aware item choice: workgroup w runs on XCD w % 8.  Items are dealt to the XCDs in runs
    // of XCD_RUN consecutive items (neighbouring cells share window rows and columns, so they
    // should share an L2), round robin, so that cheap border regions do not all land on the same
    // XCD.  The grid is a multiple of 8 * XCD_RUN, so every item index is produced exactly once.
    const int n_items = *a.n_items;
    const int j = blockIdx.x >> 3;
    const int k = ((j / XCD_RUN) * 8 + (blockIdx.x & 7)) * XCD_RUN + j % XCD_RUN;
    if (k >= n_items) return;
    const int4 item = a.items[k];
    ItemCtx c;
    c.item = k;
    c.tid = threadIdx.x; c.lane = c.tid & 63; c.wave = c.tid >> 6;
    c.n = item.z;
    corr_cell_coords(a.g, item.x, &c.b, &c.u, &c.v);
    c.u += a.g.u_min; c.v += a.g.v_min;
    c.q_pix = q_pix; c.q_cx = q_cx; c.q_cy = q_cy;
    c.lds_wave = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + c.wave * 1024);
#ifdef CORR_DEBUG_SYNC_STAGE
    c.dbg_smem = smem;
#endif
    const uint64_t base = reinterpret_cast<uint64_t>(a.f2s);
    c.rsrc[0] = (int)(uint32_t)base; c.rsrc[1] = (int)((base >> 32) & 0xffffu);
    // the range check covers voffset + soffset, so the resource spans all chunk planes
    c.rsrc[2] = (int)(a.f2_plane_bytes * (unsigned)a.NC); c.rsrc[3] = 0x00020000;
    c.rsrc_null = c.rsrc; c.rsrc_null[2] = 0;

    TRACE(0);
    // level 0's first units start to move before anything else
    Plan<0, THREE> p0;
    begin_level<0, THREE>(a, c, p0);

    if (c.tid < CORR_GROUP) {
        int pix = -1;
        float cx = 0.f, cy = 0.f;
        if (c.tid < c.n) {
            pix = a.perm[item.y + c.tid] - c.b * a.HW;
            cx = a.coords[((size_t)c.b * 2 + 0) * a.HW + pix];
            cy = a.coords[((size_t)c.b * 2 + 1) * a.HW + pix];
        }
        q_pix[c.tid] = pix; q_cx[c.tid] = cx; q_cy[c.tid] = cy;
    }
    __syncthreads();

    bf16x8 qhi[2][NCMAX], qlo[2][NCMAX];
    load_queries<THREE>(a, c, 0, qhi, qlo);
    TRACE(1);

    Plan<1, THREE> p1;
    Plan<2, THREE> p2;
    Plan<3, THREE> p3;
    level_pass<0, THREE, BIGD, NHWC>(a, c, smem, qhi, qlo, p0, p1);
    if (a.L > 1) level_pass<1, THREE, BIGD, NHWC>(a, c, smem, qhi, qlo, p1, p2);
    if (a.L > 2) level_pass<2, THREE, BIGD, NHWC>(a, c, smem, qhi, qlo, p2, p3);
    if (a.L > 3) level_pass<3, THREE, BIGD, NHWC>(a, c, smem, qhi, qlo, p3, p3);
}

template <bool THREE, bool BIGD, bool NHWC>
hipError_t launch_items(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    auto kfn = block_kernel<THREE, BIGD, NHWC>;
    // once per instantiation and process (initialisation of a local static is thread-safe)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    BlockArgs a;
    a.f1s = p->f1_split; a.f2s = p->f2_split; a.coords = q.coords; a.perm = ws.perm; a.items = ws.items;
    a.n_items = ws.n_items; a.out = q.out; a.B = p->B; a.HW = p->H * p->W; a.NC = p->D / CORR_CHUNK; a.L = p->L;
    a.tap_stride = corr_tap_stride(p, q); a.pix_stride = corr_pix_stride(p, q);
    a.g = p->grid;
    for (int l = 0; l < CORR_MAX_L; ++l) { a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l]; a.pix_base[l] = p->f2_pix_base[l]; }
    a.rec = (!THREE && (p->built & CORR_REP_BF16)) ? 32 : 64;      // bf16 mode prefers the hi-only records
    if (a.rec == 32) { a.f1s = p->f1_hi; a.f2s = p->f2_hi; }
    a.f1_stride = p->B * p->H * p->W * a.rec;
    a.f2_plane_bytes = (unsigned)((size_t)p->f2_pix_total * a.rec * 2);
    a.scale = 1.0f / sqrtf((float)p->D);
#ifdef CORR_TRACE
    a.trace = g_corr_trace;
#endif
    const int grid = (ws.max_items + 8 * XCD_RUN - 1) / (8 * XCD_RUN) * (8 * XCD_RUN);
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace

#if defined(CORR_TRACE) && CORR_BLOCK_R == 4
long long* g_corr_trace = nullptr;
extern "C" void corr_debug_set_trace(long long* p) { g_corr_trace = p; }
#endif

hipError_t CORR_CAT(launch_block_r, CORR_BLOCK_R)(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    const bool big = p->D > CORR_BLOCK_MAX_D, three = q.prec != CORR_PREC_BF16;
#define CORR_LAUNCH(NHWC)                                                                                    \
    (three ? (big ? launch_items<true, true, NHWC>(p, ws, q, s) : launch_items<true, false, NHWC>(p, ws, q, s))   \
           : (big ? launch_items<false, true, NHWC>(p, ws, q, s) : launch_items<false, false, NHWC>(p, ws, q, s)))
    return q.nhwc ? CORR_LAUNCH(true) : CORR_LAUNCH(false);
#undef CORR_LAUNCH
}
