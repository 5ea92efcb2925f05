// Per-lookup compute (paper: steps b and c, "Sparse Correlation Volume
// Computation" and "Sparse Volume Sampling"; fused as in "Fused Implementation":
// the computed block lives only in registers and LDS).
//
// One workgroup (4 waves, the only one on its CU) = one work item = (target cell of 16 x 8
// level-0 pixels, up to 128 of its queries), processed level after level.  Wave w owns queries
// 16w .. 16w+15 and 64+16w .. 64+16w+15 of the item as two MFMA column blocks (items of up to 64
// queries use one).
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
constexpr int NCMAX = CORR_BLOCK_MAX_D / CORR_CHUNK;   // chunks of query fragments a wave holds
constexpr int LDS_BYTES = 160 * 1024;
constexpr int META_BYTES = CORR_GROUP * 12;
constexpr int LDS_DATA = LDS_BYTES - META_BYTES;       // ring slots and S
constexpr int OOB = (int)0x80000000u;                  // a buffer offset beyond any chunk plane (each is below 2 GiB): loads zeros
static_assert(CORR_GROUP == 128 && NW == 4, "a wave owns two 16-query column blocks");

struct BlockArgs {
    const uint16_t* f1s;                 // [NC][B*HW][rec]
    const uint16_t* f2s;                 // [NC][P][rec], P = pixels of all levels; level l starts at pix_base[l]
    const int* perm;                     // queries sorted by (cell, source row mod 8)
    const float2* sorted_c;              // their coordinates
    const int4* items;
    const int* n_items;
    const int* q_bin;                    // [B*HW] bin of every query, -1: no bin (out of range at every level)
    float* out;
    int B, HW, NC, L;
    int tap_stride, pix_stride;          // layout of out
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L], pix_base[CORR_MAX_L];
    int f1_stride;                       // elements between chunk planes of f1s
    unsigned f2_plane_bytes;             // bytes of one chunk plane of f2s
    int rec;                             // elements per pixel record: 64 (hi + lo) or 32 (hi only)
    CellGrid g;
    float scale;
    int force_ways;                      // block_level_kernel: 0 = decide from the item count, else 2 or 4
#ifdef CORR_TRACE
    long long* trace;                    // [items][16] timestamps (debug builds)
#endif
};

// S rows are 64 queries + 4 floats of padding: the four row groups a wave writes at once then fall in
// different banks, and a row read by 64 lanes still covers every bank once
constexpr int SST = 68;                                // floats between S rows; 3 * SST < 256: a two-address LDS write reaches rows +1..+3
#ifndef CORR_LDS_PF
#define CORR_LDS_PF 3
#endif
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
    static constexpr int S_BYTES = ROWS * SST * 4;        // S of one epilogue round: [ROWS][64 queries] fp32
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
    static constexpr int NS = NS0;
    static constexpr int PRE = cmin(UP, NS);              // units that can be issued before the previous epilogue
    static_assert(NS >= 3, "ring too small");
    static_assert(G::S_BYTES <= LDS_DATA, "S does not fit");
    __device__ static constexpr int slot_off(int i) { return i < PRE ? SPREV + i * G::SLOT : (i - PRE) * G::SLOT; }
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
    unsigned lds_base;       // LDS byte address of smem
    unsigned lds_wave;       // LDS byte address of smem + wave * 1024 (uniform)
    i32x4 rsrc;              // buffer resource: chunk plane 0 of f2s (each load rebases it to its own plane)
};

// 16 bytes per lane from a buffer straight into LDS at lds_base + lane * 16.  A lane whose
// voffset lies beyond the resource's size writes zeros (measured on gfx950).
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned lds_base, int voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory");
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

// issue loads it0 .. it1-1 of unit U (chunk kc0 + U / NG, group U % NG) into its ring slot
template <int LVL, bool THREE, int U>
__device__ __forceinline__ void issue_unit(const BlockArgs& a, const ItemCtx& c,
                                           const int (&voff)[Geo<LVL, THREE>::NG][Geo<LVL, THREE>::ITERS], int kc0,
                                           int it0 = 0, int it1 = Geo<LVL, THREE>::ITERS) {
    using G = Geo<LVL, THREE>;
    using RG = Ring<LVL, THREE>;
    constexpr int g = U % G::NG, slot = U % RG::NS;
    const int kc = kc0 + U / G::NG;
    const bool real = kc < a.NC;                                  // uniform
    // The resource covers this chunk's plane alone (a plane is below 2 GiB, all planes together need not
    // be); a chunk past the last one reads an empty buffer (zeros).  readfirstlane keeps the operands scalar.
    const uint64_t pb = ((uint64_t)(uint32_t)c.rsrc[1] << 32 | (uint32_t)c.rsrc[0]) + (uint64_t)(real ? kc : 0) * a.f2_plane_bytes;
    i32x4 rs;
    rs[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)pb);
    rs[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(pb >> 32));
    rs[2] = __builtin_amdgcn_readfirstlane(real ? c.rsrc[2] : 0);
    rs[3] = __builtin_amdgcn_readfirstlane(c.rsrc[3]);
#pragma unroll
    for (int it = 0; it < G::ITERS; ++it)
        if (it >= it0 && it < it1)                                // constants once the callers' loops are unrolled
            dma16(rs, c.lds_wave + RG::slot_off(slot) + it * 4096, voff[g][it]);
}

// Query fragments of this wave for chunks kc0 .. kc0+NCMAX-1: lane holds channels 8*(lane/16) .. +7 of
// every chunk of queries 64*h + 16*wave + lane%16, h = 0, 1 (the B operands of the MFMA).
template <bool THREE>
__device__ __forceinline__ void load_queries(const BlockArgs& a, const ItemCtx& c, int kc0,
                                             bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX]) {
    const char* base = reinterpret_cast<const char*>(a.f1s);          // uniform; byte offsets fit 32 bits
    const unsigned plane = (unsigned)a.f1_stride * 2u;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pix = c.q_pix[h * 64 + c.wave * 16 + (c.lane & 15)];
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

// The chunk loop of one level over NCMAX chunks starting at kc0, software-pipelined across units.
// Units 0 .. pre-1 were issued by the caller (before the previous level's epilogue); the rest of
// the ring is filled here.  Step U multiplies the row blocks of unit U with this wave's query
// column blocks.  Half way through it the wave waits for unit U + 1 and meets the others at the one
// barrier of the step (so everyone is also done with unit U - 1, whose slot is then refilled with
// unit U - 1 + NS, a few loads at a time between the row blocks), and its last row blocks already
// read the first fragments of unit U + 1: the matrix pipe never waits for a barrier or for the
// first LDS reads of a unit.  There is no branch in the loop: a wave without queries, or a chunk past
// the last one (loaded as zeros), multiplies anyway; a branch here makes the compiler move every
// accumulator between register files around it.  The fragment reads run PF row blocks ahead of their
// MFMAs; a sched_barrier after every row block pins that distance (left alone, the scheduler sinks each
// read to just before its use, or hoists them all and spills).
template <int LVL, bool THREE, bool TWO>
struct KLoop {
    using G = Geo<LVL, THREE>;
    using RG = Ring<LVL, THREE>;
    // row blocks whose fragments are in flight ahead of the MFMAs: a lone wave per SIMD needs this many
    // LDS reads outstanding to keep the LDS pipe, and with it the matrix pipe, busy
    static constexpr int PF = cmin(CORR_LDS_PF, cmax(1, G::NB / G::NG));
    static_assert(RG::NS >= 3, "the pipelined loop refills a slot one step after it waits for the next unit");
    struct Frags { bf16x8 h[PF], l[PF]; };
    using Voff = const int (&)[G::NG][G::ITERS];
    using Acc = f32x4 (&)[G::NB][TWO ? 2 : 1];
    using QF = const bf16x8 (&)[2][NCMAX];

    static constexpr int nj(int u) { return (G::NB - u % G::NG + G::NG - 1) / G::NG; }   // row blocks of unit u
    // loads that may still be in flight behind unit u + 1 when step u waits for it
    static constexpr int younger(int u) { return cmin(G::NU - 1, RG::NS - 1 + cmax(u - 1, 0)) - (u + 1); }

    template <int U>
    __device__ static __forceinline__ void fill(const BlockArgs& a, const ItemCtx& c, Voff voff, int kc0, int pre) {
        if constexpr (U < RG::NS) {
            if (U >= pre) issue_unit<LVL, THREE, U>(a, c, voff, kc0);
            fill<U + 1>(a, c, voff, kc0, pre);
        }
    }
    // fragment of row block j of unit U: lane holds channels 8*(lane/16)..+7 of row 16*j + lane%16
    template <int U>
    __device__ static __forceinline__ void read_frag(const unsigned char* smem, int j, int frag_hi, int frag_lo,
                                                     bf16x8& h, bf16x8& l) {
        const unsigned char* rows = smem + RG::slot_off(U % RG::NS) + j * 16 * G::ROWB;
        h = *reinterpret_cast<const bf16x8*>(rows + frag_hi);
        if (THREE) l = *reinterpret_cast<const bf16x8*>(rows + frag_lo);
    }

    template <int U>
    __device__ static __forceinline__ void step(const BlockArgs& a, const ItemCtx& c, const unsigned char* smem,
                                                Voff voff, int kc0, QF qhi, QF qlo, Acc acc,
                                                int frag_hi, int frag_lo, Frags& f) {
        if constexpr (U < G::NU) {
            constexpr int g = U % G::NG, kc = U / G::NG;
            constexpr int NJ = nj(U);
            constexpr int JS = cmax(0, cmin(NJ / 2, NJ - PF));           // row block before which the step synchronises
            constexpr bool HAS_NEXT = U + 1 < G::NU;
            constexpr int IU = (U >= 1 && U - 1 + RG::NS < G::NU) ? U - 1 + RG::NS : -1;
            static_assert(NJ >= PF, "a unit holds at least PF row blocks");
            Frags nf;
            {
                bf16x8 wh[NJ + PF], wl[NJ + PF];
#pragma unroll
                for (int j = 0; j < PF; ++j) { wh[j] = f.h[j]; wl[j] = f.l[j]; }
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int b = j * G::NG + g;
                    if (j == JS && HAS_NEXT) {
                        wait_vm<G::ITERS * (HAS_NEXT ? younger(U) : 0)>();
                        __syncthreads();         // unit U + 1 is in LDS for everyone; everyone is done with unit U - 1
                    }
                    if (j + PF < NJ) read_frag<U>(smem, j + PF, frag_hi, frag_lo, wh[j + PF], wl[j + PF]);
                    else if (HAS_NEXT) read_frag<(HAS_NEXT ? U + 1 : U)>(smem, j + PF - NJ, frag_hi, frag_lo, wh[j + PF], wl[j + PF]);
                    if (THREE) {
                        acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[j], qhi[0][kc], acc[b][0], 0, 0, 0);
                        if (TWO) acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[j], qhi[1][kc], acc[b][1], 0, 0, 0);
                        acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qlo[0][kc], acc[b][0], 0, 0, 0);
                        if (TWO) acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qlo[1][kc], acc[b][1], 0, 0, 0);
                    }
                    acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qhi[0][kc], acc[b][0], 0, 0, 0);
                    if (TWO) acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[j], qhi[1][kc], acc[b][1], 0, 0, 0);
                    // nothing moves across this point: the reads for block j + PF stay PF blocks ahead of their use
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (IU >= 0)
                        if (j >= JS)
                            issue_unit<LVL, THREE, (IU >= 0 ? IU : 0)>(a, c, voff, kc0, (j - JS) * G::ITERS / (NJ - JS),
                                                                       (j - JS + 1) * G::ITERS / (NJ - JS));
                }
#pragma unroll
                for (int j = 0; j < PF; ++j) { nf.h[j] = wh[NJ + j]; nf.l[j] = wl[NJ + j]; }
            }
            step<U + 1>(a, c, smem, voff, kc0, qhi, qlo, acc, frag_hi, frag_lo, nf);
        }
    }

    __device__ static __forceinline__ void run(const BlockArgs& a, const ItemCtx& c, const unsigned char* smem,
                                               Voff voff, int kc0, int pre, QF qhi, QF qlo, Acc acc,
                                               int frag_hi, int frag_lo) {
        fill<0>(a, c, voff, kc0, pre);
        wait_vm<G::ITERS * (RG::NS - 1)>();
        __syncthreads();                                                 // unit 0 is in LDS for everyone
        Frags f;
#pragma unroll
        for (int j = 0; j < PF; ++j) read_frag<0>(smem, j, frag_hi, frag_lo, f.h[j], f.l[j]);
        step<0>(a, c, smem, voff, kc0, qhi, qlo, acc, frag_hi, frag_lo, f);
        __syncthreads();                                                 // every wave is done with the ring
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
    // NCHW: taps leave through a buffer resource over this level's KK planes of this batch item (below
    // 2 GiB): the lane's pixel is the vector offset, the tap's plane a scalar offset, no address arithmetic
    __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(o_lvl, 0, 0x7fffffff, 0x00020000);
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    const int q = h * 64 + c.lane, wave = c.wave;           // S column = lane
    if (q < c.n) {
        const float inv = __uint_as_float((uint32_t)(127 - LVL) << 23);   // 2^-LVL
        const float cxl = c.q_cx[q] * inv, cyl = c.q_cy[q] * inv;
        const float flx = floorf(cxl), fly = floorf(cyl);
        const float fx = cxl - flx, fy = cyl - fly;
        // horizontal weights carry the 1/sqrt(D) scale: tap = lerp_y(lerp_x) costs four operations
        const float wr = fx * a.scale, wl = a.scale - wr;
        const int rx = (int)flx - R - xs, ry = (int)fly - R - ys;         // in [0, CXL) x [0, CYL)
        // K = 9: columns 0..3, 3..5, 5..7, 7..9; otherwise an even split
        const int i0 = K == 9 ? (wave == 0 ? 0 : 2 * wave + 1) : wave * K / NW;
        const int i1 = K == 9 ? 2 * wave + 3 : (wave + 1) * K / NW;
        const float* s = S + (ry * G::WSX + rx + i0) * SST + c.lane;
        const int pix = c.q_pix[q];
        float* o = o_lvl + (size_t)pix * a.pix_stride + (size_t)(i0 * K) * tap_stride;
        int plane = i0 * K * a.tap_stride * 4;                            // NCHW: byte offset of tap (i, 0)'s plane (uniform)
        float left[K + 1], right[K + 1];
#pragma unroll
        for (int j = 0; j <= K; ++j) left[j] = s[j * G::WSX * SST] * wl;
        for (int i = i0; i < i1; ++i) {
            s += SST;
#pragma unroll
            for (int j = 0; j <= K; ++j) right[j] = s[j * G::WSX * SST];
            float hprev = left[0] + wr * right[0];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const float hcur = left[j + 1] + wr * right[j + 1];
                const float v = hprev + fy * (hcur - hprev);
#ifdef CORR_DEBUG_NOSTORE
                if (a.scale == 12345.f)
#endif
                {
                    if constexpr (NHWC) o[j] = v;
                    else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), orsrc, pix * 4, plane + j * a.tap_stride * 4, 0);
                }
                hprev = hcur;
            }
#pragma unroll
            for (int j = 0; j <= K; ++j) left[j] = right[j] * wl;
            o += K;
            plane += K * a.tap_stride * 4;
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

// issue units U .. U1-1 of level LVL
template <int LVL, bool THREE, int U, int U1>
__device__ __forceinline__ void issue_units(const BlockArgs& a, const ItemCtx& c, Plan<LVL, THREE>& pl) {
    if constexpr (U < U1) {
        issue_unit<LVL, THREE, U>(a, c, pl.voff, 0);
        issue_units<LVL, THREE, U + 1, U1>(a, c, pl);
    }
}

// Plan level LVL and issue its units 0 .. PRE-1 (the slots above the running epilogue's S).
template <int LVL, bool THREE>
__device__ __forceinline__ void begin_level(const BlockArgs& a, const ItemCtx& c, Plan<LVL, THREE>& pl) {
    pl.pre = 0;
    pl.touches = LVL < a.L && window_touches<LVL, THREE>(a, c);
    if (pl.touches) {
        plan<LVL, THREE>(a, c, pl.voff);
        issue_units<LVL, THREE, 0, Ring<LVL, THREE>::PRE>(a, c, pl);
        pl.pre = Ring<LVL, THREE>::PRE;
    }
}

// One level of one work item.  On entry `pl` holds the staging plan and units 0 .. pl.pre-1 are
// in flight; before its own epilogue the level plans the next one and issues its first units.
template <int LVL, bool THREE, bool BIGD, bool NHWC, bool TWO, class NextPlan, bool NEXT = true>
__device__ __forceinline__ void level_pass(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                           bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX],
                                           Plan<LVL, THREE>& pl, NextPlan& nx) {
    using G = Geo<LVL, THREE>;
    float* S = reinterpret_cast<float*>(smem);               // [ROWS][64], aliases the ring
    const int lane = c.lane, wave = c.wave;
    auto begin_next = [&]() {
        if constexpr (NEXT && LVL + 1 < CORR_MAX_L) begin_level<LVL + 1, THREE>(a, c, nx);
    };
    if (!pl.touches) {                                       // uniform: a window that is all padding gives zero taps
        begin_next();
        write_zero_taps<LVL, NHWC>(a, c);
        return;
    }

    constexpr int NH = TWO ? 2 : 1;                          // column blocks per wave
    f32x4 acc[G::NB][NH];
#pragma unroll
    for (int i = 0; i < G::NB; ++i)
#pragma unroll
        for (int h = 0; h < NH; ++h) acc[i][h] = f32x4{0.f, 0.f, 0.f, 0.f};

    // fragment read: lane holds channels 8*(lane/16)..+7 of row 16*j + lane%16 of a slot
    const int fr = lane & 15, fk = lane >> 4;
    const int frag_hi = fr * G::ROWB + ((fk ^ G::swz(fr)) << 4);
    const int frag_lo = fr * G::ROWB + (((4 + fk) ^ G::swz(fr)) << 4);

    for (int kc0 = 0; kc0 < (BIGD ? a.NC : 1); kc0 += NCMAX) {
        if (BIGD && (kc0 > 0 || LVL > 0)) load_queries<THREE>(a, c, kc0, qhi, qlo);
        KLoop<LVL, THREE, TWO>::run(a, c, smem, pl.voff, kc0, kc0 == 0 ? pl.pre : 0, qhi, qlo, acc, frag_hi, frag_lo);
    }
    TRACE(2 + 2 * LVL);
    begin_next();                                            // loads into the slots above S fly under the tap writes
    if (LVL == 0) TRACE(10);

    // lane holds queries 64*h + 16*wave + lane % 16, points 4*(lane/16)+v of every row block.
    // Round h of the epilogue takes column block h of every wave: S column 16*wave + lane%16 = query 64*h + column.
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        {
            {
                // straight from the accumulator registers (inline assembly: left to itself the compiler
                // copies every accumulator into ordinary registers first and spills the query fragments)
                unsigned addr = c.lds_base + ((4 * (lane >> 4)) * SST + wave * 16 + (lane & 15)) * 4;
#pragma unroll
                for (int b = 0; b < G::NB; ++b) {
                    // two rows per instruction (offsets in dwords: rows are SST floats apart)
                    asm volatile("ds_write2_b32 %0, %1, %2 offset1:%5\n\tds_write2_b32 %0, %3, %4 offset0:%6 offset1:%7"
                                 :: "v"(addr), "a"(acc[b][h][0]), "a"(acc[b][h][1]), "a"(acc[b][h][2]), "a"(acc[b][h][3]),
                                    "n"(SST), "n"(2 * SST), "n"(3 * SST) : "memory");
                    addr += 16 * SST * 4;
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            __syncthreads();
            if (LVL == 0) TRACE(11 + 2 * h);
            write_taps<LVL, THREE, NHWC>(a, c, S, h);
            if (LVL == 0) TRACE(12 + 2 * h);
            __syncthreads();                                 // S is dead
        }
    }
    TRACE(3 + 2 * LVL);
}

template <bool THREE, bool BIGD, bool NHWC, bool TWO>
__device__ __forceinline__ void run_levels(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                           bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX], Plan<0, THREE>& p0) {
    Plan<1, THREE> p1;
    Plan<2, THREE> p2;
    Plan<3, THREE> p3;
    level_pass<0, THREE, BIGD, NHWC, TWO>(a, c, smem, qhi, qlo, p0, p1);
    if (a.L > 1) level_pass<1, THREE, BIGD, NHWC, TWO>(a, c, smem, qhi, qlo, p1, p2);
    if (a.L > 2) level_pass<2, THREE, BIGD, NHWC, TWO>(a, c, smem, qhi, qlo, p2, p3);
    if (a.L > 3) level_pass<3, THREE, BIGD, NHWC, TWO>(a, c, smem, qhi, qlo, p3, p3);
}

// Part `part` of `parts` of the query range: zeros for every query without a bin.  Lane = query: null
// queries cluster (image borders, regions whose targets lie outside), so neighbouring lanes write neighbouring
// pixels of one tap plane and their stores merge.
__device__ __forceinline__ void zero_null_queries(const BlockArgs& a, int part, int parts) {
    const int BN = a.B * a.HW;
    const int per = (BN + parts - 1) / parts;
    const int q0 = part * per, q1 = min(BN, q0 + per);
    const int taps = a.L * KK;
    for (int i = q0; i < q1; i += NT) {               // the same trip count for every thread
        const int q = i + (int)threadIdx.x;
        if (q < q1 && a.q_bin[q] < 0) {
            const int b = q / a.HW, p = q - b * a.HW;
            float* o = a.out + (size_t)b * taps * a.HW + (size_t)p * a.pix_stride;
            for (int t = 0; t < taps; ++t) o[(size_t)t * a.tap_stride] = 0.0f;
        }
    }
}

// Which item this workgroup takes, or -1 - s when there is none and it is workgroup s of those past the item
// list.  XCD-aware choice (the grid covers the largest possible item count); SPREAD: consecutive items on
// different XCDs instead (workgroup w runs on XCD w % 8): with few items the runs of the XCD-aware choice would
// put them all on one or two XCDs and leave the other compute units idle.
template <bool SPREAD = false>
__device__ __forceinline__ int choose_item(const BlockArgs& a) {
    const int n_items = *a.n_items;
    const int k = SPREAD ? (int)blockIdx.x : corr_item_of_workgroup(blockIdx.x);
    return k < n_items ? k : -1 - (k - n_items);
}
// What a workgroup with an item sets up first: the item's record, the thread's indices, the LDS addresses, the
// buffer resource of the pyramid.
__device__ __forceinline__ void init_item(const BlockArgs& a, unsigned char* smem, int k, ItemCtx& c, int4& item) {
    int* q_pix = reinterpret_cast<int*>(smem + LDS_DATA);
    float* q_cx = reinterpret_cast<float*>(q_pix + CORR_GROUP);
    item = a.items[k];
    c.item = k;
    c.tid = threadIdx.x; c.lane = c.tid & 63;
    // the wave index as a scalar: branches on it must be scalar branches, or the compiler copies every
    // accumulator around each of them
    c.wave = __builtin_amdgcn_readfirstlane(c.tid >> 6);
    c.n = item.z;
    corr_cell_coords(a.g, item.x, &c.b, &c.u, &c.v);
    c.u += a.g.u_min; c.v += a.g.v_min;
    c.q_pix = q_pix; c.q_cx = q_cx; c.q_cy = q_cx + CORR_GROUP;
    c.lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    c.lds_wave = __builtin_amdgcn_readfirstlane(c.lds_base + c.wave * 1024);
    const uint64_t base = reinterpret_cast<uint64_t>(a.f2s);
    c.rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)base);
    c.rsrc[1] = __builtin_amdgcn_readfirstlane((int)((base >> 32) & 0xffffu));
    c.rsrc[2] = __builtin_amdgcn_readfirstlane((int)a.f2_plane_bytes); c.rsrc[3] = 0x00020000;
}
// the item's query records (pixel, x, y) from the sorted list into LDS
__device__ __forceinline__ void load_records(const BlockArgs& a, const ItemCtx& c, const int4& item) {
    if (c.tid < CORR_GROUP) {
        int pix = -1;
        float2 xy = make_float2(0.f, 0.f);
        if (c.tid < c.n) {
            pix = a.perm[item.y + c.tid] - c.b * a.HW;
            xy = a.sorted_c[item.y + c.tid];
        }
        const_cast<int*>(c.q_pix)[c.tid] = pix;
        const_cast<float*>(c.q_cx)[c.tid] = xy.x;
        const_cast<float*>(c.q_cy)[c.tid] = xy.y;
    }
    __syncthreads();
}

template <bool THREE, bool BIGD, bool NHWC>
__global__ __launch_bounds__(NT, 1) void block_kernel(BlockArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int k = choose_item(a);
    if (k < 0) {
        // No item: this workgroup writes zeros instead.  Queries without a bin never reach an item (all their taps
        // are zero); the workgroups past the item list share the query range and zero the ones they find.  They
        // are dispatched last, so the fill runs beside the last items instead of before the first.
        zero_null_queries(a, -1 - k, (int)gridDim.x - *a.n_items);
        return;
    }
    ItemCtx c;
    int4 item;
    init_item(a, smem, k, c, item);

    TRACE(0);
    // level 0's first unit starts to move before anything else
    Plan<0, THREE> p0;
    p0.pre = 0;
    p0.touches = window_touches<0, THREE>(a, c);
    if (p0.touches) { plan<0, THREE>(a, c, p0.voff); issue_units<0, THREE, 0, 1>(a, c, p0); }
    load_records(a, c, item);

    bf16x8 qhi[2][NCMAX], qlo[2][NCMAX];
    load_queries<THREE>(a, c, 0, qhi, qlo);        // ends with a full wait: unit 0 is in as well
    if (p0.touches) { issue_units<0, THREE, 1, Ring<0, THREE>::PRE>(a, c, p0); p0.pre = Ring<0, THREE>::PRE; }
    TRACE(1);

    // items of up to 64 queries fill one column block per wave: half the MFMAs and one epilogue round
    if (c.n > 64) run_levels<THREE, BIGD, NHWC, true>(a, c, smem, qhi, qlo, p0);
    else run_levels<THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, p0);
}

// Small inputs: several workgroups per item, each taking a range of levels (blockIdx.y).  A map of a few
// thousand queries has fewer items than the chip has compute units, and a lookup's time is one item's latency;
// with the levels side by side that latency is the longest range's instead of the sum of all levels.
template <int LVL, int HI, bool THREE, bool BIGD, bool NHWC, bool TWO>
__device__ __forceinline__ void level_chain(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                            bf16x8 (&qhi)[2][NCMAX], bf16x8 (&qlo)[2][NCMAX], Plan<LVL, THREE>& pl) {
    if constexpr (LVL + 1 < HI) {
        Plan<LVL + 1, THREE> nx;                   // planned, and its first units issued, under this level's epilogue
        level_pass<LVL, THREE, BIGD, NHWC, TWO, Plan<LVL + 1, THREE>, true>(a, c, smem, qhi, qlo, pl, nx);
        if (a.L > LVL + 1) level_chain<LVL + 1, HI, THREE, BIGD, NHWC, TWO>(a, c, smem, qhi, qlo, nx);
    } else {
        level_pass<LVL, THREE, BIGD, NHWC, TWO, Plan<LVL, THREE>, false>(a, c, smem, qhi, qlo, pl, pl);
    }
}
template <int LO, int HI, bool THREE, bool BIGD, bool NHWC>
__device__ __forceinline__ void level_range(const BlockArgs& a, const ItemCtx& c, const int4& item, unsigned char* smem) {
    if (LO >= a.L) return;                         // uniform: this pyramid has no such level
    Plan<LO, THREE> pl;
    begin_level<LO, THREE>(a, c, pl);              // the plan and the level's first units, before anything else
    load_records(a, c, item);
    bf16x8 qhi[2][NCMAX], qlo[2][NCMAX];
    load_queries<THREE>(a, c, 0, qhi, qlo);
    if (c.n > 64) level_chain<LO, HI, THREE, BIGD, NHWC, true>(a, c, smem, qhi, qlo, pl);
    else level_chain<LO, HI, THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, pl);
}
// Launched with gridDim.y = CORR_MAX_L.  How many of an item's workgroups work is decided here, from the item
// count the planning pass left: one per level while that many workgroups still fit the chip's compute units
// at once; two (level 0 | the other levels) up to 1.5 items per compute unit, where the finer grain still
// buys more balance than the second start costs (measured: 372 items 99 -> 90 us); else one that runs all
// levels.  The others exit.
template <bool THREE, bool BIGD, bool NHWC>
__global__ __launch_bounds__(NT, 1) void block_level_kernel(BlockArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int k = choose_item<true>(a);
    if (k < 0) {
        if (blockIdx.y == 0) zero_null_queries(a, -1 - k, (int)gridDim.x - *a.n_items);      // as in block_kernel
        return;
    }
    ItemCtx c;
    int4 item;
    init_item(a, smem, k, c, item);
    const int n_items = *a.n_items;
    const int ways = a.force_ways ? a.force_ways : CORR_MAX_L * n_items <= CORR_NUM_CU ? CORR_MAX_L : 2 * n_items <= 3 * CORR_NUM_CU ? 2 : 1;
    const int y = blockIdx.y;                      // uniform, like everything above
    if (y >= ways) return;
    if (ways == 1) {
        level_range<0, CORR_MAX_L, THREE, BIGD, NHWC>(a, c, item, smem);
    } else if (ways == 2) {
        if (y == 0) level_range<0, 1, THREE, BIGD, NHWC>(a, c, item, smem);
        else level_range<1, CORR_MAX_L, THREE, BIGD, NHWC>(a, c, item, smem);
    } else {
        switch (y) {
            case 0: level_range<0, 1, THREE, BIGD, NHWC>(a, c, item, smem); break;
            case 1: level_range<1, 2, THREE, BIGD, NHWC>(a, c, item, smem); break;
            case 2: level_range<2, 3, THREE, BIGD, NHWC>(a, c, item, smem); break;
            default: level_range<3, 4, THREE, BIGD, NHWC>(a, c, item, smem); break;
        }
    }
}

template <bool THREE, bool BIGD, bool NHWC>
hipError_t launch_items(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    auto kfn = block_kernel<THREE, BIGD, NHWC>;
    auto kfn_levels = block_level_kernel<THREE, BIGD, NHWC>;
    // once per instantiation and process (initialisation of a local static is thread-safe)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    static const hipError_t attr_levels = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn_levels),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    if (attr_levels != hipSuccess) return attr_levels;
    BlockArgs a;
    a.f1s = p->f1_split; a.f2s = p->f2_split; a.perm = ws.perm; a.sorted_c = ws.sorted_c; a.items = ws.items;
    a.n_items = ws.n_items; a.q_bin = ws.q_bin; a.out = q.out; a.B = p->B; a.HW = p->H * p->W; a.NC = p->D / CORR_CHUNK; a.L = p->L;
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
    const int grid = corr_block_grid(ws.max_items);
    // Small inputs may have fewer items than the chip has compute units; then the levels of an item run side by
    // side in workgroups of their own.  The kernel that can do that is launched up to split_levels_max queries
    // and decides from the item count (negative settings are test settings: -2 / -4 = always 2 / 4 ways).
    const long long BN = (long long)p->B * p->H * p->W, lim = q.split_levels_max;
    a.force_ways = lim == -2 ? 2 : lim == -4 ? CORR_MAX_L : 0;
    if (BN <= lim || a.force_ways) hipLaunchKernelGGL(kfn_levels, dim3(grid, CORR_MAX_L), dim3(NT), LDS_BYTES, s, a);
    else hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), LDS_BYTES, s, a);
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
