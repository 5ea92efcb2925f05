// Per-lookup compute (paper: steps b and c, "Sparse Correlation Volume
// Computation" and "Sparse Volume Sampling"; fused as in "Fused Implementation":
// the computed block lives only in registers and LDS).
//
// One workgroup = one work item = (target cell, up to 64 of its queries), processed
// level after level by four waves (the two coarsest of four levels in one fused pass).  Wave w owns queries 16w .. 16w+15 of the item.
//   queries     : each wave loads the bf16 hi (and lo) fragments of its 16 queries for all
//                 D channels once per item, straight from global memory into the MFMA
//                 B-operand layout, and keeps them in registers for all levels (D <= 256; a
//                 larger D runs in groups of 256 channels with the fragments reloaded).
//   contraction : S_l[pt][q] = <f2_l(window point pt), f1(query q)> over D.  The window is
//                 staged through LDS in 32-channel chunks (coalesced 16-byte loads of
//                 128-byte records per pixel and chunk; bf16 mode loads only the hi half);
//                 two LDS buffers alternate, one barrier per chunk, and a per-level ring of
//                 one to three chunks in registers keeps loads in flight ahead of the staging;
//                 every wave multiplies all 16-point row blocks of the window with its own
//                 query fragment on v_mfma_f32_16x16x32_bf16 (rows = window points,
//                 columns = queries).  fp32 features enter as bf16 hi + lo and the three
//                 significant partial products are accumulated in fp32
//                 (hi*hi + hi*lo + lo*hi), or hi*hi alone in bf16 mode.  The first chunk of
//                 the next level is fetched before the epilogue of the current one.
//   epilogue    : S_l goes to LDS as [pt][query]; each query reads the 2x2 stencil of its
//                 own (2r+2)^2 sub-window and writes its (2r+1)^2 taps.
// Window points outside the level are staged as zeros, which is the zero
// padding of the sampling rule.
#include "corr_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

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
constexpr int XCD_RUN = 64;   // about one 8x8 super-tile of cells
constexpr int NCMAX = CORR_BLOCK_MAX_D / CORR_CHUNK;   // chunks of query fragments a wave can hold
static_assert(CORR_GROUP == 64, "work items hold 64 queries: 16 per wave");

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
    int f1_stride, f2_stride;            // elements between chunk planes
    int rec;                             // elements per pixel record: 64 (hi + lo) or 32 (hi only)
    CellGrid g;
    float scale;
};

constexpr int cmax(int a, int b) { return a > b ? a : b; }

template <int LVL, bool THREE = true>
struct Geo {
    static constexpr int PPR = THREE ? 8 : 4;             // 16-byte pieces staged per row (hi, and lo if used)
    static constexpr int ROWB = PPR * 16;                 // LDS bytes per staged row (pieces swizzled, no padding)
    static constexpr int CXL = cmax(CX >> LVL, 1), CYL = cmax(CY >> LVL, 1);
    static constexpr int WSX = CXL + K, WSY = CYL + K;   // window sides
    static constexpr int NPTS = WSX * WSY;
    static constexpr int NWB = (NPTS + 15) / 16;          // 16-point row blocks
    static constexpr int ROWS = NWB * 16;
    static constexpr int BUF_BYTES = ROWS * ROWB;         // one staged chunk
    static constexpr int S_BYTES = ROWS * 64 * 4;
    static constexpr int UNION_BYTES = cmax(2 * BUF_BYTES, S_BYTES);
    static constexpr int ITERS = (ROWS * PPR + NT - 1) / NT;   // 16-byte pieces per thread and chunk
    // chunks kept in flight in registers ahead of the one being staged: the small windows of the
    // coarse levels have short MFMA phases, so they need more loads in flight to cover the latency
    static constexpr int PD = LVL == 0 ? 1 : (LVL == 1 ? 2 : 3);
    __device__ static int row_of(int idx) { return idx / PPR; }
    __device__ static int piece_of(int idx) { return idx % PPR; }
    // LDS byte offset of piece `piece` of row `row`.  The piece slot is XOR-swizzled with the row
    // so that the 16 rows x 16 bytes that a quarter wave reads for one MFMA fragment fall in 16
    // different 4-bank groups.
    __device__ static int lds_off(int row, int piece) {
        return row * ROWB + ((piece ^ ((row / (16 / PPR)) & (PPR - 1))) << 4);
    }
};
// A pass of the kernel covers level LVL, or (FUSE) levels LVL and LVL + 1 together: their
// windows are staged one after the other as one block of rows, contracted in the same chunk loop
// and sampled one after the other.  Fusing the two small coarse windows halves their share of
// chunk steps, barriers and pipeline fills.
template <int LVL, bool THREE = true, bool FUSE = false>
struct Pass {
    using A = Geo<LVL, THREE>;
    using B = Geo<(LVL + 1 < CORR_MAX_L ? LVL + 1 : LVL), THREE>;
    static constexpr int PPR = A::PPR, ROWB = A::ROWB;
    static constexpr int ROWS = A::ROWS + (FUSE ? B::ROWS : 0);
    static constexpr int NWB = ROWS / 16;
    static constexpr int BUF_BYTES = ROWS * ROWB;         // one staged chunk
    static constexpr int S_BYTES = ROWS * 64 * 4;
    static constexpr int UNION_BYTES = cmax(2 * BUF_BYTES, S_BYTES);
    static constexpr int ITERS = (ROWS * PPR + NT - 1) / NT;   // 16-byte pieces per thread and chunk
    static constexpr int PD = FUSE ? 2 : A::PD;
    static constexpr int NEXT = LVL + (FUSE ? 2 : 1);     // first level of the following pass
};
constexpr int UNION_BYTES = cmax(cmax(cmax(Geo<0>::UNION_BYTES, Geo<1>::UNION_BYTES),
                                      cmax(Geo<2>::UNION_BYTES, Geo<3>::UNION_BYTES)),
                                 Pass<2, true, true>::UNION_BYTES);
constexpr int META_BYTES = CORR_GROUP * 12;
constexpr int LDS_BYTES = UNION_BYTES + META_BYTES;

struct ItemCtx {
    int b, u, v, n;          // batch item, absolute cell coordinates, queries in the group
    int tid, lane, wave;
    const int* q_pix;        // LDS: pixel of each query slot or -1
    const float* q_cx;       // LDS: raw coordinates
    const float* q_cy;
};

// Per-thread staging state of one level: which 16-byte pieces of the window this thread
// moves for every chunk, and a ring of PD chunks of them in registers.
template <int LVL, bool THREE, bool FUSE = false>
struct Stage {
    using P = Pass<LVL, THREE, FUSE>;
    int goff[P::ITERS];              // element offset into f2s at chunk 0, or -1 for a zero row
    uint4 sv[P::PD][P::ITERS];
};

template <int LVL>
__device__ __forceinline__ void window_origin(const ItemCtx& c, int& xs, int& ys) {
    xs = ((c.u << CORR_LOG_CX) >> LVL) - R;
    ys = ((c.v << CORR_LOG_CY) >> LVL) - R;
}

// element offset (chunk 0) of window point `row` of level LVL of this item, or -1 for a zero row
template <int LVL, bool THREE>
__device__ __forceinline__ int point_offset(const BlockArgs& a, const ItemCtx& c, int row) {
    using G = Geo<LVL, THREE>;
    if (row >= G::NPTS) return -1;
    const int Hl = a.Hl[LVL], Wl = a.Wl[LVL];
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    const int wy = row / G::WSX, wx = row - wy * G::WSX;
    const int y = ys + wy, x = xs + wx;
    if (y < 0 || y >= Hl || x < 0 || x >= Wl) return -1;
    return (a.pix_base[LVL] + (c.b * Hl + y) * Wl + x) * (THREE ? 64 : a.rec);
}

template <int LVL, bool THREE, bool FUSE>
__device__ __forceinline__ void plan(const BlockArgs& a, const ItemCtx& c, Stage<LVL, THREE, FUSE>& st) {
    using P = Pass<LVL, THREE, FUSE>;
#pragma unroll
    for (int it = 0; it < P::ITERS; ++it) {
        const int idx = it * NT + c.tid;
        const int row = idx / P::PPR, piece = idx % P::PPR;         // pieces 0..3: hi record, 4..7: lo record
        int off;
        if (!FUSE || row < P::A::ROWS) off = point_offset<LVL, THREE>(a, c, row);
        else off = point_offset<(FUSE ? LVL + 1 : LVL), THREE>(a, c, row - P::A::ROWS);
        st.goff[it] = off < 0 ? -1 : off + piece * 8;
        // bf16x3: zero rows stay zero in every ring slot, fetch() only ever writes the lanes that load
        // (in bf16 mode the select in fetch() measured faster)
        if (THREE) {
#pragma unroll
            for (int d = 0; d < P::PD; ++d) st.sv[d][it] = make_uint4(0, 0, 0, 0);
        }
    }
}

// global -> ring slot `slot` for chunk kc
template <int LVL, bool THREE, bool FUSE>
__device__ __forceinline__ void fetch(const BlockArgs& a, Stage<LVL, THREE, FUSE>& st, int slot, int kc) {
    using P = Pass<LVL, THREE, FUSE>;
    const uint16_t* base = a.f2s + (size_t)kc * a.f2_stride;
#pragma unroll
    for (int it = 0; it < P::ITERS; ++it)
        if (THREE) {
            if (st.goff[it] >= 0) st.sv[slot][it] = *reinterpret_cast<const uint4*>(base + st.goff[it]);
        } else {
            st.sv[slot][it] = st.goff[it] >= 0 ? *reinterpret_cast<const uint4*>(base + st.goff[it]) : make_uint4(0, 0, 0, 0);
        }
}

// ring slot -> LDS buffer
template <int LVL, bool THREE, bool FUSE>
__device__ __forceinline__ void stage(const Stage<LVL, THREE, FUSE>& st, int slot, unsigned char* buf, int tid) {
    using P = Pass<LVL, THREE, FUSE>;
#pragma unroll
    for (int it = 0; it < P::ITERS; ++it) {
        const int idx = it * NT + tid;
        // only the last iteration can run past the staged rows
        if ((it + 1) * NT <= P::ROWS * P::PPR || idx / P::PPR < P::ROWS)
            *reinterpret_cast<uint4*>(buf + P::A::lds_off(idx / P::PPR, idx % P::PPR)) = st.sv[slot][it];
    }
}

// Query fragments of this wave for chunks g .. g+NCMAX-1: lane holds channels 8*(lane/16) .. +7 of
// every chunk of query 16*wave + lane%16 (the B operand of the MFMA); empty slots hold zeros.
template <bool THREE>
__device__ __forceinline__ void load_queries(const BlockArgs& a, const ItemCtx& c, int g,
                                             bf16x8 (&qhi)[NCMAX], bf16x8 (&qlo)[NCMAX]) {
    const int pix = c.q_pix[c.wave * 16 + (c.lane & 15)];
    const uint16_t* src = a.f1s + ((size_t)c.b * a.HW + max(pix, 0)) * (THREE ? 64 : a.rec) + (c.lane >> 4) * 8;
#pragma unroll
    for (int kk = 0; kk < NCMAX; ++kk) {
        uint4 h = make_uint4(0, 0, 0, 0), l = make_uint4(0, 0, 0, 0);
        if (g + kk < a.NC && pix >= 0) {
            h = *reinterpret_cast<const uint4*>(src + (size_t)(g + kk) * a.f1_stride);
            if (THREE) l = *reinterpret_cast<const uint4*>(src + (size_t)(g + kk) * a.f1_stride + 32);
        }
        qhi[kk] = __builtin_bit_cast(bf16x8, h);
        qlo[kk] = __builtin_bit_cast(bf16x8, l);
    }
}

// The taps of level LVL for the item's queries, from that level's S rows in LDS ([point][query]).
// lane = query; wave 0 takes tap columns (x offsets) 0..2, waves 1..3 two columns each.  A
// footprint column is read from LDS once (all 2r+2 rows at once, so the reads overlap) and
// serves as the right neighbour of one tap column and the left neighbour of the next.
template <int LVL, bool THREE, bool NHWC>
__device__ __forceinline__ void write_taps(const BlockArgs& a, const ItemCtx& c, const float* S) {
    using G = Geo<LVL, THREE>;
    // channels-last output: the tap stride is the constant 1, so that the compiler can merge a
    // query's consecutive taps into wide stores
    const size_t tap_stride = NHWC ? 1 : (size_t)a.tap_stride;
    float* o_lvl = a.out + (size_t)c.b * a.L * KK * a.HW + (size_t)(LVL * KK) * tap_stride;
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    const int q = c.lane, wave = c.wave;
    if (q < c.n) {
        const float inv = __uint_as_float((uint32_t)(127 - LVL) << 23);   // 2^-LVL
        const float cxl = c.q_cx[q] * inv, cyl = c.q_cy[q] * inv;
        const float flx = floorf(cxl), fly = floorf(cyl);
        const float fx = cxl - flx, fy = cyl - fly;
        const int rx = (int)flx - R - xs, ry = (int)fly - R - ys;         // in [0, CXL) x [0, CYL)
        // K = 9: columns 0..3, 3..5, 5..7, 7..9; otherwise an even split
        const int i0 = K == 9 ? (wave == 0 ? 0 : 2 * wave + 1) : wave * K / NW;
        const int i1 = K == 9 ? 2 * wave + 3 : (wave + 1) * K / NW;
        const float* s = S + (ry * G::WSX + rx + i0) * 64 + q;
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

template <int LVL, bool THREE>
__device__ __forceinline__ bool window_touches(const BlockArgs& a, const ItemCtx& c) {
    using G = Geo<LVL, THREE>;
    int xs, ys;
    window_origin<LVL>(c, xs, ys);
    return xs + G::WSX - 1 >= 0 && xs <= a.Wl[LVL] - 1 && ys + G::WSY - 1 >= 0 && ys <= a.Hl[LVL] - 1;
}

// One pass of one work item (one level, or two fused).  On entry `st` holds the staging plan and
// chunk 0 in ring slot 0 (fetched before the previous pass's epilogue); before its own epilogue
// the pass plans the next one and fetches its chunk 0 into `nx`, so that those loads fly under
// the tap writes.
template <int LVL, bool THREE, bool BIGD, bool NHWC, bool FUSE, class NextStage>
__device__ __forceinline__ void level_pass(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                           bf16x8 (&qhi)[NCMAX], bf16x8 (&qlo)[NCMAX],
                                           Stage<LVL, THREE, FUSE>& st, NextStage& nx) {
    using P = Pass<LVL, THREE, FUSE>;
    using G = typename P::A;
    constexpr int PD = P::PD;
    constexpr int LVL2 = FUSE ? LVL + 1 : LVL;               // the second level of a fused pass
    float* S = reinterpret_cast<float*>(smem);               // [ROWS][64], aliases the staging buffers
    const int tid = c.tid, lane = c.lane, wave = c.wave;
    auto prefetch_next = [&]() {
        if constexpr (P::NEXT < CORR_MAX_L) {
            if (P::NEXT < a.L) { plan(a, c, nx); fetch(a, nx, 0, 0); }
        }
    };

    // uniform for the workgroup: a window that is all padding gives zero taps
    const bool touches = window_touches<LVL, THREE>(a, c) || (FUSE && window_touches<LVL2, THREE>(a, c));
    if (!touches) {
        prefetch_next();
        write_zero_taps<LVL, NHWC>(a, c);
        if (FUSE) write_zero_taps<LVL2, NHWC>(a, c);
        return;
    }

    f32x4 acc[P::NWB];
#pragma unroll
    for (int i = 0; i < P::NWB; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bool active = wave * 16 < c.n;                     // this wave has queries
    // fragment read: lane holds channels 8*(lane/16)..+7 of row wb*16 + lane%16
    const int frag_hi = G::lds_off(lane & 15, lane >> 4);
    const int frag_lo = G::lds_off(lane & 15, 4 + (lane >> 4));

    // two LDS buffers: while the MFMAs read chunk kc from one, chunk kc+1 is written to the
    // other; one barrier per chunk.  Ring slot (k % PD) holds chunk k until it is staged.
    // The wave holds query fragments for NCMAX chunks; a larger D runs in groups of NCMAX chunks,
    // each with its own fragments and a restarted ring (BIGD; otherwise a single trip).
    for (int g = 0; g < (BIGD ? a.NC : 1); g += NCMAX) {
    const int nc = BIGD ? min(a.NC - g, NCMAX) : a.NC;
    if (BIGD) {
        if (g > 0 || LVL > 0) load_queries<THREE>(a, c, g, qhi, qlo);
        if (g > 0) fetch(a, st, 0, g);
    }
#pragma unroll
    for (int d = 1; d < PD; ++d)
        if (d < nc) fetch(a, st, d, g + d);
    stage(st, 0, smem, tid);
    if (PD < nc) fetch(a, st, 0, g + PD);
    __syncthreads();

#pragma unroll
    for (int kc = 0; kc < NCMAX; ++kc) {
        if (kc < nc) {                              // uniform
            const unsigned char* rows = smem + (kc & 1) * P::BUF_BYTES;
            unsigned char* other = smem + ((kc + 1) & 1) * P::BUF_BYTES;
            if (PD > 1 && kc + 1 < nc) {            // the data is already here: stage first
                stage(st, (kc + 1) % PD, other, tid);
                if (kc + 1 + PD < nc) fetch(a, st, (kc + 1) % PD, g + kc + 1 + PD);
            }
            if (active) {
                // window fragments are read two row blocks ahead of the MFMAs that use them
                constexpr int PF = 2;
                bf16x8 wh[P::NWB + PF], wl[P::NWB + PF];
#pragma unroll
                for (int wb = 0; wb < PF; ++wb) {
                    wh[wb] = *reinterpret_cast<const bf16x8*>(rows + wb * 16 * G::ROWB + frag_hi);
                    if (THREE) wl[wb] = *reinterpret_cast<const bf16x8*>(rows + wb * 16 * G::ROWB + frag_lo);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, THREE ? 2 * PF : PF, 0);
#pragma unroll
                for (int wb = 0; wb < P::NWB; ++wb) {
                    if (wb + PF < P::NWB) {
                        wh[wb + PF] = *reinterpret_cast<const bf16x8*>(rows + (wb + PF) * 16 * G::ROWB + frag_hi);
                        if (THREE) wl[wb + PF] = *reinterpret_cast<const bf16x8*>(rows + (wb + PF) * 16 * G::ROWB + frag_lo);
                    }
                    if (THREE) {
                        acc[wb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl[wb], qhi[kc], acc[wb], 0, 0, 0);
                        acc[wb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[wb], qlo[kc], acc[wb], 0, 0, 0);
                    }
                    acc[wb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh[wb], qhi[kc], acc[wb], 0, 0, 0);
                    // keep this order in the schedule: the reads for block wb + PF, then the MFMAs of block wb
                    if (wb + PF < P::NWB) __builtin_amdgcn_sched_group_barrier(0x100, THREE ? 2 : 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, THREE ? 3 : 1, 0);
                }
            }
            if (PD == 1 && kc + 1 < nc) {         // the loads had the MFMA phase to arrive
                stage(st, 0, other, tid);
                if (kc + 2 < nc) fetch(a, st, 0, g + kc + 2);
            }
            __syncthreads();
        }
    }
    }
    // the staging buffers are dead; S may overwrite them
    prefetch_next();

    // lane holds query 16*wave + lane % 16, points 4*(lane/16)+v of every row block
    if (active) {
#pragma unroll
        for (int wb = 0; wb < P::NWB; ++wb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                S[(wb * 16 + 4 * (lane >> 4) + v) * 64 + wave * 16 + (lane & 15)] = acc[wb][v];
    }
    __syncthreads();
    write_taps<LVL, THREE, NHWC>(a, c, S);
    if (FUSE) write_taps<LVL2, THREE, NHWC>(a, c, S + G::ROWS * 64);
    __syncthreads();                            // S is dead
}

template <bool THREE, bool BIGD, bool NHWC>
__global__ __launch_bounds__(NT, 2) void block_kernel(BlockArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    int* q_pix = reinterpret_cast<int*>(smem + UNION_BYTES);
    float* q_cx = reinterpret_cast<float*>(q_pix + CORR_GROUP);
    float* q_cy = q_cx + CORR_GROUP;

    // XCD-aware item choice: workgroup w runs on XCD w % 8.  Items are dealt to the XCDs in runs
    // of consecutive items (neighbouring cells share window rows and columns, so they should
    // share an L2), round robin, so that cheap border regions do not all land on the same XCD.
    // About 16 runs per XCD, at most XCD_RUN items each.
    const int n_items = *a.n_items;
    const int run = min(max(n_items >> 7, 8), XCD_RUN);
    const int j = blockIdx.x >> 3;
    const int k = ((j / run) * 8 + (blockIdx.x & 7)) * run + j % run;
    if (k >= n_items) return;
    const int4 item = a.items[k];
    ItemCtx c;
    c.tid = threadIdx.x; c.lane = c.tid & 63; c.wave = c.tid >> 6;
    c.n = item.z;
    corr_cell_coords(a.g, item.x, &c.b, &c.u, &c.v);
    c.u += a.g.u_min; c.v += a.g.v_min;
    c.q_pix = q_pix; c.q_cx = q_cx; c.q_cy = q_cy;

    // level 0's first chunk starts to move before anything else
    Stage<0, THREE> s0;
    plan(a, c, s0);
    fetch(a, s0, 0, 0);

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

    bf16x8 qhi[NCMAX], qlo[NCMAX];
    load_queries<THREE>(a, c, 0, qhi, qlo);

    // passes: level 0, level 1, then levels 2 and 3 together when there are four
    Stage<1, THREE> s1;
    level_pass<0, THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, s0, s1);
    if (a.L == 4) {
        Stage<2, THREE, true> s23;
        level_pass<1, THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, s1, s23);
        level_pass<2, THREE, BIGD, NHWC, true>(a, c, smem, qhi, qlo, s23, s23);
    } else if (a.L > 1) {
        Stage<2, THREE> s2;
        level_pass<1, THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, s1, s2);
        if (a.L > 2) level_pass<2, THREE, BIGD, NHWC, false>(a, c, smem, qhi, qlo, s2, s2);
    }
}

template <bool THREE, bool BIGD, bool NHWC>
hipError_t launch_items(corr_pyramid* p, const float* coords, float* out, hipStream_t s) {
    static bool attr_set = false;
    auto kfn = block_kernel<THREE, BIGD, NHWC>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    BlockArgs a;
    a.f1s = p->f1_split; a.f2s = p->f2_split; a.coords = coords; a.perm = p->perm; a.items = p->items;
    a.n_items = p->n_items; a.out = out; a.B = p->B; a.HW = p->H * p->W; a.NC = p->D / CORR_CHUNK; a.L = p->L;
    a.tap_stride = corr_tap_stride(p); a.pix_stride = corr_pix_stride(p, R);
    a.g = p->grid;
    for (int l = 0; l < CORR_MAX_L; ++l) { a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l]; a.pix_base[l] = p->f2_pix_base[l]; }
    a.rec = (!THREE && (p->built & CORR_REP_BF16)) ? 32 : 64;      // bf16 mode prefers the hi-only records
    if (a.rec == 32) { a.f1s = p->f1_hi; a.f2s = p->f2_hi; }
    a.f1_stride = p->B * p->H * p->W * a.rec; a.f2_stride = p->f2_pix_total * a.rec;
    a.scale = 1.0f / sqrtf((float)p->D);
    const int grid = (p->max_items + 8 * XCD_RUN - 1) / (8 * XCD_RUN) * (8 * XCD_RUN);
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t CORR_CAT(launch_block_r, CORR_BLOCK_R)(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s) {
    const bool big = p->D > CORR_BLOCK_MAX_D, three = prec != CORR_PREC_BF16;
#define CORR_LAUNCH(NHWC)                                                                                    \
    (three ? (big ? launch_items<true, true, NHWC>(p, coords, out, s) : launch_items<true, false, NHWC>(p, coords, out, s))   \
           : (big ? launch_items<false, true, NHWC>(p, coords, out, s) : launch_items<false, false, NHWC>(p, coords, out, s)))
    return p->out_nhwc ? CORR_LAUNCH(true) : CORR_LAUNCH(false);
#undef CORR_LAUNCH
}
