// Per-lookup compute (paper: steps b and c, "Sparse Correlation Volume
// Computation" and "Sparse Volume Sampling"; fused as in "Fused Implementation":
// the computed block lives only in registers and LDS).
//
// One workgroup (4 waves) = one work item = (target cell, <= 64 of its queries),
// processed for every pyramid level in turn:
//   contraction : S[pt][q] = <f2_l(window point pt), f1(query q)> over D, in
//                 32-channel chunks staged through LDS, on
//                 v_mfma_f32_16x16x32_bf16 with rows = window points and
//                 columns = queries; fp32 features enter as bf16 hi + lo and
//                 the three significant partial products are accumulated in
//                 fp32 (hi*hi + hi*lo + lo*hi), or hi*hi alone in bf16 mode.
//   epilogue    : S goes to LDS as [pt][query]; each query reads the 2x2 stencil
//                 of its own (2r+2)^2 sub-window and writes its (2r+1)^2 taps.
// Window points outside the level are staged as zeros, which is the zero
// padding of the sampling rule.  The query features are re-read per level from
// L2, so HBM sees them once per lookup.
#include "corr_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWB = 144;   // LDS bytes per staged row: 64 B hi + 64 B lo + 16 B pad (conflict-free b128 reads)
constexpr int R = CORR_R, K = 2 * R + 1, KK = K * K;
constexpr int CX = 1 << CORR_LOG_CX, CY = 1 << CORR_LOG_CY;

struct BlockArgs {
    const uint16_t* f1s;                 // [NC][B*HW][64]
    const uint16_t* f2s;                 // [NC][P][64], P = pixels of all levels; level l starts at pix_base[l]
    const float* coords;                 // [B][2][HW]
    const int* perm;
    const int4* items;
    const int* n_items;
    float* out;
    int B, HW, NC, L;
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L], pix_base[CORR_MAX_L];
    int f1_stride, f2_stride;            // elements between chunk planes
    CellGrid g;
    float scale;
};

constexpr int cmax(int a, int b) { return a > b ? a : b; }

template <int LVL>
struct Geo {
    static constexpr int CXL = cmax(CX >> LVL, 1), CYL = cmax(CY >> LVL, 1);
    static constexpr int WSX = CXL + K, WSY = CYL + K;   // window sides
    static constexpr int NPTS = WSX * WSY;
    static constexpr int NWB = (NPTS + 15) / 16;          // 16-point row blocks
    static constexpr int WBW = (NWB + 3) / 4;             // row blocks per wave
    static constexpr int ROWS = NWB * 16;
    static constexpr int STAGE_BYTES = (ROWS + CORR_GROUP) * ROWB;
    static constexpr int S_BYTES = ROWS * CORR_GROUP * 4;
    static constexpr int UNION_BYTES = cmax(STAGE_BYTES, S_BYTES);
    static constexpr int WIN_ITERS = (NPTS * 8 + 255) / 256;
};
constexpr int UNION_BYTES = cmax(cmax(Geo<0>::UNION_BYTES, Geo<1>::UNION_BYTES),
                                 cmax(Geo<2>::UNION_BYTES, Geo<3>::UNION_BYTES));
constexpr int META_BYTES = CORR_GROUP * 12;
constexpr int LDS_BYTES = UNION_BYTES + META_BYTES;

struct ItemCtx {
    int b, u, v, n;          // batch item, absolute cell coordinates, queries in the group
    int tid, lane, wave;
    int qoff[2];             // this thread's two 16-byte pieces of the query rows (element offset or -1)
};

template <int LVL, bool THREE>
__device__ __forceinline__ void level_pass(const BlockArgs& a, const ItemCtx& c, unsigned char* smem,
                                           const int* q_pix, const float* q_cx, const float* q_cy) {
    using G = Geo<LVL>;
    unsigned char* win = smem;                               // ROWS x ROWB
    unsigned char* qry = smem + G::ROWS * ROWB;              // 64 x ROWB
    float* S = reinterpret_cast<float*>(smem);               // [ROWS][64], aliases the staging area
    const int Hl = a.Hl[LVL], Wl = a.Wl[LVL];
    const int xs = ((c.u << CORR_LOG_CX) >> LVL) - R;        // window origin in level pixels
    const int ys = ((c.v << CORR_LOG_CY) >> LVL) - R;
    const int tid = c.tid, lane = c.lane, wave = c.wave;
    float* o_lvl = a.out + ((size_t)(c.b * a.L + LVL) * KK) * a.HW;

    // epilogue work split: 18 half-columns (x offset i, y offsets 0..4 or 5..8) dealt round-robin to the waves
    const bool touches = xs + G::WSX - 1 >= 0 && xs <= Wl - 1 && ys + G::WSY - 1 >= 0 && ys <= Hl - 1;
    if (!touches) {             // uniform for the workgroup: this level's window is all padding
        if (lane < c.n) {
            float* o = o_lvl + q_pix[lane];
            for (int uidx = wave; uidx < 2 * K; uidx += 4) {
                const int i = uidx >> 1, j0 = (uidx & 1) ? 5 : 0, j1 = (uidx & 1) ? K : 5;
                for (int j = j0; j < j1; ++j) o[(size_t)(i * K + j) * a.HW] = 0.f;
            }
        }
        return;
    }

    // rows NPTS..ROWS-1 of the window never receive data: keep them zero
    for (int i = tid; i < (G::ROWS - G::NPTS) * (ROWB / 16); i += 256)
        reinterpret_cast<uint4*>(win + G::NPTS * ROWB)[i] = make_uint4(0, 0, 0, 0);

    // staging plan: the same (point, 16-byte piece) per thread for every chunk
    int goff[G::WIN_ITERS];
#pragma unroll
    for (int it = 0; it < G::WIN_ITERS; ++it) {
        const int idx = it * 256 + tid;
        const int pt = idx >> 3, piece = idx & 7;
        goff[it] = -1;
        if (pt < G::NPTS) {
            const int wy = pt / G::WSX, wx = pt - wy * G::WSX;
            const int y = ys + wy, x = xs + wx;
            if (y >= 0 && y < Hl && x >= 0 && x < Wl) goff[it] = (a.pix_base[LVL] + (c.b * Hl + y) * Wl + x) * 64 + piece * 8;
        }
    }

    f32x4 acc[G::WBW][4];
#pragma unroll
    for (int i = 0; i < G::WBW; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nqf = (c.n + 15) >> 4;
    const int frag_off = (lane & 15) * ROWB + (lane >> 4) * 16;

    // global -> registers for chunk 0; inside the loop the next chunk's loads are
    // issued right after the LDS stores so that they fly under the MFMAs
    uint4 wv[G::WIN_ITERS], qv[2];
    auto load_chunk = [&](int kc) {
        const uint16_t* f2c = a.f2s + (size_t)kc * a.f2_stride;
        const uint16_t* f1c = a.f1s + (size_t)kc * a.f1_stride;
#pragma unroll
        for (int it = 0; it < G::WIN_ITERS; ++it)
            wv[it] = goff[it] >= 0 ? *reinterpret_cast<const uint4*>(f2c + goff[it]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int it = 0; it < 2; ++it)
            qv[it] = c.qoff[it] >= 0 ? *reinterpret_cast<const uint4*>(f1c + c.qoff[it]) : make_uint4(0, 0, 0, 0);
    };
    load_chunk(0);

    for (int kc = 0; kc < a.NC; ++kc) {
        if (kc > 0) __syncthreads();            // everyone is done reading the previous chunk
#pragma unroll
        for (int it = 0; it < G::WIN_ITERS; ++it) {
            const int idx = it * 256 + tid;
            if ((idx >> 3) < G::NPTS)
                *reinterpret_cast<uint4*>(win + (idx >> 3) * ROWB + (idx & 7) * 16) = wv[it];
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int idx = it * 256 + tid;
            *reinterpret_cast<uint4*>(qry + (idx >> 3) * ROWB + (idx & 7) * 16) = qv[it];
        }
        __syncthreads();
        if (kc + 1 < a.NC) load_chunk(kc + 1);

        bf16x8 qh[4], ql[4];
#pragma unroll
        for (int qf = 0; qf < 4; ++qf) {
            qh[qf] = *reinterpret_cast<const bf16x8*>(qry + qf * 16 * ROWB + frag_off);
            if (THREE) ql[qf] = *reinterpret_cast<const bf16x8*>(qry + qf * 16 * ROWB + frag_off + 64);
        }
#pragma unroll
        for (int i = 0; i < G::WBW; ++i) {
            const int wb = wave + 4 * i;
            if (wb < G::NWB) {
                const bf16x8 wh = *reinterpret_cast<const bf16x8*>(win + wb * 16 * ROWB + frag_off);
                bf16x8 wl;
                if (THREE) wl = *reinterpret_cast<const bf16x8*>(win + wb * 16 * ROWB + frag_off + 64);
#pragma unroll
                for (int qf = 0; qf < 4; ++qf) {
                    if (qf < nqf) {
                        if (THREE) {
                            acc[i][qf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wl, qh[qf], acc[i][qf], 0, 0, 0);
                            acc[i][qf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh, ql[qf], acc[i][qf], 0, 0, 0);
                        }
                        acc[i][qf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wh, qh[qf], acc[i][qf], 0, 0, 0);
                    }
                }
            }
        }
    }
    __syncthreads();                            // staging area is dead; S may overwrite it

    // S to LDS: lane holds query (lane % 16) of fragment qf, points 4*(lane/16)+v
#pragma unroll
    for (int i = 0; i < G::WBW; ++i) {
        const int wb = wave + 4 * i;
        if (wb < G::NWB) {
#pragma unroll
            for (int qf = 0; qf < 4; ++qf)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    S[(wb * 16 + 4 * (lane >> 4) + v) * CORR_GROUP + qf * 16 + (lane & 15)] = acc[i][qf][v] * a.scale;
        }
    }
    __syncthreads();

    // bilinear epilogue: lane = query; a wave takes half-columns of taps.  Along a
    // column the x-interpolated value of each footprint row is reused by two taps.
    if (lane < c.n) {
        const float inv = __uint_as_float((uint32_t)(127 - LVL) << 23);   // 2^-LVL
        const float cxl = q_cx[lane] * inv, cyl = q_cy[lane] * inv;
        const float flx = floorf(cxl), fly = floorf(cyl);
        const float fx = cxl - flx, fy = cyl - fly;
        const int rx = (int)flx - R - xs, ry = (int)fly - R - ys;         // in [0, CXL) x [0, CYL)
        const float* s0 = S + (ry * G::WSX + rx) * CORR_GROUP + lane;
        float* o = o_lvl + q_pix[lane];
        for (int uidx = wave; uidx < 2 * K; uidx += 4) {
            const int i = uidx >> 1, j0 = (uidx & 1) ? 5 : 0, j1 = (uidx & 1) ? K : 5;
            const float* s = s0 + (j0 * G::WSX + i) * CORR_GROUP;
            float hprev = s[0] + fx * (s[CORR_GROUP] - s[0]);
            for (int j = j0; j < j1; ++j) {
                s += G::WSX * CORR_GROUP;
                const float hcur = s[0] + fx * (s[CORR_GROUP] - s[0]);
                o[(size_t)(i * K + j) * a.HW] = hprev + fy * (hcur - hprev);
                hprev = hcur;
            }
        }
    }
    __syncthreads();                            // S is dead; the next level may stage
}

template <bool THREE>
__global__ __launch_bounds__(256, 2) void block_kernel(BlockArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    int* q_pix = reinterpret_cast<int*>(smem + UNION_BYTES);
    float* q_cx = reinterpret_cast<float*>(q_pix + CORR_GROUP);
    float* q_cy = q_cx + CORR_GROUP;

    // XCD-aware item choice: workgroup w runs on XCD w % 8; give each XCD one
    // contiguous eighth of the items (neighbouring cells share window rows and
    // columns, so they should share an L2).
    const int n_items = *a.n_items;
    const int per_xcd = (n_items + 7) >> 3;
    const int k = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || k >= n_items) return;
    const int4 item = a.items[k];
    ItemCtx c;
    c.tid = threadIdx.x; c.lane = c.tid & 63; c.wave = c.tid >> 6;
    c.n = item.z;
    corr_cell_coords(a.g, item.x, &c.b, &c.u, &c.v);
    c.u += a.g.u_min; c.v += a.g.v_min;

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
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int idx = it * 256 + c.tid;
        const int pix = q_pix[idx >> 3];
        c.qoff[it] = pix < 0 ? -1 : (c.b * a.HW + pix) * 64 + (idx & 7) * 8;
    }

    level_pass<0, THREE>(a, c, smem, q_pix, q_cx, q_cy);
    if (a.L > 1) level_pass<1, THREE>(a, c, smem, q_pix, q_cx, q_cy);
    if (a.L > 2) level_pass<2, THREE>(a, c, smem, q_pix, q_cx, q_cy);
    if (a.L > 3) level_pass<3, THREE>(a, c, smem, q_pix, q_cx, q_cy);
}

template <bool THREE>
hipError_t launch_items(corr_pyramid* p, const float* coords, float* out, hipStream_t s) {
    static bool attr_set = false;
    auto kfn = block_kernel<THREE>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    BlockArgs a;
    a.f1s = p->f1_split; a.f2s = p->f2_split; a.coords = coords; a.perm = p->perm; a.items = p->items; a.n_items = p->n_items;
    a.out = out; a.B = p->B; a.HW = p->H * p->W; a.NC = p->D / CORR_CHUNK; a.L = p->L; a.g = p->grid;
    for (int l = 0; l < CORR_MAX_L; ++l) { a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l]; a.pix_base[l] = p->f2_pix_base[l]; }
    a.f1_stride = p->B * p->H * p->W * 64; a.f2_stride = p->f2_pix_total * 64;
    a.scale = 1.0f / sqrtf((float)p->D);
    const int grid = ((p->max_items + 7) / 8) * 8;
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(256), LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_block(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s) {
    return prec == CORR_PREC_BF16 ? launch_items<false>(p, coords, out, s) : launch_items<true>(p, coords, out, s);
}
