// Host side of the C ABI declared in include/corr.h: argument checks, the
// pyramid object and its device allocations, and the order in which the kernels
// of one build / one lookup are enqueued.
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>
#include "corr_internal.h"
#include <atomic>

namespace {

bool level_sizes_ok(int H, int W, int L) {
    return L >= 1 && L <= CORR_MAX_L && (H >> (L - 1)) >= 1 && (W >> (L - 1)) >= 1;
}

corr_status check_dims(int B, int H, int W, int D, int L) {
    if (B <= 0 || H <= 0 || W <= 0 || D <= 0 || L <= 0) return CORR_ERR_INVALID_ARG;
    if (L > CORR_MAX_L) return CORR_ERR_UNSUPPORTED;
    if (!level_sizes_ok(H, W, L)) return CORR_ERR_INVALID_ARG;
    if (D % CORR_CHUNK != 0 || D > 1024) return CORR_ERR_UNSUPPORTED;
    if ((long long)B * H * W * 81 * L >= (1LL << 31)) return CORR_ERR_UNSUPPORTED;
    long long px = 0;
    for (int l = 0; l < L; ++l) px += (long long)(H >> l) * (W >> l);
    if ((long long)B * px * D * 2 >= (1LL << 31)) return CORR_ERR_UNSUPPORTED;   // 32-bit element offsets
    if ((long long)B * px * 128 >= (1LL << 31)) return CORR_ERR_UNSUPPORTED;     // byte offsets inside one chunk plane of the split pyramid
    if ((long long)B * H * W * D * 4 >= (1LL << 32)) return CORR_ERR_UNSUPPORTED;  // unsigned byte offsets into the split fmap1
    return CORR_OK;
}

void fill_geometry(corr_pyramid* p) {
    for (int l = 0; l < CORR_MAX_L; ++l) { p->Hl[l] = p->H >> l; p->Wl[l] = p->W >> l; }
    corr_fill_grid(&p->grid, p->H, p->W, p->L);
}

template <typename T>
corr_status dev_alloc(T** ptr, size_t count, size_t* total) {
    void* v = nullptr;
    const size_t bytes = count * sizeof(T);
    if (hipMalloc(&v, bytes ? bytes : 16) != hipSuccess) { (void)hipGetLastError(); return CORR_ERR_OOM; }
    *ptr = static_cast<T*>(v);
    *total += bytes;
    return CORR_OK;
}

void free_volume(corr_pyramid* p) {
    for (int l = 0; l < CORR_MAX_L; ++l)
        if (p->vol[l]) {
            (void)hipFree(p->vol[l]);
            p->bytes -= (size_t)4 * p->B * p->H * p->W * p->Hl[l] * p->Wl[l];
            p->vol[l] = nullptr;
        }
    p->vol_valid = 0;
}

void free_all(corr_pyramid* p) {
    free_volume(p);
    (void)hipFree(p->f1_nhwc); (void)hipFree(p->f1_split);
    for (int l = 0; l < CORR_MAX_L; ++l) (void)hipFree(p->f2_nhwc[l]);
    (void)hipFree(p->f2_split); (void)hipFree(p->f1_hi); (void)hipFree(p->f2_hi);
    (void)hipFree(p->ws_mem);
    delete p;
}

size_t feature_bytes(unsigned reps, int B, int H, int W, int D, int L) {
    size_t px = (size_t)H * W;            // fmap1
    for (int l = 0; l < L; ++l) px += (size_t)(H >> l) * (W >> l);
    size_t per_px = 0;
    if (reps & CORR_REP_SPLIT) per_px += (size_t)D * 4;   // bf16 hi + lo
    if (reps & CORR_REP_F32) per_px += (size_t)D * 4;
    if (reps & CORR_REP_BF16) per_px += (size_t)D * 2;
    return (size_t)B * px * per_px;
}

corr_status create(int B, int H, int W, int D, int L, unsigned reps, corr_pyramid** out) {
    corr_pyramid* p = new (std::nothrow) corr_pyramid();
    if (!p) return CORR_ERR_OOM;
    memset(p, 0, sizeof(*p));
    p->B = B; p->H = H; p->W = W; p->D = D; p->L = L; p->reps = reps;
    fill_geometry(p);
    const size_t HW = (size_t)H * W, BN = (size_t)B * HW;
    corr_status st = CORR_OK;
    auto need = [&](corr_status s) { if (st == CORR_OK) st = s; };
    if (reps & CORR_REP_F32) {
        need(dev_alloc(&p->f1_nhwc, BN * D, &p->bytes));
        for (int l = 0; l < L; ++l)
            need(dev_alloc(&p->f2_nhwc[l], (size_t)B * p->Hl[l] * p->Wl[l] * D, &p->bytes));
    }
    if (reps & (CORR_REP_SPLIT | CORR_REP_BF16)) {      // what block mode reads, and its binning workspace
        size_t px = 0;
        for (int l = 0; l < L; ++l) { p->f2_pix_base[l] = (int)px; px += (size_t)B * p->Hl[l] * p->Wl[l]; }
        p->f2_pix_total = (int)px;
        if (reps & CORR_REP_SPLIT) {
            need(dev_alloc(&p->f1_split, BN * D * 2, &p->bytes));
            need(dev_alloc(&p->f2_split, px * D * 2, &p->bytes));
        }
        if (reps & CORR_REP_BF16) {
            need(dev_alloc(&p->f1_hi, BN * D, &p->bytes));
            need(dev_alloc(&p->f2_hi, px * D, &p->bytes));
        }
        const int ncells = corr_ncells(p->grid, B);
        const WsLayout wl = corr_ws_layout((int)BN, ncells);
        unsigned char* mem = nullptr;
        need(dev_alloc(&mem, wl.total, &p->bytes));
        if (st == CORR_OK) {
            p->ws_mem = mem;
            p->ws = corr_ws_carve(mem, (int)BN, ncells);
            if (hipMemset(mem, 0, wl.total) != hipSuccess) st = CORR_ERR_HIP;   // counters start at zero
        }
    }
    if (st != CORR_OK) { free_all(p); return st; }
    *out = p;
    return CORR_OK;
}

corr_status check_against(const corr_pyramid* p, int B, int H, int W, int D, int L) {
    if (!p) return CORR_ERR_INVALID_ARG;
    if (p->B != B || p->H != H || p->W != W || p->D != D || p->L != L) return CORR_ERR_INVALID_ARG;
    return CORR_OK;
}


// ---- process-wide timing hook (measurement only)
constexpr int PROF_LOOKUPS = 256;
struct Profiler {
    int on = 0, n = 0;
    long long dropped = 0;
    hipEvent_t* ev = nullptr;      // [PROF_LOOKUPS][3]
} g_prof;

// process-wide test knob (corr_debug_set_level_split)
std::atomic<int> g_split_levels_max{CORR_SPLIT_LEVELS_MAX_QUERIES};
std::atomic<int> g_backward_form{CORR_BACKWARD_ITEMS};

hipError_t launch_block(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    return q.r == 1 ? launch_block_r1(p, ws, q, s)
         : q.r == 2 ? launch_block_r2(p, ws, q, s)
         : q.r == 3 ? launch_block_r3(p, ws, q, s)
                    : launch_block_r4(p, ws, q, s);
}

// planning pass + block kernel on workspace `ws`
hipError_t enqueue_block_lookup(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    hipEvent_t* ev = nullptr;
    if (g_prof.on && g_prof.ev) {
        if (g_prof.n < PROF_LOOKUPS) ev = g_prof.ev + (size_t)g_prof.n * 3;
        else g_prof.dropped++;
    }
    hipError_t e = hipSuccess;
    if (ev) e = hipEventRecord(ev[0], s);
    if (e == hipSuccess) e = launch_binning(p, ws, q, s);
    if (ev && e == hipSuccess) e = hipEventRecord(ev[1], s);
    if (e == hipSuccess) e = launch_block(p, ws, q, s);
    if (ev && e == hipSuccess) e = hipEventRecord(ev[2], s);
    if (ev && e == hipSuccess) g_prof.n++;
    return e;
}

corr_status check_lookup_args(const corr_pyramid* pyr, const float* coords, const float* out,
                              int B, int H, int W, int D, int L, int r) {
    if (!pyr || !coords || !out) return CORR_ERR_INVALID_ARG;
    corr_status st = check_against(pyr, B, H, W, D, L);
    if (st != CORR_OK) return st;
    if (r < 1) return CORR_ERR_INVALID_ARG;
    if (r > CORR_R) return CORR_ERR_UNSUPPORTED;
    return CORR_OK;
}

}  // namespace

// Planning workspace of corr_sample_static: one array per GPU, held until the process ends.  In
// host code the symbol is only a handle; its device address comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[CORR_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each GPU, looked up once

corr_status static_scratch(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return CORR_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return CORR_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return CORR_OK;
}
}  // namespace

extern "C" {

const char* corr_status_string(corr_status s) {
    switch (s) {
        case CORR_OK: return "ok";
        case CORR_ERR_INVALID_ARG: return "invalid argument";
        case CORR_ERR_UNSUPPORTED: return "unsupported size or parameter";
        case CORR_ERR_OOM: return "out of device memory";
        case CORR_ERR_HIP: return "HIP error";
        case CORR_ERR_MISSING_REP: return "pyramid lacks the representation this mode reads";
        case CORR_ERR_TOO_LARGE: return "input exceeds the fixed scratch buffer of corr_sample_static";
    }
    return "unknown status";
}

size_t corr_full_volume_bytes(int B, int H, int W, int L) {
    if (B <= 0 || H <= 0 || W <= 0 || !level_sizes_ok(H, W, L)) return 0;
    size_t px = 0;
    for (int l = 0; l < L; ++l) px += (size_t)(H >> l) * (W >> l);
    return (size_t)4 * B * H * W * px;
}

size_t corr_workspace_bytes(corr_mode mode, int B, int H, int W, int D, int L, int r) {
    if (check_dims(B, H, W, D, L) != CORR_OK || r < 1 || r > CORR_R) return 0;
    switch (mode) {
        case CORR_MODE_BLOCK: {
            CellGrid g;
            corr_fill_grid(&g, H, W, L);
            return feature_bytes(CORR_REP_SPLIT, B, H, W, D, L) + corr_ws_layout(B * H * W, corr_ncells(g, B)).total;
        }
        case CORR_MODE_ONDEMAND: return feature_bytes(CORR_REP_F32, B, H, W, D, L);
        case CORR_MODE_FULLVOLUME: return feature_bytes(CORR_REP_F32, B, H, W, D, L) + corr_full_volume_bytes(B, H, W, L);
    }
    return 0;
}

size_t corr_pyramid_bytes(const corr_pyramid* pyr) { return pyr ? pyr->bytes : 0; }

corr_status corr_bin_geometry(int H, int W, int L, int l, int* cell_x, int* cell_y, int* window_x, int* window_y,
                              int* cells_x, int* cells_y) {
    if (H <= 0 || W <= 0 || !level_sizes_ok(H, W, L) || l < 0 || l >= L) return CORR_ERR_INVALID_ARG;
    CellGrid g;
    corr_fill_grid(&g, H, W, L);
    const int cx = ((1 << CORR_LOG_CX) >> l) > 1 ? ((1 << CORR_LOG_CX) >> l) : 1;
    const int cy = ((1 << CORR_LOG_CY) >> l) > 1 ? ((1 << CORR_LOG_CY) >> l) : 1;
    if (cell_x) *cell_x = cx;
    if (cell_y) *cell_y = cy;
    if (window_x) *window_x = cx + 2 * CORR_R + 1;
    if (window_y) *window_y = cy + 2 * CORR_R + 1;
    if (cells_x) *cells_x = g.nbx;
    if (cells_y) *cells_y = g.nby;
    return CORR_OK;
}

corr_status corr_pyramid_build_reps(const float* fmap1, const float* fmap2, int B, int H, int W, int D, int L,
                                    unsigned reps, corr_pyramid** pyr, void* stream) {
    if (!fmap1 || !fmap2 || !pyr) return CORR_ERR_INVALID_ARG;
    if (reps == 0 || (reps & ~(CORR_REP_SPLIT | CORR_REP_F32 | CORR_REP_BF16))) return CORR_ERR_INVALID_ARG;
    corr_status st = check_dims(B, H, W, D, L);
    if (st != CORR_OK) return st;
    corr_pyramid* p = *pyr;
    if (p) {
        st = check_against(p, B, H, W, D, L);
        if (st != CORR_OK) return st;
        if ((p->reps & reps) != reps) return CORR_ERR_MISSING_REP;
    } else {
        st = create(B, H, W, D, L, reps, &p);
        if (st != CORR_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    p->vol_valid = 0;     // a cached dense volume belongs to the previous pair
    p->built = reps;      // representations not rebuilt now still hold the previous pair
    const bool sp = (reps & CORR_REP_SPLIT) != 0, fp = (reps & CORR_REP_F32) != 0, hi = (reps & CORR_REP_BF16) != 0;
    float* f1n[1] = {p->f1_nhwc};
    hipError_t e = launch_build_features(fmap1, B, D, H, W, 1, sp ? p->f1_split : nullptr, hi ? p->f1_hi : nullptr,
                                         fp ? f1n : nullptr, s);
    if (e == hipSuccess)
        e = launch_build_features(fmap2, B, D, H, W, L, sp ? p->f2_split : nullptr, hi ? p->f2_hi : nullptr,
                                  fp ? p->f2_nhwc : nullptr, s);
    if (e != hipSuccess) {
        if (!*pyr) free_all(p);
        return CORR_ERR_HIP;
    }
    *pyr = p;
    return CORR_OK;
}

corr_status corr_pyramid_build(const float* fmap1, const float* fmap2, int B, int H, int W, int D, int L,
                               corr_pyramid** pyr, void* stream) {
    return corr_pyramid_build_reps(fmap1, fmap2, B, H, W, D, L, CORR_REP_SPLIT, pyr, stream);
}

corr_status corr_pyramid_destroy(corr_pyramid* pyr, void* stream) {
    if (!pyr) return CORR_OK;
    const hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    free_all(pyr);
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_sample_mode(corr_mode mode, corr_precision prec, const float* fmap1, const corr_pyramid* pyr,
                             const float* coords, int B, int H, int W, int D, int L, int r,
                             float* out, void* stream) {
    return corr_sample_layout(mode, prec, CORR_OUT_NCHW, fmap1, pyr, coords, B, H, W, D, L, r, out, stream);
}

corr_status corr_sample_layout(corr_mode mode, corr_precision prec, corr_out_layout layout, const float* fmap1,
                               const corr_pyramid* pyr, const float* coords, int B, int H, int W, int D, int L, int r,
                               float* out, void* stream) {
    (void)fmap1;
    if (layout != CORR_OUT_NCHW && layout != CORR_OUT_NHWC) return CORR_ERR_INVALID_ARG;
    corr_status st = check_lookup_args(pyr, coords, out, B, H, W, D, L, r);
    if (st != CORR_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    LookupArgs q;
    q.coords = coords; q.out = out; q.r = r; q.nhwc = layout == CORR_OUT_NHWC; q.prec = (int)prec;
    q.split_levels_max = g_split_levels_max.load();
    switch (mode) {
        case CORR_MODE_BLOCK: {
            if (prec != CORR_PREC_BF16X3 && prec != CORR_PREC_BF16) return CORR_ERR_INVALID_ARG;
            if (!(pyr->built & (prec == CORR_PREC_BF16 ? (CORR_REP_SPLIT | CORR_REP_BF16) : CORR_REP_SPLIT)))
                return CORR_ERR_MISSING_REP;
            e = enqueue_block_lookup(pyr, pyr->ws, q, s);
            break;
        }
        case CORR_MODE_ONDEMAND: {
            if (!(pyr->built & CORR_REP_F32)) return CORR_ERR_MISSING_REP;
            e = launch_ondemand(pyr, q, s);
            break;
        }
        case CORR_MODE_FULLVOLUME: {
            if (!(pyr->built & CORR_REP_F32)) return CORR_ERR_MISSING_REP;
            if (!pyr->vol_valid) {
                // the dense volume is a lazily built representation of the pair: the one part of the
                // pyramid a lookup may fill in
                corr_pyramid* mp = const_cast<corr_pyramid*>(pyr);
                if (!mp->vol[0]) {
                    const size_t need = corr_full_volume_bytes(B, H, W, L);
                    size_t free_b = 0, total_b = 0;
                    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) return CORR_ERR_HIP;
                    if (need + (256u << 20) > free_b) return CORR_ERR_OOM;
                    for (int l = 0; l < L; ++l) {
                        st = dev_alloc(&mp->vol[l], (size_t)B * H * W * mp->Hl[l] * mp->Wl[l], &mp->bytes);
                        if (st != CORR_OK) { free_volume(mp); return st; }
                    }
                }
                e = launch_fullvol_build(mp, s);
                if (e != hipSuccess) break;
                mp->vol_valid = 1;
            }
            e = launch_fullvol_sample(pyr, q, s);
            break;
        }
        default: return CORR_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_sample(const float* fmap1, const corr_pyramid* pyr, const float* coords,
                        int B, int H, int W, int D, int L, int r, float* out, void* stream) {
    return corr_sample_mode(CORR_MODE_BLOCK, CORR_PREC_BF16X3, fmap1, pyr, coords, B, H, W, D, L, r, out, stream);
}

corr_status corr_sample_static(const float* fmap1, const corr_pyramid* pyr, const float* coords,
                               int B, int H, int W, int D, int L, int r, float* out, void* stream) {
    (void)fmap1;
    corr_status st = check_lookup_args(pyr, coords, out, B, H, W, D, L, r);
    if (st != CORR_OK) return st;
    if (!(pyr->built & CORR_REP_SPLIT)) return CORR_ERR_MISSING_REP;
    const int BN = B * H * W, ncells = corr_ncells(pyr->grid, B);
    if (corr_ws_layout(BN, ncells).total > (size_t)CORR_STATIC_SCRATCH_BYTES) return CORR_ERR_TOO_LARGE;
    void* mem = nullptr;
    st = static_scratch(&mem);
    if (st != CORR_OK) return st;
    const BinWs ws = corr_ws_carve(mem, BN, ncells);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the array keeps the last call's contents, laid out for that call's sizes: the bin counters and
    // the item / ticket counters must start at zero (fill kernels, so the call can be graph-captured)
    hipError_t e = launch_fill_i32(ws.bin_count, 0, (size_t)ws.nbins, s);
    if (e == hipSuccess) e = launch_fill_i32(ws.n_items, 0, CORR_NCOUNTERS, s);
    LookupArgs q;
    q.coords = coords; q.out = out; q.r = r; q.nhwc = 0; q.prec = (int)CORR_PREC_BF16X3;
    q.split_levels_max = g_split_levels_max.load();
    if (e == hipSuccess) e = enqueue_block_lookup(pyr, ws, q, s);
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_last_block_stats(const corr_pyramid* pyr, int r, corr_block_stats* stats, void* stream) {
    if (!pyr || !stats || r < 1 || r > CORR_R) return CORR_ERR_INVALID_ARG;
    if (!(pyr->reps & (CORR_REP_SPLIT | CORR_REP_BF16))) return CORR_ERR_MISSING_REP;
    long long h[CORR_NSTATS];
    int hn[4];
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_bin_stats(pyr, pyr->ws, r, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipMemcpyAsync(h, pyr->ws.stats, sizeof(h), hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipMemcpyAsync(hn, pyr->ws.n_items, sizeof(hn), hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CORR_ERR_HIP;
    h[0] = hn[0];
    h[1] = (long long)pyr->B * pyr->H * pyr->W * pyr->L;
    h[3] = h[4] = 0;
    long long ql = 0;
    for (int l = 0; l < 4; ++l) { h[3] += h[8 + 4 * l + 1]; h[4] += h[8 + 4 * l + 2]; ql += h[8 + 4 * l + 3]; }
    h[2] = h[1] - ql;
    stats->items = h[0]; stats->query_levels = h[1]; stats->null_query_levels = h[2];
    stats->mma_point_queries = h[3]; stats->used_point_queries = h[4];
    for (int l = 0; l < 4; ++l) {
        stats->level_items[l] = h[8 + 4 * l + 0];
        stats->level_mma_point_queries[l] = h[8 + 4 * l + 1];
        stats->level_used_point_queries[l] = h[8 + 4 * l + 2];
        stats->level_queries[l] = h[8 + 4 * l + 3];
    }
    return CORR_OK;
}

corr_status corr_copy_f32(float* dst, const float* src, size_t n, void* stream) {
    if (!dst || !src || (n & 3) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return CORR_ERR_INVALID_ARG;
    return launch_copy_f32(dst, src, n, static_cast<hipStream_t>(stream)) == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_profile_enable(int enable) {
    if (enable && !g_prof.ev) {
        const int n = PROF_LOOKUPS * 3;
        g_prof.ev = new (std::nothrow) hipEvent_t[n];
        if (!g_prof.ev) return CORR_ERR_OOM;
        for (int i = 0; i < n; ++i)
            if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
                delete[] g_prof.ev; g_prof.ev = nullptr;
                return CORR_ERR_HIP;
            }
    }
    g_prof.on = enable ? 1 : 0;
    g_prof.n = 0;
    g_prof.dropped = 0;
    return CORR_OK;
}

corr_status corr_profile_read(corr_profile* prof) {
    if (!prof) return CORR_ERR_INVALID_ARG;
    memset(prof, 0, sizeof(*prof));
    if (!g_prof.ev) return CORR_OK;
    for (int i = 0; i < g_prof.n; ++i) {
        hipEvent_t* ev = g_prof.ev + (size_t)i * 3;
        if (hipEventSynchronize(ev[2]) != hipSuccess) return CORR_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[0], ev[1]) != hipSuccess) return CORR_ERR_HIP;
        prof->binning_ms += ms;
        if (hipEventElapsedTime(&ms, ev[1], ev[2]) != hipSuccess) return CORR_ERR_HIP;
        prof->block_ms += ms;
    }
    prof->lookups = g_prof.n;
    prof->dropped = g_prof.dropped;
    g_prof.n = 0;
    g_prof.dropped = 0;
    return CORR_OK;
}

corr_status corr_debug_read_plan(const corr_pyramid* pyr, int32_t* counts, int32_t* items, size_t items_cap,
                                 int32_t* perm, size_t perm_cap, void* stream) {
    if (!pyr || !counts || !items || !perm) return CORR_ERR_INVALID_ARG;
    if (!pyr->ws_mem) return CORR_ERR_MISSING_REP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int hn[4];
    if (hipMemcpyAsync(hn, pyr->ws.n_items, sizeof(hn), hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CORR_ERR_HIP;
    counts[0] = hn[0]; counts[1] = hn[1];
    if ((size_t)hn[0] > items_cap || (size_t)hn[1] > perm_cap) return CORR_ERR_INVALID_ARG;
    if (hn[0] > 0 && hipMemcpyAsync(items, pyr->ws.items, (size_t)hn[0] * 16, hipMemcpyDeviceToHost, s) != hipSuccess)
        return CORR_ERR_HIP;
    if (hn[1] > 0 && hipMemcpyAsync(perm, pyr->ws.perm, (size_t)hn[1] * 4, hipMemcpyDeviceToHost, s) != hipSuccess)
        return CORR_ERR_HIP;
    return hipStreamSynchronize(s) == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

size_t corr_backward_workspace_bytes(int B, int H, int W, int D, int L) {
    if (check_dims(B, H, W, D, L) != CORR_OK) return 0;
    return corr_backward_workspace_bytes_internal(B, H, W, D, L);
}

corr_status corr_sample_backward(const corr_pyramid* pyr, const float* coords, const float* d_out,
                                 int B, int H, int W, int D, int L, int r,
                                 float* d_fmap1, float* d_fmap2, void* workspace, size_t workspace_bytes, void* stream) {
    if (!d_fmap1 || !d_fmap2 || !workspace) return CORR_ERR_INVALID_ARG;
    corr_status st = check_lookup_args(pyr, coords, d_out, B, H, W, D, L, r);
    if (st != CORR_OK) return st;
    if (!(pyr->built & CORR_REP_F32)) return CORR_ERR_MISSING_REP;
    if (workspace_bytes < corr_backward_workspace_bytes_internal(B, H, W, D, L)) return CORR_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return CORR_ERR_INVALID_ARG;
    // the item form addresses one batch item's feature map, and one level's planes of d_out, through 31-bit byte offsets
    if ((unsigned long long)H * W * D * 4ull >= (1ull << 31)) return CORR_ERR_UNSUPPORTED;
    if ((unsigned long long)H * W * (2 * r + 1) * (2 * r + 1) * 4ull >= (1ull << 31)) return CORR_ERR_UNSUPPORTED;
    const hipError_t e = launch_backward(pyr, coords, d_out, r, d_fmap1, d_fmap2, static_cast<float*>(workspace),
                                         g_backward_form.load(), g_split_levels_max.load(), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

int corr_debug_set_backward_form(int form) {
    return g_backward_form.exchange(form == CORR_BACKWARD_QUERIES ? CORR_BACKWARD_QUERIES : CORR_BACKWARD_ITEMS);
}

int corr_debug_set_level_split(int max_queries) {
    return g_split_levels_max.exchange(max_queries == -1 ? CORR_SPLIT_LEVELS_MAX_QUERIES : max_queries);
}

corr_status corr_debug_item_map(int max_items, int32_t* map, size_t map_cap, int* grid) {
    if (max_items < 0 || !grid) return CORR_ERR_INVALID_ARG;
    *grid = corr_block_grid(max_items);
    if (!map) return CORR_OK;
    if (map_cap < (size_t)*grid) return CORR_ERR_INVALID_ARG;
    for (int w = 0; w < *grid; ++w) map[w] = corr_item_of_workgroup(w);
    return CORR_OK;
}

corr_status corr_debug_cell_coords(const corr_pyramid* pyr, int cell_id, int* b, int* u, int* v) {
    if (!pyr || !b || !u || !v || cell_id < 0 || cell_id >= corr_ncells(pyr->grid, pyr->B)) return CORR_ERR_INVALID_ARG;
    corr_cell_coords(pyr->grid, cell_id, b, u, v);
    *u += pyr->grid.u_min; *v += pyr->grid.v_min;
    return CORR_OK;
}

corr_status corr_debug_read_level(const corr_pyramid* pyr, unsigned rep, int level, float* dst, void* stream) {
    if (!pyr || !dst || level < -1 || level >= pyr->L) return CORR_ERR_INVALID_ARG;
    if (rep != CORR_REP_F32 && rep != CORR_REP_SPLIT && rep != CORR_REP_BF16) return CORR_ERR_INVALID_ARG;
    if (!(pyr->built & rep)) return CORR_ERR_MISSING_REP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int D = pyr->D, NC = D / CORR_CHUNK;
    const size_t npix = level < 0 ? (size_t)pyr->B * pyr->H * pyr->W : (size_t)pyr->B * pyr->Hl[level] * pyr->Wl[level];
    if (rep == CORR_REP_F32) {
        const float* src = level < 0 ? pyr->f1_nhwc : pyr->f2_nhwc[level];
        if (hipMemcpyAsync(dst, src, npix * D * 4, hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
        return hipStreamSynchronize(s) == hipSuccess ? CORR_OK : CORR_ERR_HIP;
    }
    // chunk planes of [pixel][rec] bf16 records: rec = 64 (32 hi, 32 lo) or 32 (hi)
    const int rec = rep == CORR_REP_SPLIT ? 64 : 32;
    const uint16_t* base = rep == CORR_REP_SPLIT ? (level < 0 ? pyr->f1_split : pyr->f2_split)
                                                 : (level < 0 ? pyr->f1_hi : pyr->f2_hi);
    const size_t plane = level < 0 ? (size_t)pyr->B * pyr->H * pyr->W : (size_t)pyr->f2_pix_total;
    const size_t first = level < 0 ? 0 : (size_t)pyr->f2_pix_base[level];
    uint16_t* tmp = static_cast<uint16_t*>(malloc(npix * rec * 2));
    if (!tmp) return CORR_ERR_OOM;
    corr_status st = CORR_OK;
    for (int kc = 0; kc < NC && st == CORR_OK; ++kc) {
        if (hipMemcpyAsync(tmp, base + ((size_t)kc * plane + first) * rec, npix * rec * 2, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) { st = CORR_ERR_HIP; break; }
        for (size_t p = 0; p < npix; ++p)
            for (int k = 0; k < CORR_CHUNK; ++k) {
                uint32_t hb = (uint32_t)tmp[p * rec + k] << 16, lb = rec == 64 ? (uint32_t)tmp[p * rec + 32 + k] << 16 : 0u;
                float hf, lf;
                memcpy(&hf, &hb, 4); memcpy(&lf, &lb, 4);
                dst[p * D + kc * CORR_CHUNK + k] = hf + lf;
            }
    }
    free(tmp);
    return st;
}

}  // extern "C"
