// Host side of the C ABI declared in include/corr.h: argument checks, the
// pyramid object and its device allocations, and the order in which the kernels
// of one build / one lookup are enqueued.
#include <new>
#include <string.h>
#include "corr_internal.h"

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
    return CORR_OK;
}

void fill_geometry(corr_pyramid* p) {
    const int BN = p->B * p->H * p->W;
    for (int l = 0; l < CORR_MAX_L; ++l) { p->Hl[l] = p->H >> l; p->Wl[l] = p->W >> l; }
    corr_fill_grid(&p->grid, p->H, p->W, p->L, CORR_R);
    p->nbins = p->B * 64 * p->grid.tnx * p->grid.tny;
    p->max_items = BN / CORR_GROUP + (p->nbins < BN ? p->nbins : BN) + 1;
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
    (void)hipFree(p->bin_count); (void)hipFree(p->bin_off); (void)hipFree(p->q_bin); (void)hipFree(p->q_rank);
    if (p->prof_ev) {
        for (int i = 0; i < CORR_PROF_LOOKUPS * 3; ++i) (void)hipEventDestroy(p->prof_ev[i]);
        delete[] p->prof_ev;
    }
    (void)hipFree(p->perm); (void)hipFree(p->items); (void)hipFree(p->n_items); (void)hipFree(p->stats);
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
        need(dev_alloc(&p->bin_count, (size_t)p->nbins, &p->bytes));
        need(dev_alloc(&p->bin_off, (size_t)p->nbins, &p->bytes));
        need(dev_alloc(&p->q_bin, BN, &p->bytes));
        need(dev_alloc(&p->q_rank, BN, &p->bytes));
        need(dev_alloc(&p->perm, BN, &p->bytes));
        need(dev_alloc(&p->items, (size_t)p->max_items, &p->bytes));
        need(dev_alloc(&p->n_items, (size_t)4, &p->bytes));
        need(dev_alloc(&p->stats, (size_t)CORR_NSTATS, &p->bytes));
        if (st == CORR_OK) {
            if (hipMemset(p->bin_count, 0, sizeof(int) * p->nbins) != hipSuccess ||
                hipMemset(p->stats, 0, sizeof(long long) * CORR_NSTATS) != hipSuccess ||
                hipMemset(p->n_items, 0, sizeof(int) * 4) != hipSuccess)
                st = CORR_ERR_HIP;
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
    }
    return "unknown status";
}

size_t corr_full_volume_bytes(int B, int H, int W, int L) {
    if (B <= 0 || H <= 0 || W <= 0 || !level_sizes_ok(H, W, L)) return 0;
    size_t px = 0;
    for (int l = 0; l < L; ++l) px += (size_t)(H >> l) * (W >> l);
    return (size_t)4 * B * H * W * px;
}

size_t corr_workspace_bytes(unsigned reps, int B, int H, int W, int D, int L) {
    if (check_dims(B, H, W, D, L) != CORR_OK) return 0;
    size_t bytes = feature_bytes(reps, B, H, W, D, L);
    if (reps & (CORR_REP_SPLIT | CORR_REP_BF16)) {
        corr_pyramid tmp;
        memset(&tmp, 0, sizeof(tmp));
        tmp.B = B; tmp.H = H; tmp.W = W; tmp.D = D; tmp.L = L;
        fill_geometry(&tmp);
        const size_t BN = (size_t)B * H * W;
        bytes += (size_t)tmp.nbins * 8 + BN * 12 + (size_t)tmp.max_items * 16 + 16 + CORR_NSTATS * 8;
    }
    return bytes;
}

size_t corr_pyramid_bytes(const corr_pyramid* pyr) { return pyr ? pyr->bytes : 0; }

corr_status corr_bin_geometry(int H, int W, int L, int l, int* cell_x, int* cell_y, int* window_x, int* window_y,
                              int* cells_x, int* cells_y) {
    if (H <= 0 || W <= 0 || !level_sizes_ok(H, W, L) || l < 0 || l >= L) return CORR_ERR_INVALID_ARG;
    CellGrid g;
    corr_fill_grid(&g, H, W, L, CORR_R);
    const int cx = ((1 << g.log_cx) >> l) > 1 ? ((1 << g.log_cx) >> l) : 1;
    const int cy = ((1 << g.log_cy) >> l) > 1 ? ((1 << g.log_cy) >> l) : 1;
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

corr_status corr_pyramid_destroy(corr_pyramid* pyr) {
    if (!pyr) return CORR_OK;
    const hipError_t e = hipDeviceSynchronize();
    free_all(pyr);
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_sample_mode(corr_mode mode, corr_precision prec, const float* fmap1, corr_pyramid* pyr,
                             const float* coords, int B, int H, int W, int D, int L, int r,
                             float* out, void* stream) {
    return corr_sample_layout(mode, prec, CORR_OUT_NCHW, fmap1, pyr, coords, B, H, W, D, L, r, out, stream);
}

corr_status corr_sample_layout(corr_mode mode, corr_precision prec, corr_out_layout layout, const float* fmap1,
                               corr_pyramid* pyr, const float* coords, int B, int H, int W, int D, int L, int r,
                               float* out, void* stream) {
    (void)fmap1;
    if (!pyr || !coords || !out) return CORR_ERR_INVALID_ARG;
    if (layout != CORR_OUT_NCHW && layout != CORR_OUT_NHWC) return CORR_ERR_INVALID_ARG;
    corr_status st = check_against(pyr, B, H, W, D, L);
    if (st != CORR_OK) return st;
    if (r < 1) return CORR_ERR_INVALID_ARG;
    if (r > 4) return CORR_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    pyr->out_nhwc = layout == CORR_OUT_NHWC;       // read by the launchers below
    switch (mode) {
        case CORR_MODE_BLOCK: {
            if (prec != CORR_PREC_BF16X3 && prec != CORR_PREC_BF16) return CORR_ERR_INVALID_ARG;
            if (!(pyr->built & (prec == CORR_PREC_BF16 ? (CORR_REP_SPLIT | CORR_REP_BF16) : CORR_REP_SPLIT)))
                return CORR_ERR_MISSING_REP;
            hipEvent_t* ev = nullptr;
            if (pyr->prof_on && pyr->prof_ev && pyr->prof_n < CORR_PROF_LOOKUPS)
                ev = pyr->prof_ev + (size_t)pyr->prof_n * 3;
            if (ev && hipEventRecord(ev[0], s) != hipSuccess) return CORR_ERR_HIP;
            e = launch_binning(pyr, coords, r, out, s);
            if (ev && e == hipSuccess) e = hipEventRecord(ev[1], s);
            if (e == hipSuccess)
                e = r == 1 ? launch_block_r1(pyr, coords, (int)prec, out, s)
                  : r == 2 ? launch_block_r2(pyr, coords, (int)prec, out, s)
                  : r == 3 ? launch_block_r3(pyr, coords, (int)prec, out, s)
                           : launch_block_r4(pyr, coords, (int)prec, out, s);
            if (ev && e == hipSuccess) e = hipEventRecord(ev[2], s);
            if (ev && e == hipSuccess) pyr->prof_n++;
            break;
        }
        case CORR_MODE_ONDEMAND: {
            if (!(pyr->built & CORR_REP_F32)) return CORR_ERR_MISSING_REP;
            e = launch_ondemand(pyr, coords, r, out, s);
            break;
        }
        case CORR_MODE_FULLVOLUME: {
            if (!(pyr->built & CORR_REP_F32)) return CORR_ERR_MISSING_REP;
            if (!pyr->vol_valid) {
                if (!pyr->vol[0]) {
                    const size_t need = corr_full_volume_bytes(B, H, W, L);
                    size_t free_b = 0, total_b = 0;
                    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) return CORR_ERR_HIP;
                    if (need + (256u << 20) > free_b) return CORR_ERR_OOM;
                    for (int l = 0; l < L; ++l) {
                        st = dev_alloc(&pyr->vol[l], (size_t)B * H * W * pyr->Hl[l] * pyr->Wl[l], &pyr->bytes);
                        if (st != CORR_OK) { free_volume(pyr); return st; }
                    }
                }
                e = launch_fullvol_build(pyr, s);
                if (e != hipSuccess) break;
                pyr->vol_valid = 1;
            }
            e = launch_fullvol_sample(pyr, coords, r, out, s);
            break;
        }
        default: return CORR_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? CORR_OK : CORR_ERR_HIP;
}

corr_status corr_sample(const float* fmap1, corr_pyramid* pyr, const float* coords,
                        int B, int H, int W, int D, int L, int r, float* out, void* stream) {
    return corr_sample_mode(CORR_MODE_BLOCK, CORR_PREC_BF16X3, fmap1, pyr, coords, B, H, W, D, L, r, out, stream);
}

corr_status corr_last_block_stats(corr_pyramid* pyr, corr_block_stats* stats, void* stream) {
    if (!pyr || !stats) return CORR_ERR_INVALID_ARG;
    if (!(pyr->reps & (CORR_REP_SPLIT | CORR_REP_BF16))) return CORR_ERR_MISSING_REP;
    long long h[CORR_NSTATS];
    int hn[4];
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_bin_stats(pyr, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipMemcpyAsync(h, pyr->stats, sizeof(h), hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
    if (hipMemcpyAsync(hn, pyr->n_items, sizeof(hn), hipMemcpyDeviceToHost, s) != hipSuccess) return CORR_ERR_HIP;
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

corr_status corr_profile_enable(corr_pyramid* pyr, int enable) {
    if (!pyr) return CORR_ERR_INVALID_ARG;
    if (enable && !pyr->prof_ev) {
        const int n = CORR_PROF_LOOKUPS * 3;
        pyr->prof_ev = new (std::nothrow) hipEvent_t[n];
        if (!pyr->prof_ev) return CORR_ERR_OOM;
        for (int i = 0; i < n; ++i)
            if (hipEventCreate(&pyr->prof_ev[i]) != hipSuccess) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(pyr->prof_ev[j]);
                delete[] pyr->prof_ev; pyr->prof_ev = nullptr;
                return CORR_ERR_HIP;
            }
    }
    pyr->prof_on = enable ? 1 : 0;
    pyr->prof_n = 0;
    return CORR_OK;
}

corr_status corr_profile_read(corr_pyramid* pyr, corr_profile* prof) {
    if (!pyr || !prof) return CORR_ERR_INVALID_ARG;
    memset(prof, 0, sizeof(*prof));
    if (!pyr->prof_ev) return CORR_OK;
    for (int i = 0; i < pyr->prof_n; ++i) {
        hipEvent_t* ev = pyr->prof_ev + (size_t)i * 3;
        if (hipEventSynchronize(ev[2]) != hipSuccess) return CORR_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[0], ev[1]) != hipSuccess) return CORR_ERR_HIP;
        prof->binning_ms += ms;
        if (hipEventElapsedTime(&ms, ev[1], ev[2]) != hipSuccess) return CORR_ERR_HIP;
        prof->block_ms += ms;
    }
    prof->lookups = pyr->prof_n;
    pyr->prof_n = 0;
    return CORR_OK;
}

}  // extern "C"
