// C-ABI run calls of libnpas: launch planning, single layers, glue layers and
// the stack runner.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <array>
#include <cstring>
#include <map>
#include <mutex>
#include <memory>

#include "npas_internal.h"

namespace npas {

static uint32_t magic_div(uint32_t d) { return d <= 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); }

// Best output tile of at most `max_pix` pixels for one launch: candidates are scored by
// how much of the MFMA columns and of the tile grid does useful work, then by halo
// overhead.  `max_vec` bounds the 16-byte vectors of one staged patch chunk (0 = no bound).
static bool pick_tile(const npas_packed *p, ConvGeom &g, int max_pix, int cols_small, size_t lds_budget, int nbuf,
                      size_t extra_lds, int max_vec, double *cover_out)
{
    const bool pointwise = p->KH == 1 && p->KW == 1;
    const int stride = g.stride;
    double best = -1e30;
    bool found = false;
    for (int TW = 1; TW <= std::min(g.Wo, max_pix); ++TW)
        for (int TH = 1; TH <= std::min(g.Ho, max_pix / TW); ++TH) {
            int PH = pointwise ? TH : (TH - 1) * stride + p->KH;
            int PW = pointwise ? TW : (TW - 1) * stride + p->KW;
            size_t lds = (((size_t)PH * PW * g.pitch + 15) / 16 * 16) * nbuf + extra_lds;
            if (lds > lds_budget) continue;
            if (max_vec && (long)PH * PW * (p->fmt.CC / 8) > max_vec) continue;
            int used_cols = TH * TW > cols_small ? max_pix : cols_small; // kernel instances walk fixed column counts
            double cover = (double)g.Ho * g.Wo /
                           ((double)((g.Ho + TH - 1) / TH) * ((g.Wo + TW - 1) / TW) * used_cols);
            double halo = (double)PH * PW / ((double)TH * TW);
            double score = cover - 0.05 * halo + 0.1 * ((double)used_cols / max_pix);
            if (score > best) {
                best = score;
                found = true;
                g.TH = TH; g.TW = TW; g.PH = PH; g.PW = PW;
                if (cover_out) *cover_out = cover;
            }
        }
    return found;
}

// Plans one conv launch: tile shape, grid, LDS bytes.  A workgroup owns TH x TW output
// pixels of one image and stages the matching input patch.
int plan_conv(const npas_packed *p, int N, int H, int W, int stride, int pad, ConvPlan *out)
{
    const DeviceFormat &d = p->fmt;
    ConvGeom g;
    memset(&g, 0, sizeof(g));
    g.KH = p->KH; g.KW = p->KW; g.stride = stride; g.pad = pad;
    g.C = p->C; g.F = p->F;
    const bool pointwise = p->KH == 1 && p->KW == 1;
    if (pointwise && stride == 1 && pad == 0) { // every pixel independent: flatten the batch
        g.N = 1; g.H = 1; g.W = N * H * W;
    } else {
        g.N = N; g.H = H; g.W = W;
    }
    g.Ho = (g.H + 2 * pad - p->KH) / stride + 1;
    g.Wo = (g.W + 2 * pad - p->KW) / stride + 1;
    g.pstep = pointwise ? stride : 1;
    g.lstep = pointwise ? 1 : stride;
    g.vec = (p->C % 8 == 0 && d.CC % 8 == 0) ? 1 : 0;
    const bool slab = d.variant == V_MFMA_SLAB;
    // LDS bytes per patch pixel: 16-byte aligned rows for the slab path's 16-byte reads,
    // rows displaced by 8 bytes for the element path's 2-byte gathers (bank spread)
    g.pitch = (d.CC * 2 + 15) / 16 * 16 + (slab ? 16 : 8);

    if (slab) {
        // persistent double-buffered kernel: two patch buffers, shapes listed at launch_slab_dt
        const size_t budget = 96 * 1024;
        const int max_vec = 256 * 8;
        ConvGeom g128 = g, g64 = g;
        double c128 = 0, c64 = 0;
        if (d.NT == 2) {
            g.shape = 2;
            if (!pick_tile(p, g, 128, 128, budget, 2, 0, max_vec, nullptr)) goto nofit;
        } else if (p->F <= 64) {
            g.shape = 1;
            if (!pick_tile(p, g, 128, 128, budget, 2, 0, max_vec, nullptr)) goto nofit;
        } else {
            bool ok128 = pick_tile(p, g128, 128, 128, budget, 2, 0, max_vec, &c128);
            bool ok64 = pick_tile(p, g64, 64, 64, budget, 2, 0, max_vec, &c64);
            if (!ok128 && !ok64) goto nofit;
            long items128 = ok128 ? (long)g128.N * ((g128.Ho + g128.TH - 1) / g128.TH) * ((g128.Wo + g128.TW - 1) / g128.TW) : 0;
            // the wider tile unless it wastes MFMA columns or leaves most of the chip idle
            bool use64 = !ok128 || (ok64 && (c64 > 1.15 * c128 || items128 * ((p->F + 127) / 128) < 256));
            g = use64 ? g64 : g128;
            g.shape = use64 ? 3 : 0;
        }
        const int wgf = (g.shape == 0 || g.shape == 3) ? 2 : 1;
        g.tilesY = (g.Ho + g.TH - 1) / g.TH;
        g.tilesX = (g.Wo + g.TW - 1) / g.TW;
        g.div_tw = magic_div(g.TW);
        g.div_pw = magic_div(g.PW);
        g.div_vec = magic_div(std::max(1, d.CC / 8));
        g.div_pitch = magic_div(g.pitch);
        g.nfsplit = (d.ntiles + wgf - 1) / wgf; // filter blocks per pixel tile
        g.tiles_per_split = wgf;
        const long items = (long)g.N * g.tilesY * g.tilesX * g.nfsplit;
        out->g = g;
        {
            const bool small = g.PH * g.PW * (d.CC / 8) <= 1024;
            const int occ = g.shape == 0 ? 2 : (small ? (g.shape == 2 ? 4 : 3) : (g.shape == 2 ? 3 : 2));
            out->grid = (unsigned)std::min<long>(items, 256L * occ);
        }
        out->lds_bytes = (((size_t)g.PH * g.PW * g.pitch + 15) / 16 * 16) * 2;
        return NPAS_OK;
    }
    {
        g.koff_cap = std::min(512, std::max(32, d.max_list));
        const size_t koff_bytes = (size_t)4 * g.koff_cap * 4;
        if (!pick_tile(p, g, 128, 64, 64 * 1024, 1, koff_bytes, 0, nullptr)) goto nofit;
        g.tilesY = (g.Ho + g.TH - 1) / g.TH;
        g.tilesX = (g.Wo + g.TW - 1) / g.TW;
        g.div_tw = magic_div(g.TW);
        g.div_pw = magic_div(g.PW);
        g.div_vec = magic_div(std::max(1, d.CC / 8));
        const long ptiles = (long)g.N * g.tilesY * g.tilesX;
        const int quads = (d.ntiles + 3) / 4; // filter tiles are walked four at a time (one per wave)
        int nfsplit;
        if (d.nchunks > 1) nfsplit = quads; // accumulators live across chunks: one quad per workgroup
        else {
            long want = (2048 + ptiles - 1) / ptiles; // aim for >= 2048 workgroups
            nfsplit = (int)std::max(1L, std::min<long>(quads, want));
        }
        int quads_per = (quads + nfsplit - 1) / nfsplit;
        nfsplit = (quads + quads_per - 1) / quads_per;
        g.nfsplit = nfsplit;
        g.tiles_per_split = quads_per * 4;
        out->g = g;
        out->grid = (unsigned)(ptiles * nfsplit);
        out->lds_bytes = ((size_t)g.PH * g.PW * g.pitch + 15) / 16 * 16 + koff_bytes;
        return NPAS_OK;
    }
nofit:
    set_error("no output tile fits in LDS (kernel %dx%d stride %d)", p->KH, p->KW, stride);
    return NPAS_E_SHAPE;
}

static int check_run(const npas_packed *p, const void *x, void *y, int N, int H, int W, int stride, int pad)
{
    if (!p || !x || !y) {
        set_error("NULL argument (handle=%p x_dev=%p y_dev=%p)", (const void *)p, x, y);
        return NPAS_E_NULL;
    }
    if (p->scheme == NPAS_SCHEME_DEPTHWISE) {
        set_error("a depthwise handle runs through npas_depthwise3x3, not the convolution / FC calls");
        return NPAS_E_SHAPE;
    }
    if (N <= 0 || H <= 0 || W <= 0 || stride <= 0 || pad < 0) {
        set_error("bad geometry N=%d H=%d W=%d stride=%d pad=%d", N, H, W, stride, pad);
        return NPAS_E_SHAPE;
    }
    int Ho = (H + 2 * pad - p->KH) / stride + 1, Wo = (W + 2 * pad - p->KW) / stride + 1;
    if (H + 2 * pad < p->KH || W + 2 * pad < p->KW || Ho <= 0 || Wo <= 0) {
        set_error("empty output for input %dx%d, kernel %dx%d, stride %d, pad %d", H, W, p->KH, p->KW, stride, pad);
        return NPAS_E_SHAPE;
    }
    if ((double)N * H * W * p->C > 2147483647.0 || (double)N * Ho * Wo * p->F > 2147483647.0) {
        set_error("tensor has more than 2^31-1 elements");
        return NPAS_E_SHAPE;
    }
    if (p->dev.device < 0) {
        set_error("packed layer has no device copy (packed on a machine without a GPU)");
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// Output tile of the k x k streaming kernel: NI images x TH x TW output pixels (at most 256,
// the MFMA columns of a workgroup) whose halo patch fits the kernel's limits.  Picks the
// plan with the best ratio of useful to computed columns, then the smaller halo.  Returns
// false when no plan exists or the launch would leave most of the chip idle (the slab
// kernel's smaller tiles serve those cases better).
static bool plan_spatial_search(const npas_packed *p, int N, int H, int W, int pad, int stride, bool force, int maxpix, SpatialRingArgs *a);

// The search is a few thousand candidates; its result depends only on the shapes, so it is
// kept per shape (launches of a stack repeat the same few shapes).
bool plan_spatial(const npas_packed *p, int N, int H, int W, int pad, int stride, SpatialRingArgs *a)
{
    static std::mutex mu;
    static std::map<std::array<int, 11>, std::pair<bool, SpatialRingArgs>> cache;
    // forced (tests): take this kernel whenever a plan exists
    const int force = switches().force == FV_SPATIAL;
    const std::array<int, 11> key = {p->KH, p->KW, p->C, p->F, p->ring.nfb, N, H, W, pad, force, stride};
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it == cache.end()) {
        SpatialRingArgs g;
        std::memset(&g, 0, sizeof g);
        // 256-pixel tiles; if those would leave most of the chip idle, 128-pixel tiles (half the multiplying waves)
        // (stride 2: 128-pixel tiles only, the four phase planes of a 256-pixel tile do not fit)
        bool ok = stride == 1 && plan_spatial_search(p, N, H, W, pad, stride, false, 256, &g);
        if (!ok) ok = plan_spatial_search(p, N, H, W, pad, stride, false, 128, &g);
        if (!ok && force) ok = plan_spatial_search(p, N, H, W, pad, stride, true, stride == 1 ? 256 : 128, &g);
        it = cache.emplace(key, std::make_pair(ok, g)).first;
    }
    *a = it->second.second;
    return it->second.first;
}

static bool plan_spatial_search(const npas_packed *p, int N, int H, int W, int pad, int stride, bool force, int maxpix, SpatialRingArgs *a)
{
    const int KH = p->KH, KW = p->KW, T = KH * KW;
    const bool s2 = stride == 2; // 3 x 3, pad 1: four phase planes of (TH + 1) x (TW + 1) pixels, one copy
    if (stride != 1 && !(s2 && KH == 3 && KW == 3 && pad == 1)) return false;
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
    const int lds_total = 160 * 1024 - 2048 /* bias buffers */ - (s2 ? 4096 : 2048) /* patch pixel table */ - 1024 /* tile pixel table */, wstage = 16384;
    const int nbuf = s2 ? 4 : 2; // patch buffers (planes) of npb KB each
    const int max_npb = std::min(s2 ? 124 : 1 << 20, (lds_total - 3 * wstage) / (1024 * nbuf));
    if (T < 2 || p->C % 64 != 0 || Ho <= 0 || Wo <= 0 || (long)N * H * W >= (1L << 24)) return false; // (the kernel forms patch addresses with 24-bit multiplies)
    double best = -1.0;
    int bNI = 0, bTH = 0, bTW = 0;
    for (int TH = 1; TH <= std::min(Ho, 255); ++TH)
        for (int TW = 1; TW <= std::min(Wo, 255) && TH * TW <= maxpix; ++TW) {
            const int PH = s2 ? TH + 1 : TH + KH - 1, PW = s2 ? TW + 1 : TW + KW - 1;
            const long ty = (Ho + TH - 1) / TH, tx = (Wo + TW - 1) / TW;
            const int maxNI = std::min(N, maxpix / (TH * TW));
            for (int NI = 1; NI <= maxNI; ++NI) {
                const int npb = (NI * PH * PW + 7) / 8;
                if (npb > max_npb) break;
                const long tn = (N + NI - 1) / NI;
                const int depth = std::min(6, (lds_total - 1024 * nbuf * npb) / wstage);
                const double eff = (double)N * Ho * Wo / ((double)tn * ty * tx * (double)maxpix);
                const double halo = (double)(NI * PH * PW) / (double)(NI * TH * TW);
                const double score = eff - 0.02 * halo + 0.02 * (depth - 3);
                if (score > best) {
                    best = score;
                    bNI = NI; bTH = TH; bTW = TW;
                }
            }
        }
    if (best < 0) return false;
    a->N = N; a->H = H; a->W = W; a->C = p->C; a->F = p->F; a->Ho = Ho; a->Wo = Wo;
    a->KH = KH; a->KW = KW; a->pad = pad; a->stride = stride;
    a->pg = maxpix / 64;
    a->NI = bNI; a->TH = bTH; a->TW = bTW; a->PH = s2 ? bTH + 1 : bTH + KH - 1; a->PW = s2 ? bTW + 1 : bTW + KW - 1;
    a->tilesN = (N + bNI - 1) / bNI; a->tilesY = (Ho + bTH - 1) / bTH; a->tilesX = (Wo + bTW - 1) / bTW;
    a->nfb = p->ring.nfb;
    a->npb = (bNI * a->PH * a->PW + 7) / 8;
    a->depth = std::min(6, (lds_total - 1024 * nbuf * a->npb) / wstage);
    a->div_tw = magic_div((uint32_t)bTW); a->div_pw = magic_div((uint32_t)a->PW);
    a->div_thtw = magic_div((uint32_t)(bTH * bTW)); a->div_phpw = magic_div((uint32_t)(a->PH * a->PW));
    const long items = (long)a->tilesN * a->tilesY * a->tilesX * a->nfb;
    const double eff = (double)N * Ho * Wo / ((double)a->tilesN * a->tilesY * a->tilesX * (double)maxpix);
    // worth it when the launch fills most of the chip and neither the 256 pixel columns nor the
    // 128 filter rows of a workgroup are mostly padding (measured against the slab kernel)
    const double fill = (double)p->F / (128.0 * a->nfb);
    // with 128-pixel tiles a long reduction (many stages per item) pays from fewer items on: the slab kernel's
    // workgroups would walk it with one step of lookahead (512 -> 512 at 7 x 7, batch 32: 64 items, 64 -> 47 us)
    // (at stride 2 only from 64 stages per item on: 256 -> 256 onto 14 x 14 at batch 32, 100 items of 36 stages, 32 against 27 us)
    const bool enough = items >= 192 || (maxpix == 128 && items >= 48 && items * (p->C / 64) * T >= 3000 && (!s2 || (p->C / 64) * T >= 64));
    return force || (enough && eff >= 0.6 && fill >= 0.75);
}

// Tile plan of the resident-weights k x k kernel (at most 64 filters, all weight stages in LDS): the
// spatial ring's search with the LDS that the weights leave, scored by useful columns times how evenly the
// items fill rounds of 256 workgroups.  False when the weights do not fit or the launch is too small.
bool plan_resident(const npas_packed *p, int N, int H, int W, int pad, SpatialRingArgs *a)
{
    struct Entry { bool fits, worth; SpatialRingArgs g; };
    static std::mutex mu;
    static std::map<std::array<int, 8>, Entry> cache;
    const std::array<int, 8> key = {p->KH, p->KW, p->C, p->F, N, H, W, pad};
    const bool force = switches().force == FV_RESIDENT; // tests: take this kernel whenever a plan exists
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it != cache.end()) {
        *a = it->second.g;
        return it->second.fits && (force || it->second.worth);
    }
    SpatialRingArgs g;
    std::memset(&g, 0, sizeof g);
    const int KH = p->KH, KW = p->KW, T = KH * KW;
    const int Ho = H + 2 * pad - KH + 1, Wo = W + 2 * pad - KW + 1;
    bool ok = T >= 2 && p->C % 64 == 0 && p->F <= 64 && p->ring.present && Ho > 0 && Wo > 0;
    const int nst = ok ? (p->C / 64) * T : 0;
    double best = -1e30;
    int bNI = 0, bTH = 0, bTW = 0;
    if (ok && spatial_resident_lds_bytes(8, nst) <= 160 * 1024) {
        for (int TH = 1; TH <= std::min(Ho, 255); ++TH)
            for (int TW = 1; TW <= std::min(Wo, 255) && TH * TW <= 256; ++TW) {
                const int PH = TH + KH - 1, PW = TW + KW - 1;
                const long ty = (Ho + TH - 1) / TH, tx = (Wo + TW - 1) / TW;
                const int maxNI = std::min(N, 256 / (TH * TW));
                for (int NI = 1; NI <= maxNI; ++NI) {
                    const int npb = (NI * PH * PW + 7) / 8;
                    if (spatial_resident_lds_bytes(npb, nst) > 160 * 1024) break;
                    const long items = (long)((N + NI - 1) / NI) * ty * tx;
                    const double eff = (double)N * Ho * Wo / ((double)items * 256.0);
                    const double rounds = (double)items / (double)((items + 255) / 256 * 256);
                    const double halo = (double)(PH * PW) / (double)(TH * TW);
                    const double score = eff * rounds - 0.02 * halo;
                    if (score > best) {
                        best = score;
                        bNI = NI; bTH = TH; bTW = TW;
                    }
                }
            }
    }
    ok = ok && bNI > 0;
    bool worth = false;
    if (ok) {
        g.N = N; g.H = H; g.W = W; g.C = p->C; g.F = p->F; g.Ho = Ho; g.Wo = Wo;
        g.KH = KH; g.KW = KW; g.pad = pad;
        g.pg = 4; g.stride = 1;
        g.NI = bNI; g.TH = bTH; g.TW = bTW; g.PH = bTH + KH - 1; g.PW = bTW + KW - 1;
        g.tilesN = (N + bNI - 1) / bNI; g.tilesY = (Ho + bTH - 1) / bTH; g.tilesX = (Wo + bTW - 1) / bTW;
        g.nfb = 1;
        g.npb = (bNI * g.PH * g.PW + 7) / 8;
        g.depth = nst;
        g.div_tw = magic_div((uint32_t)bTW); g.div_pw = magic_div((uint32_t)g.PW);
        g.div_thtw = magic_div((uint32_t)(bTH * bTW)); g.div_phpw = magic_div((uint32_t)(g.PH * g.PW));
        const long items = (long)g.tilesN * g.tilesY * g.tilesX;
        const double eff = (double)N * Ho * Wo / ((double)items * 256.0);
        worth = items >= 192 && eff >= 0.6;
    }
    cache.emplace(key, Entry{ok, worth, g});
    *a = g;
    return ok && (force || worth);
}

// Which kernel a run call launches for this layer and geometry.
enum Route { R_VALU, R_WAVE_F32, R_FC_GATHER, R_POINTWISE_RING, R_SPATIAL_RING, R_SPATIAL_RESIDENT, R_SMALLC, R_SMALLM, R_SLAB, R_GATHER };

// Tile and patch of a small-channel launch: TH x TW = 256 output pixels with the fewest computed-but-
// unused ones, the patch within 48 KB of LDS.  False when no tile shape fits.
static bool plan_smallc(const npas_packed *p, int N, int H, int W, int stride, int pad, SmallCArgs *a)
{
    const int Ho = (H + 2 * pad - p->KH) / stride + 1, Wo = (W + 2 * pad - p->KW) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return false;
    long best = -1;
    for (int th = 1; th <= 256; th *= 2) {
        const int tw = 256 / th;
        const int ph = (th - 1) * stride + p->KH, pw = (tw - 1) * stride + p->KW;
        const int pitch = (pw * p->C * 2 + 3) / 4 * 4 + 4;
        if ((long)ph * pitch > 48 * 1024 || (long)ph * pw * p->C > 256 * 24 || (long)ph * ((pw * p->C + 2) / 2) > 128 * 24) continue; // LDS, and 24 staged values (12 words) per thread
        const int ty = (Ho + th - 1) / th, tx = (Wo + tw - 1) / tw;
        const long cost = (long)ty * tx * 4096 + std::abs(th - tw); // tiles first, then the squarer shape (smaller patch)
        if (best < 0 || cost < best) {
            best = cost;
            a->TH = th; a->TW = tw; a->tilesY = ty; a->tilesX = tx; a->PH = ph; a->PW = pw; a->pitch = pitch;
        }
    }
    if (best < 0) return false;
    a->pool = 0; a->PTH = a->PTW = a->PHo = a->PWo = 0; a->div_ptw = 0;
    a->N = N; a->H = H; a->W = W; a->C = p->C; a->F = p->F; a->Ho = Ho; a->Wo = Wo;
    a->KH = p->KH; a->KW = p->KW; a->stride = stride; a->pad = pad;
    a->K = p->C * p->KH * p->KW; a->nsteps = p->smallc.nsteps;
    a->nitems = (uint32_t)N * (uint32_t)(a->tilesY * a->tilesX);
    a->div_tw = magic_div((uint32_t)a->TW);
    a->div_kwc = magic_div((uint32_t)(p->KW * p->C));
    a->div_rowlen = magic_div((uint32_t)(a->PW * p->C));
    a->row2 = (a->PW * p->C + 2) / 2; // the row's values plus one of slack for an odd start, in words
    a->div_row2 = magic_div((uint32_t)a->row2);
    a->div_tiles = magic_div((uint32_t)(a->tilesY * a->tilesX));
    a->div_tx = magic_div((uint32_t)a->tilesX);
    return true;
}

// The same kernel with the 3 x 3 / stride 2 / pad 1 max pool that follows done inside it: tiles of 8 x 7 pooled
// pixels = 17 x 15 conv pixels (255 of the kernel's 256 operand rows; neighbouring tiles share one conv row and
// column, 14 % more multiplies for a conv output that never reaches memory).
static bool plan_smallc_pool(const npas_packed *p, int N, int H, int W, int stride, int pad, SmallCArgs *a)
{
    const int Ho = (H + 2 * pad - p->KH) / stride + 1, Wo = (W + 2 * pad - p->KW) / stride + 1;
    if (!p->smallc.present || Ho <= 0 || Wo <= 0) return false;
    std::memset(a, 0, sizeof *a);
    a->pool = 1; a->PTH = 8; a->PTW = 7;
    a->PHo = (Ho - 1) / 2 + 1; a->PWo = (Wo - 1) / 2 + 1;
    a->TH = 2 * a->PTH + 1; a->TW = 2 * a->PTW + 1;
    a->tilesY = (a->PHo + a->PTH - 1) / a->PTH; a->tilesX = (a->PWo + a->PTW - 1) / a->PTW;
    a->PH = (a->TH - 1) * stride + p->KH; a->PW = (a->TW - 1) * stride + p->KW;
    a->pitch = (a->PW * p->C * 2 + 3) / 4 * 4 + 4;
    if ((long)a->PH * a->pitch > 48 * 1024 || (long)a->PH * a->PW * p->C > 256 * 24 || (long)a->PH * ((a->PW * p->C + 2) / 2) > 128 * 24) return false;
    a->N = N; a->H = H; a->W = W; a->C = p->C; a->F = p->F; a->Ho = Ho; a->Wo = Wo;
    a->KH = p->KH; a->KW = p->KW; a->stride = stride; a->pad = pad;
    a->K = p->C * p->KH * p->KW; a->nsteps = p->smallc.nsteps;
    a->nitems = (uint32_t)N * (uint32_t)(a->tilesY * a->tilesX);
    a->div_tw = magic_div((uint32_t)a->TW);
    a->div_ptw = magic_div((uint32_t)a->PTW);
    a->div_kwc = magic_div((uint32_t)(p->KW * p->C));
    a->div_rowlen = magic_div((uint32_t)(a->PW * p->C));
    a->row2 = (a->PW * p->C + 2) / 2;
    a->div_row2 = magic_div((uint32_t)a->row2);
    a->div_tiles = magic_div((uint32_t)(a->tilesY * a->tilesX));
    a->div_tx = magic_div((uint32_t)a->tilesX);
    return true;
}

// conv (small-channel kernel) + max pool 3 x 3 / 2 as one launch; y is the pooled tensor
int run_conv_maxpool(const npas_packed *p, const void *x, void *y, int N, int H, int W, int stride, int pad, const void *bias,
                     int act, void *stream)
{
    SmallCArgs sc;
    if (!plan_smallc_pool(p, N, H, W, stride, pad, &sc)) {
        set_error("conv + max pool: the layer does not fit the small-channel kernel");
        return NPAS_E_SHAPE;
    }
    sc.x = x; sc.y = y; sc.residual = nullptr; sc.bias = (const float *)bias;
    sc.wimg = p->dev.scimg;
    sc.act = act;
    return launch_conv_smallc(p->dtype, sc, stream);
}

static Route choose_route(const npas_packed *p, int N, int H, int W, int stride, int pad, SpatialRingArgs *sp,
                          SmallCArgs *sc = nullptr)
{
    if (p->fmt.variant == V_VALU_F32) {
        // few lanes in all (a small layer: the launch is a chain of load latencies): split every reduction over 8 lanes
        const long Ho0 = (H + 2 * pad - p->KH) / stride + 1, Wo0 = (W + 2 * pad - p->KW) / stride + 1;
        const bool small = (double)N * Ho0 * Wo0 * p->fmt.nvg * 8.0 <= 4.0 * 1024 * 1024;
        return p->wavef.present && small && switches().force != FV_VALU ? R_WAVE_F32 : R_VALU;
    }
    // sparse 1x1 / FC layer on few pixels: the exact per-tile lists (nothing pruned is multiplied, compact weights)
    if (p->fc.present && p->KH == 1 && p->KW == 1 && pad == 0 && switches().force != FV_NOFCGATHER) {
        const long M0 = (long)N * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
        if (M0 <= 1024) return R_FC_GATHER;
    }
    SmallCArgs sc_local;
    if (p->smallc.present && plan_smallc(p, N, H, W, stride, pad, sc ? sc : &sc_local)) return R_SMALLC;
    // A gather-format layer (few surviving positions) leaves the ring kernels, which multiply
    // everything, only the launches they win (measured on the 3x3 256 -> 256 rate sweep and the
    // 16 x 32-block FC layer): those above 1/8 density.
    const bool gather = p->fmt.variant == V_MFMA_GATHER;
    const bool ring_ok = p->ring.present && (!gather || p->fmt.density >= 0.125);
    if (ring_ok && p->KH == 1 && p->KW == 1 && pad == 0) {
        // up to 256 output pixels (batch 1 from the 14 x 14 stage on, FC layers) the kernel that splits the
        // reduction over a workgroup's waves is faster than the ring's smallest tiles (measured layer by layer)
        const long Ho1 = (H - 1) / stride + 1, Wo1 = (W - 1) / stride + 1;
        // (beyond that while its workgroups, 64 pixels x 16 filters each, still fit one round: 2048 -> 512 at 7 x 7,
        // batch 8: 18.4 -> 11.6 us; with more workgroups than that it loses, 512 -> 2048 at the same size: 9.3 -> 21 us)
        const long M1 = (long)N * Ho1 * Wo1;
        if (M1 <= 256 || (p->C >= 1024 && ((M1 + 63) / 64) * ((p->F + 15) / 16) <= 256)) return R_SMALLM; // (and the reduction long)
        return R_POINTWISE_RING;
    }
    const int fv = switches().force;
    if (ring_ok && stride == 1 && (p->KH > 1 || p->KW > 1) && p->F <= 64 && fv != FV_NORESIDENT && plan_resident(p, N, H, W, pad, sp))
        return R_SPATIAL_RESIDENT;
    {
        const bool s2_off = stride == 2 && fv == FV_NOSPATIAL2;
        if (ring_ok && (stride == 1 || stride == 2) && !s2_off && (p->KH > 1 || p->KW > 1) && plan_spatial(p, N, H, W, pad, stride, sp))
            return R_SPATIAL_RING;
    }
    // few output pixels (small batch, late stages): the tiled kernels would run a handful of workgroups, each
    // walking the whole reduction alone; split the reduction over the waves of many small workgroups instead
    if (ring_ok && (p->KH > 1 || p->KW > 1)) {
        const long Ho = (H + 2 * pad - p->KH) / stride + 1, Wo = (W + 2 * pad - p->KW) / stride + 1;
        const bool force = fv == FV_SMALLM;
        // ... or little work altogether (a 56 x 56 x 64 -> 64 layer at batch 1: 5.8 against 8.8 us)
        const double macs = (double)N * Ho * Wo * p->F * p->C * p->KH * p->KW;
        if (Ho > 0 && Wo > 0 && (force || (long)N * Ho * Wo <= 1024 || macs <= 200e6)) return R_SMALLM;
    }
    return gather ? R_GATHER : R_SLAB;
}

const char *route_name(const npas_packed *p, int N, int H, int W, int stride, int pad)
{
    SpatialRingArgs sp;
    switch (choose_route(p, N, H, W, stride, pad, &sp)) {
    case R_VALU: return "conv_valu_f32";
    case R_WAVE_F32: return "conv_wave_f32";
    case R_FC_GATHER: return "fc_gather_mfma";
    case R_POINTWISE_RING: return "pointwise_ring";
    case R_SPATIAL_RING: return "spatial_ring";
    case R_SPATIAL_RESIDENT: return "spatial_resident";
    case R_SMALLC: return "conv_smallc_mfma";
    case R_SMALLM: return "conv_smallm_mfma";
    case R_SLAB: return "conv_slab_mfma";
    default: return "conv_gather_mfma";
    }
}

int run_conv(const npas_packed *p, const ConvPlan *plan, const void *x, void *y, int N, int H, int W, int stride,
             int pad, const void *bias, const void *residual, int act, void *stream)
{
    if (!valid_act(act)) {
        set_error("unknown activation %d", act);
        return NPAS_E_SHAPE;
    }
    SpatialRingArgs sp;
    SmallCArgs sc;
    const Route route = choose_route(p, N, H, W, stride, pad, &sp, &sc);
    if (route == R_SMALLC) { // fewer than 8 input channels: whole reduction in a few MFMA steps
        sc.x = x; sc.y = y; sc.residual = residual; sc.bias = (const float *)bias;
        sc.wimg = p->dev.scimg;
        sc.act = act;
        return launch_conv_smallc(p->dtype, sc, stream);
    }
    if (route == R_SMALLM) {
        SmallMArgs a;
        a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias; a.wimg = p->dev.wimg;
        a.N = N; a.H = H; a.W = W; a.C = p->C; a.F = p->F;
        a.Ho = (H + 2 * pad - p->KH) / stride + 1; a.Wo = (W + 2 * pad - p->KW) / stride + 1;
        a.KH = p->KH; a.KW = p->KW; a.stride = stride; a.pad = pad; a.act = act;
        a.M = N * a.Ho * a.Wo;
        a.nptiles = (a.M + 63) / 64;
        a.nimg = p->ring.nfb * 8;
        a.div_howo = magic_div((uint32_t)(a.Ho * a.Wo)); a.div_wo = magic_div((uint32_t)a.Wo);
        a.div_kw = magic_div((uint32_t)p->KW); a.div_T2 = magic_div((uint32_t)(2 * p->KH * p->KW));
        return launch_conv_smallm(p->dtype, a, stream);
    }
    if (route == R_FC_GATHER) {
        FcGatherArgs a;
        a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
        a.tptr = p->dev.fc_tptr; a.koff = p->dev.fc_koff; a.wimg = p->dev.fc_wimg;
        a.C = p->C; a.F = p->F; a.ntiles = p->fc.ntiles; a.act = act;
        a.H = H; a.W = W; a.stride = stride;
        a.Ho = (H - 1) / stride + 1; a.Wo = (W - 1) / stride + 1;
        a.M = N * a.Ho * a.Wo;
        a.pitch = 2 * p->C + 8;
        a.div_howo = magic_div((uint32_t)(a.Ho * a.Wo)); a.div_wo = magic_div((uint32_t)a.Wo);
        const long nptiles = (a.M + 15) / 16;
        // eight waves per workgroup = tiles x runs of a tile's list: as few tiles (as many runs) as keeps the
        // launch within about two workgroups per CU (each stages the 16 activation rows again)
        a.tiles_per_wg = 8;
        for (int tpw = 1; tpw < 8; tpw *= 2)
            if (nptiles * ((a.ntiles + tpw - 1) / tpw) <= 512) {
                a.tiles_per_wg = tpw;
                break;
            }
        return launch_fc_gather(p->dtype, a, stream);
    }
    if (route == R_WAVE_F32) {
        WaveF32Args a;
        a.x = (const float *)x; a.y = (float *)y; a.residual = (const float *)residual; a.bias = (const float *)bias;
        a.wg_ptr = p->dev.wv_ptr; a.vg_f0 = p->dev.vg_f0; a.kent = p->dev.wv_kent; a.w = p->dev.wv_w;
        a.nvg = p->fmt.nvg; a.VB = p->fmt.VB;
        a.N = N; a.H = H; a.W = W; a.C = p->C; a.F = p->F;
        a.Ho = (H + 2 * pad - p->KH) / stride + 1; a.Wo = (W + 2 * pad - p->KW) / stride + 1;
        a.KH = p->KH; a.KW = p->KW; a.stride = stride; a.pad = pad; a.act = act;
        return launch_conv_wave_f32(a, stream);
    }
    if (route == R_VALU) {
        ConvValuArgs a;
        a.x = (const float *)x; a.y = (float *)y; a.residual = (const float *)residual; a.bias = (const float *)bias;
        a.vg_ptr = p->dev.vg_ptr; a.vg_f0 = p->dev.vg_f0; a.vkent = p->dev.vkent; a.vw = p->dev.vw;
        a.nvg = p->fmt.nvg; a.VB = p->fmt.VB;
        a.N = N; a.H = H; a.W = W; a.C = p->C; a.F = p->F;
        a.Ho = (H + 2 * pad - p->KH) / stride + 1; a.Wo = (W + 2 * pad - p->KW) / stride + 1;
        a.KH = p->KH; a.KW = p->KW; a.stride = stride; a.pad = pad; a.act = act;
        return launch_conv_valu(a, stream);
    }
    if (route == R_POINTWISE_RING) { // streaming 1x1 path
        RingArgs a;
        a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
        a.rg_ptr = p->dev.rg_ptr; a.rg_chunk = p->dev.rg_chunk; a.wimg = p->dev.wimg;
        a.C = p->C; a.F = p->F;
        a.H = H; a.W = W; a.stride = stride;
        a.Ho = (H - 1) / stride + 1; a.Wo = (W - 1) / stride + 1;
        a.M = N * a.Ho * a.Wo;
        a.nptiles = (a.M + 255) / 256;
        a.nfb = p->ring.nfb;
        a.small = 0;
        const long items_small = (long)((a.M + 63) / 64) * ((p->F + 63) / 64), items_med = (long)((a.M + 127) / 128) * a.nfb;
        if ((long)a.nptiles * a.nfb < 96 && items_small > 256 && items_med <= 256) {
            // ... unless those take two rounds where 128 x 128 tiles (four multiplying waves instead of one) take
            // one: a stage costs about the same in both (1024 -> 256 at 14 x 14, batch 32: 19.9 -> 11.2 us)
            a.small = 2;
            a.nptiles = (a.M + 127) / 128;
        } else if ((long)a.nptiles * a.nfb < 96) { // most CUs would get no tile: smaller tiles, deeper ring
            a.small = 1;
            a.nptiles = (a.M + 63) / 64;
            a.nfb = (p->F + 63) / 64;
        } else {
            // 128 x 128 items (a little more than half the time of a 256 x 128 one: the weights are fetched
            // per 128 pixels) when they divide over the 256 workgroups with fewer idle slots
            const long big = (long)a.nptiles * a.nfb, med = (long)((a.M + 127) / 128) * a.nfb;
            const double t_big = (double)((big + 255) / 256), t_med = 0.56 * (double)((med + 255) / 256);
            if (t_med < 0.75 * t_big) {
                a.small = 2;
                a.nptiles = (a.M + 127) / 128;
            }
        }
        // Items of equal size in whole rounds: with the number of rounds the full tiles need, as many pixel
        // tiles as fill those rounds, each of P <= tile height pixels (784 items of 256 pixels on 256
        // workgroups are 4 rounds, the last all but empty; 1008 items of 200 pixels are 4 rounds of 200).
        const int th = a.small == 1 ? 64 : a.small == 2 ? 128 : 256;
        a.P = th;
        if (a.small != 1 && !switches().no_balance) {
            const long rounds = ((long)a.nptiles * a.nfb + 255) / 256;
            const long want = rounds * 256 / a.nfb; // pixel tiles that fill the rounds
            if (want > a.nptiles) {
                const int pp = (int)((a.M + want - 1) / want);
                a.P = std::max(th / 2, std::min(th, (pp + 7) / 8 * 8));
                a.nptiles = (a.M + a.P - 1) / a.P;
            }
        }
        a.act = act;
        a.flat = stride == 1;
        a.div_howo = magic_div((uint32_t)(a.Ho * a.Wo));
        a.div_wo = magic_div((uint32_t)a.Wo);
        return launch_pointwise_ring(p->dtype, a, stream);
    }
    if (route == R_SPATIAL_RESIDENT) { // k x k, at most 64 filters: all weights stay in LDS
        SpatialRingArgs &a = sp;
        a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
        a.wimg = p->dev.wimg; a.zeros = p->dev.zeros;
        a.act = act;
        return launch_spatial_resident(p->dtype, a, stream);
    }
    if (route == R_SPATIAL_RING) { // k x k streaming path, when a tile plan fills the chip
        SpatialRingArgs &a = sp;
        a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
        a.wimg = p->dev.wimg; a.zeros = p->dev.zeros;
        a.act = act;
        return launch_spatial_ring(p->dtype, a, stream);
    }
    std::shared_ptr<const ConvPlan> cached;
    if (!plan) { // plans are kept per handle and geometry: a stack repeats the same launches call after call
        const std::array<int, 5> key = {N, H, W, stride, pad};
        std::lock_guard<std::mutex> lock(p->plan_mu);
        for (const auto &e : p->plans)
            if (e.first == key) cached = e.second;
        if (!cached) {
            auto fresh = std::make_shared<ConvPlan>();
            int rc = plan_conv(p, N, H, W, stride, pad, fresh.get());
            if (rc) return rc;
            if (p->plans.size() >= 16) p->plans.erase(p->plans.begin());
            p->plans.emplace_back(key, fresh);
            cached = fresh;
        }
        plan = cached.get();
    }
    ConvMfmaArgs a;
    a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
    a.tc_ptr = p->dev.tc_ptr; a.kent = p->dev.kent; a.wfrag = p->dev.wfrag;
    a.CC = p->fmt.CC; a.nchunks = p->fmt.nchunks; a.ntiles = p->fmt.ntiles; a.NT = p->fmt.NT;
    a.g = plan->g;
    a.g.act = act;
    return launch_conv_mfma(p->dtype, p->fmt.variant, a, plan->grid, plan->lds_bytes, stream);
}

} // namespace npas

using namespace npas;

// ---- stack ---------------------------------------------------------------------
struct npas_stack {
    struct Node {
        npas_layer_desc d;
        int H, W, C;    // input dims
        int Ho, Wo, F;  // output dims (FC / avgpool: Ho = Wo = 1)
        int dtype;
        bool pair_head = false;           // first layer of a fused 1x1 pair (runs the next layer too)
        const void *fused_blob = nullptr; // that pair's weight images on the device (NULL without a GPU)
        int fpp_nt1 = 0;                  // live intermediate tiles of that pair
        uint32_t fpp_use[2] = {0, 0};     // chunk masks of that pair
        bool fused_away = false;          // second layer of a fused pair: runs inside the first
        bool pool_fused = false;          // conv whose max pool (the next layer) is done in the same kernel
        // first layer of a fused 1x1 -> depthwise 3x3 -> 1x1 block (runs the next two layers too): device images and tile
        bool ir_head = false;
        const void *ir_w1 = nullptr, *ir_w3 = nullptr;
        const int *ir_perm = nullptr;
        const uint32_t *ir_wdw = nullptr;
        int ir_nslots = 0, ir_TH = 0, ir_TW = 0, ir_residual = 0;
    };
    std::vector<Node> nodes;
    std::vector<void *> blobs; // device allocations owned by the stack (fused-pair weight images)
    int H = 0, W = 0, C = 0, dtype = 0;
    unsigned flags = 0;
    // per-tensor placement for a given N is computed on the fly (sizes scale with N)
    std::vector<int> last_use; // last layer reading tensor t
    mutable std::mutex place_mu;
    mutable int place_N = -1;
    mutable size_t place_need = 0;
    mutable std::vector<size_t> place_off;
};

namespace npas {

static size_t tensor_elems_per_image(const npas_stack *s, int t)
{
    if (t == 0) return (size_t)s->H * s->W * s->C;
    const npas_stack::Node &n = s->nodes[t - 1];
    return (size_t)n.Ho * n.Wo * n.F;
}

// Layers a launch starting at layer i covers beyond i (fused pair, conv + max pool: 1; fused block: 2).
static int absorbed_after(const npas_stack::Node &n) { return n.ir_head ? 2 : (n.pair_head || n.pool_fused) ? 1 : 0; }

// Greedy first-fit placement of the intermediate tensors (1 .. n-1) into the
// workspace; a tensor's slot is free again after the last launch reading it has run.
// `last_use[t]` is the last layer reading tensor t; a fused launch reads its inputs while it writes the
// output of the last layer it absorbs, which npas_stack_create has recorded by moving last_use of those
// inputs to that layer.  Returns total bytes; offsets[t] for intermediates.
static size_t place_tensors(const npas_stack *s, int N, std::vector<size_t> *offsets)
{
    const int nt = (int)s->nodes.size() + 1;
    std::vector<size_t> off(nt, 0), sz(nt, 0);
    struct Live { size_t off, sz; int until; };
    std::vector<Live> live;
    size_t total = 0;
    const int esz = dtype_size(s->dtype);
    for (int t = 1; t < nt - 1; ++t) { // tensor t is written by layer t-1
        const npas_stack::Node &w = s->nodes[t - 1];
        if (w.pair_head || w.ir_head || w.pool_fused) continue;          // intermediate of a fused pair / block never reaches memory
        if (t >= 2 && s->nodes[t - 2].ir_head) continue;                 // nor does the second one of a fused block
        sz[t] = (tensor_elems_per_image(s, t) * N * esz + 255) / 256 * 256;
        // drop tensors whose last reader ran before layer t-1
        live.erase(std::remove_if(live.begin(), live.end(), [&](const Live &l) { return l.until < t - 1; }),
                   live.end());
        std::sort(live.begin(), live.end(), [](const Live &a, const Live &b) { return a.off < b.off; });
        size_t pos = 0;
        for (const Live &l : live) {
            if (pos + sz[t] <= l.off) break;
            pos = std::max(pos, l.off + l.sz);
        }
        off[t] = pos;
        live.push_back({pos, sz[t], s->last_use[t]});
        total = std::max(total, pos + sz[t]);
    }
    if (offsets) *offsets = off;
    return total;
}

} // namespace npas

namespace npas {

// Dense [F][C] weights (storage bits, zero where pruned) of a packed 1x1 layer.
static std::vector<uint16_t> dense_pointwise(const npas_packed *p)
{
    std::vector<uint16_t> d((size_t)p->F * p->C, 0);
    const uint16_t *wc = reinterpret_cast<const uint16_t *>(p->w_compact.data());
    for (int g = 0; g < p->G; ++g)
        for (int k = p->grp_ptr[g]; k < p->grp_ptr[g + 1]; ++k)
            for (int j = 0; j < p->Bf && g * p->Bf + j < p->F; ++j)
                d[(size_t)(g * p->Bf + j) * p->C + p->k_pos[k]] = wc[(size_t)k * p->Bf + j];
    return d;
}

// Plan and weight images of a fused pointwise pair (layouts: see fused_pointwise_pair_kernel).
struct FppPlan {
    int nt1 = 0;               // live intermediate tiles, rounded up to even
    uint32_t use[2] = {0, 0};  // chunks each layer-2 tile needs
    std::vector<uint16_t> blob;
};

static FppPlan build_fpp(const npas_packed *p1, const npas_packed *p2)
{
    FppPlan plan;
    const int F1 = p1->F, nt2 = (p2->F + 15) / 16;
    // intermediate channels each 16-filter tile of layer 2 keeps (union of its filter groups' lists)
    std::vector<uint8_t> need[2] = {std::vector<uint8_t>(F1, 0), std::vector<uint8_t>(F1, 0)};
    for (int g = 0; g < p2->G; ++g)
        for (int u = 0; u < nt2; ++u) {
            int f_lo = std::max(g * p2->Bf, 16 * u), f_hi = std::min({(g + 1) * p2->Bf, 16 * u + 16, p2->F});
            if (f_lo >= f_hi) continue;
            for (int k = p2->grp_ptr[g]; k < p2->grp_ptr[g + 1]; ++k) need[u][p2->k_pos[k]] = 1;
        }
    // slot order: channels only tile 0 needs, then shared ones, then those only tile 1 needs;
    // dead channels get no slot.  Optionally pad so that tile 1's range starts on a chunk.
    std::vector<int> only0, both, only1;
    for (int c = 0; c < F1; ++c) {
        if (need[0][c] && need[1][c]) both.push_back(c);
        else if (need[0][c]) only0.push_back(c);
        else if (need[1][c]) only1.push_back(c);
    }
    auto cost = [&](int pad, std::vector<int> *perm_out, uint32_t use_out[2]) {
        std::vector<int> perm(only0);
        perm.insert(perm.end(), pad, -1);
        perm.insert(perm.end(), both.begin(), both.end());
        perm.insert(perm.end(), only1.begin(), only1.end());
        int tiles = std::max(2, ((int)perm.size() + 31) / 32 * 2);
        perm.resize((size_t)tiles * 16, -1);
        uint32_t use[2] = {0, 0};
        for (size_t s = 0; s < perm.size(); ++s)
            for (int u = 0; u < nt2; ++u)
                if (perm[s] >= 0 && need[u][perm[s]]) use[u] |= 1u << (s / 32);
        if (perm_out) *perm_out = perm;
        if (use_out) { use_out[0] = use[0]; use_out[1] = use[1]; }
        return tiles + __builtin_popcount(use[0]) + __builtin_popcount(use[1]);
    };
    int pad = (int)((32 - only0.size() % 32) % 32);
    if (only1.empty() || cost(pad, nullptr, nullptr) >= cost(0, nullptr, nullptr)) pad = 0;
    std::vector<int> perm;
    cost(pad, &perm, plan.use);
    plan.nt1 = (int)perm.size() / 16;
    const int nt1 = plan.nt1, nch = nt1 / 2;
    std::vector<uint16_t> d1 = dense_pointwise(p1), d2 = dense_pointwise(p2);
    plan.blob.assign((size_t)(nt1 + nt2 * nch) * 512, 0);
    for (int t = 0; t < nt1; ++t)
        for (int lane = 0; lane < 64; ++lane)
            for (int i = 0; i < 8; ++i) {
                int r = lane & 15, q = lane >> 4, f = perm[16 * t + r], c = 8 * q + i;
                if (f >= 0 && c < p1->C) plan.blob[((size_t)t * 64 + lane) * 8 + i] = d1[(size_t)f * p1->C + c];
            }
    for (int u = 0; u < nt2; ++u)
        for (int j = 0; j < nch; ++j)
            for (int lane = 0; lane < 64; ++lane)
                for (int i = 0; i < 8; ++i) {
                    // rows past the last filter repeat the tile's valid rows in groups of four
                    int r = lane & 15, q = lane >> 4;
                    int nvq = std::min(4, (p2->F - 16 * u) / 4);
                    int f = 16 * u + 4 * ((r >> 2) % nvq) + (r & 3);
                    int c = perm[16 * (2 * j + (i >> 2)) + 4 * q + (i & 3)];
                    if (f < p2->F && c >= 0)
                        plan.blob[((size_t)(nt1 + u * nch + j) * 64 + lane) * 8 + i] = d2[(size_t)f * p2->C + c];
                }
    return plan;
}

// Plan and weight images of a fused inverted-residual block (layouts: see fused_inverted_residual_kernel).
struct IrPlan {
    int nslots = 0;                 // live intermediate channels, padded to a multiple of 32
    std::vector<uint16_t> w1, w3;   // A-operand images
    std::vector<uint32_t> wdw;      // [9][nslots]: the weight's storage bits in the low (even slot) or high (odd slot) half
    std::vector<int> perm;          // [nslots]: intermediate channel of each slot, -1 = padding
};

static IrPlan build_ir(const npas_packed *p1, const npas_packed *pdw, const npas_packed *p3)
{
    IrPlan plan;
    const int mid = p1->F, nt3 = (p3->F + 15) / 16;
    std::vector<uint8_t> live(mid, 0); // intermediate channels some filter of layer 3 keeps
    for (int g = 0; g < p3->G; ++g)
        for (int k = p3->grp_ptr[g]; k < p3->grp_ptr[g + 1]; ++k) live[p3->k_pos[k]] = 1;
    std::vector<int> perm;
    for (int c = 0; c < mid; ++c)
        if (live[c]) perm.push_back(c);
    perm.resize(std::max<size_t>(32, (perm.size() + 31) / 32 * 32), -1);
    plan.nslots = (int)perm.size();
    const int nt1 = plan.nslots / 16, nk = plan.nslots / 32;
    std::vector<uint16_t> d1 = dense_pointwise(p1), d3 = dense_pointwise(p3);
    plan.w1.assign((size_t)nt1 * 512, 0);
    for (int t = 0; t < nt1; ++t)
        for (int lane = 0; lane < 64; ++lane)
            for (int i = 0; i < 8; ++i) {
                const int r = lane & 15, q = lane >> 4, f = perm[16 * t + r], c = 8 * q + i;
                if (f >= 0 && c < p1->C) plan.w1[((size_t)t * 64 + lane) * 8 + i] = d1[(size_t)f * p1->C + c];
            }
    plan.w3.assign((size_t)nt3 * nk * 512, 0);
    for (int u = 0; u < nt3; ++u)
        for (int k = 0; k < nk; ++k)
            for (int lane = 0; lane < 64; ++lane)
                for (int i = 0; i < 8; ++i) {
                    const int r = lane & 15, q = lane >> 4, f = 16 * u + r, c = perm[32 * k + 8 * q + i];
                    if (f < p3->F && c >= 0) plan.w3[((size_t)(u * nk + k) * 64 + lane) * 8 + i] = d3[(size_t)f * p3->C + c];
                }
    plan.wdw.assign((size_t)9 * plan.nslots, 0u);
    const uint16_t *wd = reinterpret_cast<const uint16_t *>(pdw->w_compact.data());
    for (int s = 0; s < plan.nslots; ++s)
        if (perm[s] >= 0)
            for (int t = 0; t < 9; ++t) plan.wdw[(size_t)t * plan.nslots + s] = (uint32_t)wd[(size_t)perm[s] * 9 + t] << (s & 1 ? 16 : 0);
    plan.perm = perm;
    return plan;
}

// Output tile of the fused block for an H x W map: the shape that costs least, counting the
// halo pixels expanded (cheap) and the 16-pixel blocks of depthwise work (about four times dearer),
// among those whose LDS footprint leaves room for several workgroups per CU.
static void plan_ir_tile(int Ho, int Wo, int nslots, int stride, int *TH, int *TW)
{
    double best = 1e300;
    *TH = 1; *TW = 1;
    for (int th = 1; th <= 32; ++th)
        for (int tw = 1; tw <= 64; ++tw) {
            const int ph = (th - 1) * stride + 3, pw = (tw - 1) * stride + 3; // input pixels under the tile, with halo
            if (ph * pw > 256) continue; // four 16-pixel halo blocks per wave at most
            if (fused_ir_lds_bytes(th, tw, nslots, stride) > 64 * 1024) continue;
            const double tiles = (double)((Ho + th - 1) / th) * ((Wo + tw - 1) / tw);
            const double cost = tiles * (1.0 * ((ph * pw + 15) / 16) + 4.0 * ((th * tw + 15) / 16) + 2.0);
            if (cost < best) {
                best = cost;
                *TH = th; *TW = tw;
            }
        }
}

// a 16-bit 1 x 1 layer at stride 1 without padding (the fused block takes a bias, the fused pair does not)
static bool is_pointwise16(const npas_layer_desc &d)
{
    return d.kind == NPAS_LAYER_CONV && d.packed && d.packed->KH == 1 && d.packed->KW == 1 && d.stride == 1 &&
           d.pad == 0 && d.packed->dtype != NPAS_F32;
}
static bool is_plain_pointwise(const npas_layer_desc &d) { return is_pointwise16(d) && !d.bias_dev; }

} // namespace npas

extern "C" {

int npas_conv2d_sparse(const npas_packed *p, const void *x_dev, void *y_dev, int N, int H, int W, int stride,
                       int pad, const void *bias_dev, const void *residual_dev, npas_act act, void *hip_stream)
{
    int rc = check_run(p, x_dev, y_dev, N, H, W, stride, pad);
    if (rc) return rc;
    return run_conv(p, nullptr, x_dev, y_dev, N, H, W, stride, pad, bias_dev, residual_dev, act, hip_stream);
}

const char *npas_conv2d_kernel_name(const npas_packed *p, int N, int H, int W, int stride, int pad)
{
    if (!p || N <= 0 || H <= 0 || W <= 0 || stride <= 0 || pad < 0) return nullptr;
    return route_name(p, N, H, W, stride, pad);
}

int npas_fc_sparse(const npas_packed *p, const void *x_dev, void *y_dev, int B, const void *bias_dev, npas_act act,
                   void *hip_stream)
{
    if (p && (p->KH != 1 || p->KW != 1)) {
        set_error("npas_fc_sparse needs a layer packed as FC or 1x1 (got %dx%d)", p->KH, p->KW);
        return NPAS_E_SHAPE;
    }
    int rc = check_run(p, x_dev, y_dev, B, 1, 1, 1, 0);
    if (rc) return rc;
    return run_conv(p, nullptr, x_dev, y_dev, B, 1, 1, 1, 0, bias_dev, nullptr, act, hip_stream);
}

static int run_depthwise(const npas_packed *p, const void *x, void *y, int N, int H, int W, int stride, const void *bias,
                         const void *residual, int act, void *stream)
{
    if (!p || !x || !y) {
        set_error("NULL argument (handle=%p x_dev=%p y_dev=%p)", (const void *)p, x, y);
        return NPAS_E_NULL;
    }
    if (p->scheme != NPAS_SCHEME_DEPTHWISE) {
        set_error("npas_depthwise3x3 needs a handle from npas_pack_depthwise3x3 (scheme %d)", p->scheme);
        return NPAS_E_SHAPE;
    }
    if (N <= 0 || H <= 0 || W <= 0 || stride <= 0 || (double)N * H * W * p->C > 2147483647.0) {
        set_error("bad geometry N=%d H=%d W=%d stride=%d", N, H, W, stride);
        return NPAS_E_SHAPE;
    }
    if (!valid_act(act)) {
        set_error("unknown activation %d", act);
        return NPAS_E_SHAPE;
    }
    if (p->dev.device < 0) {
        set_error("packed layer has no device copy (packed on a machine without a GPU)");
        return NPAS_E_HIP;
    }
    const void *w = p->dtype == NPAS_F32 ? (const void *)p->dev.vw : p->dev.wfrag;
    return launch_depthwise3x3(p->dtype, x, y, w, (const float *)bias, residual, N, H, W, p->C, stride, act, stream);
}

int npas_depthwise3x3(const npas_packed *p, const void *x_dev, void *y_dev, int N, int H, int W, int stride,
                      const void *bias_dev, const void *residual_dev, npas_act act, void *hip_stream)
{
    return run_depthwise(p, x_dev, y_dev, N, H, W, stride, bias_dev, residual_dev, act, hip_stream);
}

static int check_pool(const void *x, void *y, int N, int H, int W, int C, int dt)
{
    if (!x || !y) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (double)N * H * W * C > 2147483647.0) {
        set_error("bad shape N=%d H=%d W=%d C=%d", N, H, W, C);
        return NPAS_E_SHAPE;
    }
    if (dt != NPAS_F32 && dt != NPAS_BF16 && dt != NPAS_F16) {
        set_error("unknown storage type %d", dt);
        return NPAS_E_DTYPE;
    }
    return NPAS_OK;
}

int npas_debug_launch_empty(int count, void *hip_stream)
{
    if (count < 0 || count > 100000) {
        set_error("bad launch count %d", count);
        return NPAS_E_SHAPE;
    }
    return launch_empty(count, hip_stream);
}

int npas_maxpool3x3s2(const void *x_dev, void *y_dev, int N, int H, int W, int C, npas_dtype dt, void *hip_stream)
{
    int rc = check_pool(x_dev, y_dev, N, H, W, C, dt);
    return rc ? rc : launch_maxpool(x_dev, y_dev, N, H, W, C, dt, hip_stream);
}

int npas_global_avgpool(const void *x_dev, void *y_dev, int N, int H, int W, int C, npas_dtype dt, void *hip_stream)
{
    int rc = check_pool(x_dev, y_dev, N, H, W, C, dt);
    return rc ? rc : launch_avgpool(x_dev, y_dev, N, H, W, C, dt, hip_stream);
}

int npas_stack_create(const npas_layer_desc *layers, int n_layers, int H, int W, unsigned flags, npas_stack **out)
{
    if (!layers || !out) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    *out = nullptr;
    if (n_layers <= 0 || H <= 0 || W <= 0) {
        set_error("bad stack geometry n_layers=%d H=%d W=%d", n_layers, H, W);
        return NPAS_E_SHAPE;
    }
    std::unique_ptr<npas_stack> s(new npas_stack);
    s->flags = flags;
    s->H = H; s->W = W;
    s->last_use.assign(n_layers + 1, -1);
    struct Dim { int H, W, C; };
    std::vector<Dim> dims(n_layers + 1);
    bool have_in = false;
    for (int i = 0; i < n_layers; ++i) {
        const npas_layer_desc &d = layers[i];
        if (d.src < 0 || d.src > i || d.res > i || d.res < -1) {
            set_error("layer %d reads tensor src=%d res=%d that is not produced yet", i, d.src, d.res);
            return NPAS_E_SHAPE;
        }
        const bool pruned = d.kind == NPAS_LAYER_CONV || d.kind == NPAS_LAYER_FC;
        const bool weighted = pruned || d.kind == NPAS_LAYER_DEPTHWISE3X3;
        if (weighted && !d.packed) {
            set_error("layer %d has no packed handle", i);
            return NPAS_E_NULL;
        }
        if (!have_in) { // the stack input's channel count and type come from the first pruned layer reading it
            if (!(pruned && d.src == 0)) {
                if (i == 0) {
                    set_error("layer 0 must be a CONV or FC layer reading the stack input");
                    return NPAS_E_SHAPE;
                }
            } else {
                s->C = d.packed->C; s->dtype = d.packed->dtype;
                dims[0] = {H, W, s->C};
                have_in = true;
            }
        }
        if (!have_in) {
            set_error("layer 0 must be a CONV or FC layer reading the stack input");
            return NPAS_E_SHAPE;
        }
        npas_stack::Node nd;
        nd.d = d;
        nd.dtype = s->dtype;
        const Dim in = dims[d.src];
        nd.H = in.H; nd.W = in.W; nd.C = in.C;
        switch (d.kind) {
        case NPAS_LAYER_CONV:
            if (d.packed->C != in.C || d.stride <= 0 || d.pad < 0 || in.H + 2 * d.pad < d.packed->KH ||
                in.W + 2 * d.pad < d.packed->KW) {
                set_error("layer %d: conv geometry does not fit its input (%dx%dx%d)", i, in.H, in.W, in.C);
                return NPAS_E_SHAPE;
            }
            nd.Ho = (in.H + 2 * d.pad - d.packed->KH) / d.stride + 1;
            nd.Wo = (in.W + 2 * d.pad - d.packed->KW) / d.stride + 1;
            nd.F = d.packed->F;
            break;
        case NPAS_LAYER_FC:
            if (d.packed->KH != 1 || d.packed->KW != 1 || d.packed->C != in.H * in.W * in.C) {
                set_error("layer %d: FC input size %d does not match %dx%dx%d", i, d.packed->C, in.H, in.W, in.C);
                return NPAS_E_SHAPE;
            }
            nd.H = nd.W = 1; nd.C = d.packed->C;
            nd.Ho = nd.Wo = 1; nd.F = d.packed->F;
            break;
        case NPAS_LAYER_DEPTHWISE3X3:
            if (d.packed->scheme != NPAS_SCHEME_DEPTHWISE || d.packed->C != in.C || d.stride <= 0) {
                set_error("layer %d: depthwise layer does not fit its input (%dx%dx%d)", i, in.H, in.W, in.C);
                return NPAS_E_SHAPE;
            }
            nd.Ho = (in.H - 1) / d.stride + 1; nd.Wo = (in.W - 1) / d.stride + 1; nd.F = in.C;
            break;
        case NPAS_LAYER_MAXPOOL3X3S2:
            nd.Ho = (in.H - 1) / 2 + 1; nd.Wo = (in.W - 1) / 2 + 1; nd.F = in.C;
            break;
        case NPAS_LAYER_GLOBAL_AVGPOOL:
            nd.Ho = nd.Wo = 1; nd.F = in.C;
            break;
        default:
            set_error("layer %d: unknown kind %d", i, d.kind);
            return NPAS_E_SHAPE;
        }
        if (d.kind == NPAS_LAYER_CONV && d.packed->scheme == NPAS_SCHEME_DEPTHWISE) {
            set_error("layer %d: a depthwise handle needs a DEPTHWISE3X3 layer", i);
            return NPAS_E_SHAPE;
        }
        if (weighted && !valid_act(d.act)) {
            set_error("layer %d: unknown activation %d", i, d.act);
            return NPAS_E_SHAPE;
        }
        if (weighted && d.packed->dtype != s->dtype) {
            set_error("layer %d: storage type %d differs from the stack's %d", i, d.packed->dtype, s->dtype);
            return NPAS_E_DTYPE;
        }
        if (d.res >= 0) {
            const Dim r = dims[d.res];
            if ((d.kind != NPAS_LAYER_CONV && d.kind != NPAS_LAYER_DEPTHWISE3X3) || r.H != nd.Ho || r.W != nd.Wo || r.C != nd.F) {
                set_error("layer %d: residual tensor %d has the wrong shape", i, d.res);
                return NPAS_E_SHAPE;
            }
            s->last_use[d.res] = i;
        }
        s->last_use[d.src] = i;
        dims[i + 1] = {nd.Ho, nd.Wo, nd.F};
        s->nodes.push_back(nd);
    }
    // Uploads a fused launch's weight images; without a GPU the plan is kept (placement and launch count are the
    // same) and the run call fails like any other on such a machine.
    int ndev = 0;
    const bool have_dev = hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0;
    if (!have_dev) (void)hipGetLastError();
    auto upload_blob = [&](const void *data, size_t bytes, void **dptr) -> int {
        *dptr = nullptr;
        if (!have_dev) return NPAS_OK;
        if (hipMalloc(dptr, bytes) != hipSuccess || hipMemcpy(*dptr, data, bytes, hipMemcpyHostToDevice) != hipSuccess) {
            if (*dptr) (void)hipFree(*dptr);
            set_error("could not upload the weight images of a fused launch (%zu bytes)", bytes);
            for (void *q : s->blobs) (void)hipFree(q);
            s->blobs.clear();
            return NPAS_E_HIP;
        }
        s->blobs.push_back(*dptr);
        return NPAS_OK;
    };
    auto busy = [](const npas_stack::Node &n) { return n.fused_away || n.pair_head || n.ir_head || n.pool_fused; };
    if (flags & NPAS_STACK_FUSE_INVERTED_RESIDUAL) {
        for (int i = 0; i + 2 < n_layers; ++i) {
            npas_stack::Node &a = s->nodes[i], &b = s->nodes[i + 1], &c = s->nodes[i + 2];
            if (busy(a) || busy(b) || busy(c) || !is_pointwise16(a.d) || !is_pointwise16(c.d) || a.d.res >= 0) continue;
            if (b.d.kind != NPAS_LAYER_DEPTHWISE3X3 || (b.d.stride != 1 && b.d.stride != 2) || b.d.res >= 0) continue;
            if (b.d.stride == 2 && c.d.res >= 0) continue; // the block input has another shape than its output
            if (b.d.src != i + 1 || c.d.src != i + 2 || (c.d.res >= 0 && c.d.res != a.d.src)) continue;
            bool other_reader = false; // the two tensors inside the block must have no reader outside it
            for (int j = i + 1; j < n_layers; ++j) {
                const npas_layer_desc &dj = s->nodes[j].d;
                if ((j != i + 1 && dj.src == i + 1) || dj.res == i + 1) other_reader = true;
                if ((j != i + 2 && dj.src == i + 2) || dj.res == i + 2) other_reader = true;
            }
            if (other_reader) continue;
            const npas_packed *p1 = a.d.packed, *p3 = c.d.packed;
            if (p1->C > 32 || p1->C % 8 || p3->F % 4 || p3->F > 32 || (c.d.res >= 0 && p3->F != p1->C)) continue;
            IrPlan ip = build_ir(p1, b.d.packed, p3);
            if (ip.nslots > 192) continue;
            int th, tw;
            const int st2 = b.d.stride;
            plan_ir_tile((a.H - 1) / st2 + 1, (a.W - 1) / st2 + 1, ip.nslots, st2, &th, &tw);
            if (fused_ir_lds_bytes(th, tw, ip.nslots, st2) > 64 * 1024) continue;
            const size_t b1 = ip.w1.size() * 2, b3 = ip.w3.size() * 2, bd = ip.wdw.size() * 4, bp = ip.perm.size() * 4;
            const size_t o3 = (b1 + 255) / 256 * 256, od = o3 + (b3 + 255) / 256 * 256, op = od + (bd + 255) / 256 * 256;
            std::vector<uint8_t> blob(op + bp);
            std::memcpy(blob.data(), ip.w1.data(), b1);
            std::memcpy(blob.data() + o3, ip.w3.data(), b3);
            std::memcpy(blob.data() + od, ip.wdw.data(), bd);
            std::memcpy(blob.data() + op, ip.perm.data(), bp);
            void *dptr = nullptr;
            if (int rc = upload_blob(blob.data(), blob.size(), &dptr)) return rc;
            a.ir_head = true;
            if (dptr) {
                a.ir_w1 = dptr;
                a.ir_w3 = (const uint8_t *)dptr + o3;
                a.ir_wdw = (const uint32_t *)((const uint8_t *)dptr + od);
                a.ir_perm = (const int *)((const uint8_t *)dptr + op);
            }
            a.ir_nslots = ip.nslots; a.ir_TH = th; a.ir_TW = tw; a.ir_residual = c.d.res >= 0;
            b.fused_away = true;
            c.fused_away = true;
        }
    }
    if (flags & NPAS_STACK_FUSE_CONV_MAXPOOL) {
        for (int i = 0; i + 1 < n_layers; ++i) {
            npas_stack::Node &a = s->nodes[i], &b = s->nodes[i + 1];
            if (busy(a) || busy(b) || a.d.kind != NPAS_LAYER_CONV || b.d.kind != NPAS_LAYER_MAXPOOL3X3S2 || b.d.src != i + 1 || a.d.res >= 0) continue;
            bool other_reader = false;
            for (int j = i + 1; j < n_layers; ++j)
                if ((j != i + 1 && s->nodes[j].d.src == i + 1) || s->nodes[j].d.res == i + 1) other_reader = true;
            SmallCArgs sc;
            if (other_reader || !plan_smallc_pool(a.d.packed, 1, a.H, a.W, a.d.stride, a.d.pad, &sc)) continue;
            a.pool_fused = true;
            b.fused_away = true;
        }
    }
    if (flags & NPAS_STACK_FUSE_POINTWISE) {
        for (int i = 0; i + 1 < n_layers; ++i) {
            npas_stack::Node &a = s->nodes[i], &b = s->nodes[i + 1];
            // neither layer may already belong to (or head) another fused launch
            if (busy(a) || busy(b) || !is_plain_pointwise(a.d) || !is_plain_pointwise(b.d)) continue;
            // the intermediate (tensor i+1) must feed layer i+1 only, and neither layer adds a residual
            if (b.d.src != i + 1 || a.d.res >= 0 || b.d.res >= 0) continue;
            bool other_reader = false;
            for (int j = i + 1; j < n_layers; ++j)
                if ((j != i + 1 && s->nodes[j].d.src == i + 1) || s->nodes[j].d.res == i + 1) other_reader = true;
            if (other_reader) continue;
            const npas_packed *p1 = a.d.packed, *p2 = b.d.packed;
            if (p1->C > 32 || p1->C % 8 || p2->F % 4 || p2->F > 32) continue;
            FppPlan fp = build_fpp(p1, p2);
            if (!fpp_supported(fp.nt1, (p2->F + 15) / 16)) continue;
            void *dptr = nullptr;
            if (int rc = upload_blob(fp.blob.data(), fp.blob.size() * 2, &dptr)) return rc;
            a.pair_head = true;
            a.fused_blob = dptr;
            a.fpp_nt1 = fp.nt1;
            a.fpp_use[0] = fp.use[0];
            a.fpp_use[1] = fp.use[1];
            b.fused_away = true;
        }
    }
    // A fused launch reads its inputs while it writes the output of the last layer it absorbs: keep them
    // allocated until then (the workspace placement frees a tensor after the layer recorded here).
    for (int i = 0; i < n_layers; ++i) {
        const npas_stack::Node &h = s->nodes[i];
        const int last = i + absorbed_after(h);
        if (last == i) continue;
        for (int j = i; j <= last; ++j) {
            const npas_layer_desc &d = s->nodes[j].d;
            if (d.src <= i) s->last_use[d.src] = std::max(s->last_use[d.src], last);
            if (d.res >= 0 && d.res <= i) s->last_use[d.res] = std::max(s->last_use[d.res], last);
        }
    }
    *out = s.release();
    return NPAS_OK;
}

size_t npas_stack_workspace_bytes(const npas_stack *s, int N)
{
    if (!s || N <= 0) return 0;
    return place_tensors(s, N, nullptr);
}

int npas_stack_num_launches(const npas_stack *s)
{
    if (!s) return 0;
    int n = 0;
    for (const npas_stack::Node &nd : s->nodes) n += nd.fused_away ? 0 : 1;
    return n;
}

int npas_stack_describe(const npas_stack *s, int N, int64_t *rows_host, int max_rows)
{
    if (!s || (!rows_host && max_rows > 0)) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    if (N <= 0 || max_rows < 0) {
        set_error("bad batch %d or row count %d", N, max_rows);
        return NPAS_E_SHAPE;
    }
    std::vector<size_t> off;
    (void)place_tensors(s, N, &off);
    const int nl = (int)s->nodes.size();
    const int64_t esz = dtype_size(s->dtype);
    auto where = [&](int t) -> int64_t { return t < 0 ? -3 : t == 0 ? -1 : t == nl ? -2 : (int64_t)off[t]; };
    auto bytes = [&](int t) -> int64_t { return t < 0 ? 0 : (int64_t)tensor_elems_per_image(s, t) * N * esz; };
    int r = 0;
    for (int i = 0; i < nl; ++i) {
        const npas_stack::Node &n = s->nodes[i];
        if (n.fused_away) continue;
        const int last = i + absorbed_after(n);
        const int res = n.ir_head ? s->nodes[last].d.res : n.d.res; // a fused block adds its input at its last layer
        if (r < max_rows) {
            const int64_t row[NPAS_DESCRIBE_COLS] = {i, last, n.d.src, res, last + 1, where(n.d.src), where(res), where(last + 1),
                                                     bytes(n.d.src), bytes(res), bytes(last + 1)};
            std::memcpy(rows_host + (size_t)r * NPAS_DESCRIBE_COLS, row, sizeof row);
        }
        ++r;
    }
    return r;
}

} // extern "C"

namespace npas {

// The body of npas_run_stack; also behind the allocation-free entry point.
int run_stack_impl(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *workspace_dev, size_t workspace_bytes,
                   void *hip_stream)
{
    if (!s || !x_dev || !y_dev) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    if (N <= 0) {
        set_error("bad batch %d", N);
        return NPAS_E_SHAPE;
    }
    // placement depends on N only; the last one is kept (and read under the lock: no copy, no allocation per call)
    std::lock_guard<std::mutex> lock(s->place_mu);
    if (s->place_N != N) {
        s->place_need = place_tensors(s, N, &s->place_off);
        s->place_N = N;
    }
    const std::vector<size_t> &off = s->place_off;
    const size_t need = s->place_need;
    if (need > 0 && (!workspace_dev || workspace_bytes < need || ((uintptr_t)workspace_dev & 255))) {
        set_error("workspace: need %zu bytes, 256-byte aligned; got %zu at %p", need, workspace_bytes, workspace_dev);
        return NPAS_E_WORKSPACE;
    }
    const int nl = (int)s->nodes.size();
    auto tensor = [&](int t) -> void * {
        if (t == 0) return const_cast<void *>(x_dev);
        if (t == nl) return y_dev;
        return (uint8_t *)workspace_dev + off[t];
    };
    for (int i = 0; i < nl; ++i) {
        const npas_stack::Node &n = s->nodes[i];
        if (n.fused_away) continue;
        const void *x = tensor(n.d.src);
        void *y = tensor(i + 1);
        int rc = NPAS_OK;
        if (n.ir_head) { // this layer and the next two as one kernel; the tensors between them are never stored
            const npas_packed *p1 = n.d.packed, *p3 = s->nodes[i + 2].d.packed;
            rc = check_run(p1, x, tensor(i + 3), N, n.H, n.W, 1, 0);
            if (!rc && !n.ir_w1) {
                set_error("fused block has no device copy (stack created on a machine without a GPU)");
                rc = NPAS_E_HIP;
            }
            if (!rc) {
                const npas_layer_desc &d2 = s->nodes[i + 1].d, &d3 = s->nodes[i + 2].d;
                IrLaunch l;
                l.x = x; l.y = tensor(i + 3); l.w1 = n.ir_w1; l.w3 = n.ir_w3; l.wdw = n.ir_wdw; l.perm = n.ir_perm;
                l.b1 = (const float *)n.d.bias_dev; l.b2 = (const float *)d2.bias_dev; l.b3 = (const float *)d3.bias_dev;
                l.N = N; l.H = n.H; l.W = n.W; l.C1 = p1->C; l.F3 = p3->F; l.nslots = n.ir_nslots; l.TH = n.ir_TH; l.TW = n.ir_TW;
                l.stride = d2.stride; l.act1 = n.d.act; l.act2 = d2.act; l.act3 = d3.act; l.residual = n.ir_residual;
                rc = launch_fused_inverted_residual(p1->dtype, l, hip_stream);
            }
            if (rc) return rc;
            continue;
        }
        if (n.pool_fused) { // this layer and the max pool after it as one kernel; the conv output is never stored
            rc = check_run(n.d.packed, x, tensor(i + 2), N, n.H, n.W, n.d.stride, n.d.pad);
            if (!rc) rc = run_conv_maxpool(n.d.packed, x, tensor(i + 2), N, n.H, n.W, n.d.stride, n.d.pad, n.d.bias_dev, n.d.act, hip_stream);
            if (rc) return rc;
            continue;
        }
        if (n.pair_head) { // this layer and the next as one kernel; the tensor between them is never stored
            const npas_packed *p1 = n.d.packed, *p2 = s->nodes[i + 1].d.packed;
            rc = check_run(p1, x, tensor(i + 2), N, n.H, n.W, 1, 0);
            if (!rc && !n.fused_blob) {
                set_error("fused pair has no device copy (stack created on a machine without a GPU)");
                rc = NPAS_E_HIP;
            }
            if (!rc)
                rc = launch_fused_pointwise_pair(p1->dtype, x, tensor(i + 2), n.fused_blob, N * n.H * n.W, p1->C,
                                                 n.fpp_nt1, p2->F, n.d.act, s->nodes[i + 1].d.act, n.fpp_use[0],
                                                 n.fpp_use[1], hip_stream);
            if (rc) return rc;
            continue;
        }
        switch (n.d.kind) {
        case NPAS_LAYER_CONV:
            rc = check_run(n.d.packed, x, y, N, n.H, n.W, n.d.stride, n.d.pad);
            if (!rc)
                rc = run_conv(n.d.packed, nullptr, x, y, N, n.H, n.W, n.d.stride, n.d.pad, n.d.bias_dev,
                              n.d.res >= 0 ? tensor(n.d.res) : nullptr, n.d.act, hip_stream);
            break;
        case NPAS_LAYER_FC:
            rc = check_run(n.d.packed, x, y, N, 1, 1, 1, 0);
            if (!rc) rc = run_conv(n.d.packed, nullptr, x, y, N, 1, 1, 1, 0, n.d.bias_dev, nullptr, n.d.act, hip_stream);
            break;
        case NPAS_LAYER_DEPTHWISE3X3:
            rc = run_depthwise(n.d.packed, x, y, N, n.H, n.W, n.d.stride, n.d.bias_dev, n.d.res >= 0 ? tensor(n.d.res) : nullptr,
                               n.d.act, hip_stream);
            break;
        case NPAS_LAYER_MAXPOOL3X3S2:
            rc = launch_maxpool(x, y, N, n.H, n.W, n.C, n.dtype, hip_stream);
            break;
        case NPAS_LAYER_GLOBAL_AVGPOOL:
            rc = launch_avgpool(x, y, N, n.H, n.W, n.C, n.dtype, hip_stream);
            break;
        }
        if (rc) return rc;
    }
    return NPAS_OK;
}

} // namespace npas

extern "C" {

int npas_run_stack(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *workspace_dev,
                   size_t workspace_bytes, void *hip_stream)
{
    return npas::run_stack_impl(s, x_dev, y_dev, N, workspace_dev, workspace_bytes, hip_stream);
}

void npas_stack_free(npas_stack *s)
{
    if (!s) return;
    for (void *q : s->blobs) (void)hipFree(q);
    delete s;
}

} // extern "C"
