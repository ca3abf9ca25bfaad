// Host side of libnpas: scheme validation, the canonical compact form, the
// device execution formats, and their upload.
//
// Scheme definitions follow the paper: block-punched and block-based pruning in
// section 3 (Fig. 1 (f), (g)), pattern-based pruning with kernel removal in
// section 2.1 (Fig. 1 (e)).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "npas_internal.h"

namespace npas {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

const char *last_error() { return g_err; }

static int parse_force(const char *v)
{
    static const char *names[] = {"", "gather", "slab", "noring", "nosmallc", "spatial", "nospatial2", "smallm",
                                  "resident", "noresident", "nofcgather", "valu"};
    if (!v) return FV_NONE;
    for (int i = 1; i < (int)(sizeof(names) / sizeof(names[0])); ++i)
        if (strcmp(v, names[i]) == 0) return i;
    return FV_NONE;
}

static Switches &switches_rw()
{
    static Switches sw = [] {
        Switches s;
        s.force = parse_force(getenv("NPAS_FORCE_VARIANT"));
        s.no_balance = getenv("NPAS_NO_BALANCE") != nullptr;
        return s;
    }();
    return sw;
}

const Switches &switches() { return switches_rw(); }

static inline size_t widx(int f, int c, int kh, int kw, int C, int KH, int KW)
{
    return (((size_t)f * C + c) * KH + kh) * KW + kw;
}

// Copies one weight (storage type) or writes +0.
static inline void put_weight(uint8_t *dst, const uint8_t *src, int esz, bool keep)
{
    if (keep) memcpy(dst, src, esz);
    else memset(dst, 0, esz);
}

static int check_mask_values(const uint8_t *m, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (m[i] > 1) {
            set_error("mask[%zu] = %d is neither 0 nor 1", i, (int)m[i]);
            return NPAS_E_MASK_VALUE;
        }
    return NPAS_OK;
}

// Block-punched rule: inside a group of Bf filters the mask does not depend on
// the filter (channel blocks need no check of their own: the rule constrains
// the filter axis only; Bc is recorded as the scheme parameter).
static int validate_block_punched(const uint8_t *m, int F, int C, int KH, int KW, int Bf)
{
    size_t per = (size_t)C * KH * KW;
    for (int f = 0; f < F; ++f) {
        int lead = f - f % Bf;
        if (f == lead) continue;
        if (memcmp(m + (size_t)f * per, m + (size_t)lead * per, per) != 0) {
            size_t p = 0;
            while (m[(size_t)f * per + p] == m[(size_t)lead * per + p]) ++p;
            set_error("mask is not block-punched: filter %d differs from filter %d of its block at "
                      "position (c=%zu, kh=%zu, kw=%zu)", f, lead, p / (KH * KW), (p / KW) % KH, p % KW);
            return NPAS_E_MASK_NOT_BLOCK_UNIFORM;
        }
    }
    return NPAS_OK;
}

// Block-based rule: inside every Br x Bcol block mask = rowkeep AND colkeep.
static int validate_fc_block(const uint8_t *m, int OUT, int IN, int Br, int Bcol)
{
    std::vector<uint8_t> rowkeep(Br), colkeep(Bcol);
    for (int r0 = 0; r0 < OUT; r0 += Br)
        for (int c0 = 0; c0 < IN; c0 += Bcol) {
            int nr = std::min(Br, OUT - r0), nc = std::min(Bcol, IN - c0);
            std::fill(rowkeep.begin(), rowkeep.end(), 0);
            std::fill(colkeep.begin(), colkeep.end(), 0);
            for (int r = 0; r < nr; ++r)
                for (int c = 0; c < nc; ++c)
                    if (m[(size_t)(r0 + r) * IN + c0 + c]) rowkeep[r] = colkeep[c] = 1;
            for (int r = 0; r < nr; ++r)
                for (int c = 0; c < nc; ++c)
                    if (m[(size_t)(r0 + r) * IN + c0 + c] != (rowkeep[r] & colkeep[c])) {
                        set_error("mask is not block-based: block at (row %d, col %d) is not whole "
                                  "rows/columns (entry %d,%d)", r0, c0, r0 + r, c0 + c);
                        return NPAS_E_MASK_NOT_BLOCK_UNIFORM;
                    }
        }
    return NPAS_OK;
}

// Canonical compact form shared by all schemes: per group of Bf filters, the
// ascending list of positions (kh*KW+kw)*C + c kept by any filter of the group,
// and the group's weights at those positions.
static void pack_canonical(npas_packed *p, const uint8_t *w, const uint8_t *m)
{
    const int F = p->F, C = p->C, KH = p->KH, KW = p->KW, Bf = p->Bf, esz = dtype_size(p->dtype);
    p->G = (F + Bf - 1) / Bf;
    p->grp_ptr.assign(p->G + 1, 0);
    p->k_pos.clear();
    p->w_compact.clear();
    std::vector<uint8_t> row((size_t)Bf * esz);
    for (int g = 0; g < p->G; ++g) {
        p->grp_ptr[g] = (int32_t)p->k_pos.size();
        int f0 = g * Bf, nf = std::min(Bf, F - f0);
        for (int kh = 0; kh < KH; ++kh)
            for (int kw = 0; kw < KW; ++kw)
                for (int c = 0; c < C; ++c) {
                    bool any = false;
                    for (int j = 0; j < nf && !any; ++j) any = m[widx(f0 + j, c, kh, kw, C, KH, KW)] != 0;
                    if (!any) continue;
                    p->k_pos.push_back((kh * KW + kw) * C + c);
                    for (int j = 0; j < Bf; ++j) {
                        bool keep = j < nf && m[widx(f0 + j, c, kh, kw, C, KH, KW)];
                        put_weight(&row[(size_t)j * esz], keep ? w + widx(f0 + j, c, kh, kw, C, KH, KW) * esz : nullptr,
                                   esz, keep);
                    }
                    p->w_compact.insert(p->w_compact.end(), row.begin(), row.end());
                }
    }
    p->grp_ptr[p->G] = (int32_t)p->k_pos.size();
}

// ---- device execution formats ------------------------------------------------

static void build_mfma_gather(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    DeviceFormat &d = p->fmt;
    const int F = p->F, C = p->C, KH = p->KH, KW = p->KW;
    d.variant = V_MFMA_GATHER;
    int cc = (KH == 1 && KW == 1) ? 256 : 64;
    d.CC = std::min(C, cc);
    d.nchunks = (C + d.CC - 1) / d.CC;
    d.ntiles = (F + 15) / 16;
    d.tc_ptr.assign((size_t)d.ntiles * d.nchunks + 1, 0);
    d.kent.clear();
    d.wfrag.clear();
    d.max_list = 0;
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(w);
    std::vector<uint32_t> ent;
    std::vector<size_t> base; // weight index of filter 16t at each entry
    for (int t = 0; t < d.ntiles; ++t) {
        int f0 = 16 * t, nf = std::min(16, F - f0);
        for (int ch = 0; ch < d.nchunks; ++ch) {
            int c0 = ch * d.CC, c1 = std::min(C, c0 + d.CC);
            ent.clear();
            base.clear();
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw)
                    for (int c = c0; c < c1; ++c) {
                        bool any = false;
                        for (int j = 0; j < nf && !any; ++j) any = m[widx(f0 + j, c, kh, kw, C, KH, KW)] != 0;
                        if (!any) continue;
                        ent.push_back((uint32_t)kh << 24 | (uint32_t)kw << 16 | (uint32_t)(c - c0));
                        base.push_back(widx(f0, c, kh, kw, C, KH, KW));
                    }
            size_t n = ent.size(), npad = (n + 31) / 32 * 32;
            d.tc_ptr[(size_t)t * d.nchunks + ch] = (int32_t)d.kent.size();
            d.max_list = std::max(d.max_list, (int)npad);
            size_t e0 = d.kent.size();
            d.kent.resize(e0 + npad, n ? ent[0] : 0u);
            std::copy(ent.begin(), ent.end(), d.kent.begin() + e0);
            size_t w0 = d.wfrag.size();
            d.wfrag.resize(w0 + npad * 16, 0);
            const size_t fstride = (size_t)C * KH * KW;
            for (size_t e = 0; e < n; ++e) {
                size_t blk = e / 32, k = e % 32, q = k / 8, i = k % 8;
                for (int r = 0; r < nf; ++r) {
                    size_t wi = base[e] + (size_t)r * fstride;
                    if (m[wi]) d.wfrag[w0 + blk * 512 + (q * 16 + r) * 8 + i] = w16[wi];
                }
            }
        }
    }
    d.tc_ptr.back() = (int32_t)d.kent.size();
}


// Slab format (see npas_internal.h).  NT = row tiles per wave: a wave reuses each
// gathered activation fragment NT times.
static void build_mfma_slab(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    DeviceFormat &d = p->fmt;
    const int F = p->F, C = p->C, KH = p->KH, KW = p->KW;
    d.variant = V_MFMA_SLAB;
    d.NT = F > 32 ? 4 : 2;
    d.CC = std::min(C, 64);
    d.nchunks = (C + d.CC - 1) / d.CC;
    const int SF = 16 * d.NT;
    d.ntiles = (F + SF - 1) / SF;
    d.tc_ptr.assign((size_t)d.ntiles * d.nchunks + 1, 0);
    d.kent.clear();
    d.wfrag.clear();
    d.max_list = 0;
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(w);
    const size_t fstride = (size_t)C * KH * KW;
    std::vector<uint32_t> ent;
    std::vector<size_t> base;
    for (int st = 0; st < d.ntiles; ++st) {
        int f0 = SF * st, nf = std::min(SF, F - f0);
        for (int ch = 0; ch < d.nchunks; ++ch) {
            int c0 = ch * d.CC, c1 = std::min(C, c0 + d.CC);
            ent.clear();
            base.clear();
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw)
                    for (int c = c0; c < c1; c += 8) {
                        bool any = false;
                        for (int j = 0; j < nf && !any; ++j)
                            for (int i = 0; i < 8 && !any; ++i) any = m[widx(f0 + j, c + i, kh, kw, C, KH, KW)] != 0;
                        if (!any) continue;
                        ent.push_back((uint32_t)kh << 24 | (uint32_t)kw << 16 | (uint32_t)(c - c0));
                        base.push_back(widx(f0, c, kh, kw, C, KH, KW));
                    }
            size_t n = ent.size(), npad = (n + 3) / 4 * 4;
            d.tc_ptr[(size_t)st * d.nchunks + ch] = (int32_t)d.kent.size();
            d.max_list = std::max(d.max_list, (int)npad);
            size_t e0 = d.kent.size();
            d.kent.resize(e0 + npad, n ? ent[0] : 0u);
            std::copy(ent.begin(), ent.end(), d.kent.begin() + e0);
            size_t w0 = d.wfrag.size();
            d.wfrag.resize(w0 + npad / 4 * d.NT * 512, 0);
            const size_t cstride = (size_t)KH * KW; // channel stride in W[F][C][KH][KW]
            for (size_t e = 0; e < n; ++e) {
                size_t step = e / 4, q = e % 4;
                for (int j = 0; j < d.NT; ++j)
                    for (int r = 0; r < 16; ++r) {
                        int f = f0 + 16 * j + r;
                        if (f >= F) continue;
                        for (int i = 0; i < 8; ++i) {
                            size_t wi = base[e] + (size_t)(16 * j + r) * fstride + (size_t)i * cstride;
                            if (m[wi]) d.wfrag[w0 + (step * d.NT + j) * 512 + (q * 16 + r) * 8 + i] = w16[wi];
                        }
                    }
            }
        }
    }
    d.tc_ptr.back() = (int32_t)d.kent.size();
}

// Mean fraction of a 16-filter tile's positions that survive in the union of its groups.
static double union_density(const npas_packed *p, const uint8_t *m)
{
    const int F = p->F, C = p->C, T = p->KH * p->KW;
    size_t kept = 0, total = 0;
    for (int t = 0; t * 16 < F; ++t) {
        int f0 = 16 * t, nf = std::min(16, F - f0);
        for (size_t pos = 0; pos < (size_t)C * T; ++pos) {
            bool any = false;
            for (int j = 0; j < nf && !any; ++j) any = m[(size_t)(f0 + j) * C * T + pos] != 0;
            kept += any;
        }
        total += (size_t)C * T;
    }
    return total ? (double)kept / (double)total : 1.0;
}

// Ring format (see npas_internal.h): what the ring kernels stream through LDS.
static void build_ring(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    RingFormat &r = p->ring;
    const int F = p->F, C = p->C, T = p->KH * p->KW;
    r.present = true;
    r.taps = T;
    r.nfb = (F + 127) / 128;
    r.rg_ptr.assign(r.nfb + 1, 0);
    r.rg_chunk.clear();
    r.wimg.assign((size_t)r.nfb * (C / 64) * T * 16 * 512, 0);
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(w);
    size_t w0 = 0;
    for (int fb = 0; fb < r.nfb; ++fb) {
        r.rg_ptr[fb] = (int32_t)r.rg_chunk.size();
        const int f0 = 128 * fb;
        for (int cc = 0; cc < C / 64; ++cc) {
            r.rg_chunk.push_back((uint32_t)cc);
            for (int tap = 0; tap < T; ++tap, w0 += 16 * 512)
                for (int step = 0; step < 2; ++step)
                    for (int tile = 0; tile < 8; ++tile)
                        for (int lane = 0; lane < 64; ++lane)
                            for (int i = 0; i < 8; ++i) {
                                // row rr of tile (h, j) is filter 64 h + 4 rr + j of the block: the four tiles of a
                                // 64-filter half give each MFMA result column four consecutive filters
                                int rr = lane & 15, q = lane >> 4, f = f0 + 64 * (tile >> 2) + 4 * rr + (tile & 3);
                                int c = 64 * cc + 32 * step + 8 * q + i;
                                if (f >= F) continue;
                                size_t wi = ((size_t)f * C + c) * T + tap;
                                if (m[wi]) r.wimg[w0 + (size_t)(step * 8 + tile) * 512 + lane * 8 + i] = w16[wi];
                            }
        }
    }
    r.rg_ptr[r.nfb] = (int32_t)r.rg_chunk.size();
}

// Small-channel format (see npas_internal.h): the stem of an image network has 3 input channels,
// too few for 8-channel slabs; its whole reduction fits a handful of MFMA steps instead.
static void build_smallc(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    SmallCFormat &sc = p->smallc;
    const int F = p->F, C = p->C, T = p->KH * p->KW, K = C * T;
    sc.present = true;
    sc.nsteps = (K + 31) / 32;
    sc.wimg.assign((size_t)sc.nsteps * 4 * 512, 0);
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(w);
    for (int step = 0; step < sc.nsteps; ++step)
        for (int j = 0; j < 4; ++j)
            for (int lane = 0; lane < 64; ++lane)
                for (int i = 0; i < 8; ++i) {
                    const int r = lane & 15, q = lane >> 4, f = 4 * r + j, k = 32 * step + 8 * q + i;
                    if (f >= F || k >= K) continue;
                    const int tap = k / C, c = k % C;
                    const size_t wi = ((size_t)f * C + c) * T + tap;
                    if (m[wi]) sc.wimg[((size_t)(step * 4 + j) * 64 + lane) * 8 + i] = w16[wi];
                }
}

// Exact-list format (see npas_internal.h): built for 16-bit 1x1 / FC layers sparse enough for it to pay.
static void build_fc(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    FcFormat &fc = p->fc;
    const int F = p->F, C = p->C;
    fc.present = true;
    fc.ntiles = (F + 15) / 16;
    fc.tptr.assign(fc.ntiles + 1, 0);
    fc.koff.clear();
    fc.wimg.clear();
    fc.max_steps = 0;
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(w);
    std::vector<int> list;
    for (int t = 0; t < fc.ntiles; ++t) {
        const int f0 = 16 * t, nf = std::min(16, F - f0);
        list.clear();
        for (int c = 0; c < C; ++c) {
            bool any = false;
            for (int j = 0; j < nf && !any; ++j) any = m[(size_t)(f0 + j) * C + c] != 0;
            if (any) list.push_back(c);
        }
        const int steps = ((int)list.size() + 31) / 32;
        fc.tptr[t] = (int32_t)(fc.koff.size() / 32);
        fc.max_steps = std::max(fc.max_steps, steps);
        const size_t k0 = fc.koff.size(), w0 = fc.wimg.size();
        fc.koff.resize(k0 + (size_t)steps * 32, 0);
        fc.wimg.resize(w0 + (size_t)steps * 512, 0);
        for (size_t e = 0; e < list.size(); ++e) {
            fc.koff[k0 + e] = (uint16_t)(2 * list[e]);
            const size_t step = e / 32, q = (e % 32) / 8, i = e % 8;
            for (int r = 0; r < nf; ++r) {
                const size_t wi = (size_t)(f0 + r) * C + list[e];
                if (m[wi]) fc.wimg[w0 + step * 512 + (q * 16 + r) * 8 + i] = w16[wi];
            }
        }
    }
    fc.tptr[fc.ntiles] = (int32_t)(fc.koff.size() / 32);
}

// Lane-split fp32 format (see npas_internal.h): the sub-group lists of build_valu_f32, padded to multiples of 8.
static void build_wave_f32(npas_packed *p)
{
    const DeviceFormat &d = p->fmt;
    WaveF32Format &wf = p->wavef;
    wf.present = true;
    wf.wg_ptr.assign(1, 0);
    wf.kent.clear();
    wf.w.clear();
    for (int v = 0; v < d.nvg; ++v) {
        const int k0 = d.vg_ptr[v], k1 = d.vg_ptr[v + 1];
        for (int k = k0; k < k1; ++k) {
            wf.kent.push_back(d.vkent[k]);
            for (int j = 0; j < d.VB; ++j) wf.w.push_back(d.vw[(size_t)k * d.VB + j]);
        }
        const uint32_t fill = k1 > k0 ? d.vkent[k0] : 0u;
        while ((wf.kent.size() - (size_t)wf.wg_ptr[v]) % 8 != 0) {
            wf.kent.push_back(fill);
            for (int j = 0; j < d.VB; ++j) wf.w.push_back(0.0f);
        }
        wf.wg_ptr.push_back((int32_t)wf.kent.size());
    }
}

static void build_valu_f32(npas_packed *p, const uint8_t *m, const uint8_t *w)
{
    (void)m;
    DeviceFormat &d = p->fmt;
    d.variant = V_VALU_F32;
    const int Bf = p->Bf, C = p->C, KW = p->KW;
    int vb = 1;
    while (vb < Bf && vb < 8) vb *= 2;
    d.VB = vb;
    d.vg_ptr.clear();
    d.vg_f0.clear();
    d.vkent.clear();
    d.vw.clear();
    const float *wc = reinterpret_cast<const float *>(p->w_compact.data());
    for (int g = 0; g < p->G; ++g) {
        int k0 = p->grp_ptr[g], k1 = p->grp_ptr[g + 1];
        int nf = std::min(Bf, p->F - g * Bf);
        for (int j0 = 0; j0 < nf; j0 += vb) {
            d.vg_ptr.push_back((int32_t)d.vkent.size());
            d.vg_f0.push_back(g * Bf + j0);
            for (int k = k0; k < k1; ++k) {
                int pos = p->k_pos[k], tap = pos / C, c = pos % C;
                d.vkent.push_back((uint32_t)(tap / KW) << 24 | (uint32_t)(tap % KW) << 16 | (uint32_t)c);
                for (int j = 0; j < vb; ++j)
                    d.vw.push_back(j0 + j < Bf ? wc[(size_t)k * Bf + j0 + j] : 0.0f);
            }
        }
    }
    d.vg_ptr.push_back((int32_t)d.vkent.size());
    d.nvg = (int)d.vg_f0.size();
    (void)w;
}

int build_device_format(npas_packed *p, const std::vector<uint8_t> &mask_full, const void *w_host)
{
    if (p->C > 65535 || p->KH > 255 || p->KW > 255) {
        set_error("layer too large for the entry coding (C <= 65535, KH, KW <= 255)");
        return NPAS_E_SHAPE;
    }
    if (p->dtype == NPAS_F32) {
        build_valu_f32(p, mask_full.data(), (const uint8_t *)w_host);
        if (switches().force != FV_VALU) build_wave_f32(p);
    } else {
        // Element gather skips exactly what a 16-filter tile's groups punch, at about four
        // times the operand-fetch cost per kept position of the slab path; it pays once
        // fewer than a quarter of a tile's positions survive, and it is the only path for
        // channel counts that are not a multiple of 8 or filter counts that are not a multiple of 4.
        const int force = switches().force; // gather | slab | noring | nosmallc: testing aid
        const bool slab_ok = p->C % 8 == 0 && p->F % 4 == 0;
        p->fmt.density = union_density(p, mask_full.data());
        bool gather = !slab_ok || p->fmt.density < 0.25;
        if (slab_ok && (force == FV_GATHER || force == FV_SLAB)) gather = force == FV_GATHER;
        if (gather) build_mfma_gather(p, mask_full.data(), (const uint8_t *)w_host);
        else build_mfma_slab(p, mask_full.data(), (const uint8_t *)w_host);
        // layers with whole 64-channel chunks also get the streaming (ring) format, which the run calls
        // prefer for 1x1 layers without padding and k x k layers at stride 1 unless the layer is sparse
        // enough for the gather kernel to win (the ring multiplies every position)
        if (p->C % 64 == 0 && p->F % 4 == 0 && (double)((p->F + 127) / 128) * p->C * p->KH * p->KW * 256.0 < 256e6 &&
            force != FV_NORING)
            build_ring(p, mask_full.data(), (const uint8_t *)w_host);
        // sparse 1x1 / FC layers also get the exact per-tile lists (a staged activation row must fit in LDS sixteen times)
        if (p->KH == 1 && p->KW == 1 && p->F % 4 == 0 && p->C % 8 == 0 && p->C <= 4096 && p->fmt.density <= 0.5 && force != FV_NOFCGATHER)
            build_fc(p, mask_full.data(), (const uint8_t *)w_host);
        if (p->C < 8 && p->F <= 64 && p->F % 4 == 0 && p->C * p->KH * p->KW <= 160 && p->KH * p->KW > 1 &&
            force != FV_NOSMALLC)
            build_smallc(p, mask_full.data(), (const uint8_t *)w_host);
    }
    return NPAS_OK;
}

template <typename T>
static size_t place(std::vector<uint8_t> &blob, const std::vector<T> &v)
{
    size_t off = (blob.size() + 255) / 256 * 256;
    blob.resize(off + v.size() * sizeof(T));
    if (!v.empty()) memcpy(blob.data() + off, v.data(), v.size() * sizeof(T));
    return off;
}

int upload(npas_packed *p, void *hip_stream)
{
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        p->dev.device = -1; // host-only handle: export works, run calls fail loudly
        return NPAS_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return NPAS_OK;
    const DeviceFormat &d = p->fmt;
    std::vector<uint8_t> blob;
    size_t o_tc = place(blob, d.tc_ptr), o_ke = place(blob, d.kent), o_wf = place(blob, d.wfrag);
    size_t o_vp = place(blob, d.vg_ptr), o_vf = place(blob, d.vg_f0), o_vk = place(blob, d.vkent),
           o_vw = place(blob, d.vw);
    size_t o_rp = place(blob, p->ring.rg_ptr), o_rc = place(blob, p->ring.rg_chunk), o_ri = place(blob, p->ring.wimg);
    size_t o_sc = place(blob, p->smallc.wimg);
    size_t o_ft = place(blob, p->fc.tptr), o_fk = place(blob, p->fc.koff), o_fw = place(blob, p->fc.wimg);
    size_t o_wp = place(blob, p->wavef.wg_ptr), o_wk = place(blob, p->wavef.kent), o_ww = place(blob, p->wavef.w);
    blob.resize((blob.size() + 255) / 256 * 256 + 256);
    void *ptr = nullptr;
    hipError_t e = hipMalloc(&ptr, blob.size());
    if (e != hipSuccess) {
        set_error("hipMalloc(%zu) failed: %s", blob.size(), hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    // on the caller's stream; the source is a local buffer, so wait for the copy before it goes away
    e = hipMemcpyAsync(ptr, blob.data(), blob.size(), hipMemcpyHostToDevice, (hipStream_t)hip_stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)hip_stream);
    if (e != hipSuccess) {
        (void)hipFree(ptr);
        set_error("hipMemcpy to device failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    uint8_t *b = (uint8_t *)ptr;
    p->dev.device = dev;
    p->dev.blob = ptr;
    p->dev.bytes = blob.size();
    p->dev.tc_ptr = (const int32_t *)(b + o_tc);
    p->dev.kent = (const uint32_t *)(b + o_ke);
    p->dev.wfrag = b + o_wf;
    p->dev.vg_ptr = (const int32_t *)(b + o_vp);
    p->dev.vg_f0 = (const int32_t *)(b + o_vf);
    p->dev.vkent = (const uint32_t *)(b + o_vk);
    p->dev.vw = (const float *)(b + o_vw);
    p->dev.rg_ptr = (const int32_t *)(b + o_rp);
    p->dev.rg_chunk = (const uint32_t *)(b + o_rc);
    p->dev.wimg = b + o_ri;
    p->dev.scimg = b + o_sc;
    p->dev.fc_tptr = (const int32_t *)(b + o_ft);
    p->dev.fc_koff = (const uint16_t *)(b + o_fk);
    p->dev.fc_wimg = b + o_fw;
    p->dev.wv_ptr = (const int32_t *)(b + o_wp);
    p->dev.wv_kent = (const uint32_t *)(b + o_wk);
    p->dev.wv_w = (const float *)(b + o_ww);
    p->dev.zeros = b + blob.size() - 256; // the blob ends with 256 zero bytes
    return NPAS_OK;
}

static int finish_pack(npas_packed *p, const std::vector<uint8_t> &mask, const void *w, void *hip_stream, npas_packed **out)
{
    int rc = build_device_format(p, mask, w);
    if (rc == NPAS_OK) rc = upload(p, hip_stream);
    if (rc != NPAS_OK) {
        delete p;
        return rc;
    }
    *out = p;
    return NPAS_OK;
}

static int check_common(const void *w, const uint8_t *m, npas_packed **out, int F, int C, int KH, int KW, int Bf,
                        int Bc, int dt)
{
    if (!w || !m || !out) {
        set_error("NULL argument (w_host=%p mask_host=%p out=%p)", w, (const void *)m, (void *)out);
        return NPAS_E_NULL;
    }
    *out = nullptr;
    if (F <= 0 || C <= 0 || KH <= 0 || KW <= 0 || Bf <= 0 || Bc <= 0) {
        set_error("non-positive dimension (F=%d C=%d KH=%d KW=%d Bf=%d Bc=%d)", F, C, KH, KW, Bf, Bc);
        return NPAS_E_SHAPE;
    }
    if ((double)F * C * KH * KW > 2.0e9) {
        set_error("weight tensor too large (%d x %d x %d x %d)", F, C, KH, KW);
        return NPAS_E_SHAPE;
    }
    if (dt != NPAS_F32 && dt != NPAS_BF16 && dt != NPAS_F16) {
        set_error("unknown storage type %d", dt);
        return NPAS_E_DTYPE;
    }
    return NPAS_OK;
}

} // namespace npas

using namespace npas;

extern "C" {

const char *npas_last_error(void) { return npas::last_error(); }

void npas_debug_set_switches(const char *force_variant, int no_balance)
{
    npas::Switches &sw = npas::switches_rw();
    sw.force = npas::parse_force(force_variant);
    sw.no_balance = no_balance != 0;
}

int npas_pack_block_punched(const void *w_host, const uint8_t *mask_host, int F, int C, int KH, int KW, int Bf,
                            int Bc, npas_dtype dt, void *hip_stream, npas_packed **out)
{
    int rc = check_common(w_host, mask_host, out, F, C, KH, KW, Bf, Bc, dt);
    if (rc) return rc;
    size_t n = (size_t)F * C * KH * KW;
    if ((rc = check_mask_values(mask_host, n))) return rc;
    if ((rc = validate_block_punched(mask_host, F, C, KH, KW, Bf))) return rc;
    npas_packed *p = new npas_packed;
    p->scheme = NPAS_SCHEME_BLOCK_PUNCHED;
    p->dtype = dt;
    p->F = F; p->C = C; p->KH = KH; p->KW = KW; p->Bf = std::min(Bf, F); p->Bc = std::min(Bc, C);
    pack_canonical(p, (const uint8_t *)w_host, mask_host);
    std::vector<uint8_t> mask(mask_host, mask_host + n);
    return finish_pack(p, mask, w_host, hip_stream, out);
}

int npas_pack_fc_block(const void *w_host, const uint8_t *mask_host, int OUT, int IN, int Br, int Bcol,
                       npas_dtype dt, void *hip_stream, npas_packed **out)
{
    int rc = check_common(w_host, mask_host, out, OUT, IN, 1, 1, Br, Bcol, dt);
    if (rc) return rc;
    size_t n = (size_t)OUT * IN;
    if ((rc = check_mask_values(mask_host, n))) return rc;
    if ((rc = validate_fc_block(mask_host, OUT, IN, Br, Bcol))) return rc;
    npas_packed *p = new npas_packed;
    p->scheme = NPAS_SCHEME_FC_BLOCK;
    p->dtype = dt;
    p->F = OUT; p->C = IN; p->KH = 1; p->KW = 1; p->Bf = std::min(Br, OUT); p->Bc = std::min(Bcol, IN);
    pack_canonical(p, (const uint8_t *)w_host, mask_host);
    std::vector<uint8_t> mask(mask_host, mask_host + n);
    return finish_pack(p, mask, w_host, hip_stream, out);
}

int npas_pack_pattern(const void *w_host, const uint8_t *mask_host, int F, int C, const uint8_t *library_host,
                      int n_pat, npas_dtype dt, void *hip_stream, npas_packed **out)
{
    int rc = check_common(w_host, mask_host, out, F, C, 3, 3, 1, 1, dt);
    if (rc) return rc;
    if (!library_host) {
        set_error("NULL pattern library");
        return NPAS_E_NULL;
    }
    if (n_pat <= 0 || n_pat > 254) {
        set_error("n_pat = %d outside 1..254", n_pat);
        return NPAS_E_SHAPE;
    }
    size_t n = (size_t)F * C * 9;
    if ((rc = check_mask_values(mask_host, n))) return rc;
    if ((rc = check_mask_values(library_host, (size_t)n_pat * 9))) return rc;
    const int esz = dtype_size(dt);
    npas_packed *p = new npas_packed;
    p->scheme = NPAS_SCHEME_PATTERN;
    p->dtype = dt;
    p->F = F; p->C = C; p->KH = 3; p->KW = 3; p->Bf = 1; p->Bc = 1;
    p->n_pat = n_pat;
    p->library.assign(library_host, library_host + (size_t)n_pat * 9);
    p->pat_id.assign((size_t)F * C, 255);
    p->w4.assign((size_t)F * C * 4 * esz, 0);
    const uint8_t *w = (const uint8_t *)w_host;
    for (size_t k = 0; k < (size_t)F * C; ++k) {
        const uint8_t *mk = mask_host + k * 9;
        int nz = 0;
        for (int t = 0; t < 9; ++t) nz += mk[t];
        if (nz == 0) continue; // removed kernel (connectivity pruning)
        int id = -1;
        for (int q = 0; q < n_pat && id < 0; ++q)
            if (memcmp(mk, library_host + (size_t)q * 9, 9) == 0) id = q;
        if (id < 0) {
            set_error("kernel (f=%zu, c=%zu) keeps %d taps that match no library pattern", k / C, k % C, nz);
            delete p;
            return NPAS_E_MASK_NOT_IN_LIBRARY;
        }
        p->pat_id[k] = (uint8_t)id;
        int j = 0;
        for (int t = 0; t < 9 && j < 4; ++t)
            if (mk[t]) memcpy(&p->w4[(k * 4 + j++) * esz], w + (k * 9 + t) * esz, esz);
    }
    pack_canonical(p, w, mask_host);
    std::vector<uint8_t> mask(mask_host, mask_host + n);
    return finish_pack(p, mask, w_host, hip_stream, out);
}

int npas_pack_depthwise3x3(const void *w_host, int C, npas_dtype dt, void *hip_stream, npas_packed **out)
{
    if (!w_host || !out) {
        set_error("NULL argument (w_host=%p out=%p)", w_host, (void *)out);
        return NPAS_E_NULL;
    }
    *out = nullptr;
    if (C <= 0 || C > 65535) {
        set_error("bad channel count %d", C);
        return NPAS_E_SHAPE;
    }
    if (dt != NPAS_F32 && dt != NPAS_BF16 && dt != NPAS_F16) {
        set_error("unknown storage type %d", (int)dt);
        return NPAS_E_DTYPE;
    }
    npas_packed *p = new npas_packed;
    p->scheme = NPAS_SCHEME_DEPTHWISE;
    p->dtype = dt;
    p->F = C; p->C = C; p->KH = 3; p->KW = 3; p->Bf = 1; p->Bc = 1; p->G = 0;
    p->grp_ptr.assign(1, 0);
    const size_t esz = dt == NPAS_F32 ? 4 : 2;
    p->w_compact.assign((const uint8_t *)w_host, (const uint8_t *)w_host + (size_t)C * 9 * esz);
    // device order: tap-major [9][C], so that a thread's channel vector of one tap is one 16-byte load
    p->fmt.variant = V_DEPTHWISE;
    if (dt == NPAS_F32) {
        const float *w = (const float *)w_host;
        p->fmt.vw.resize((size_t)9 * C);
        for (int c = 0; c < C; ++c)
            for (int t = 0; t < 9; ++t) p->fmt.vw[(size_t)t * C + c] = w[(size_t)c * 9 + t];
    } else {
        const uint16_t *w = (const uint16_t *)w_host;
        p->fmt.wfrag.resize((size_t)9 * C);
        for (int c = 0; c < C; ++c)
            for (int t = 0; t < 9; ++t) p->fmt.wfrag[(size_t)t * C + c] = w[(size_t)c * 9 + t];
    }
    int rc = upload(p, hip_stream);
    if (rc != NPAS_OK) {
        delete p;
        return rc;
    }
    *out = p;
    return NPAS_OK;
}

int npas_packed_info(const npas_packed *p, int64_t info[16])
{
    if (!p || !info) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    const DeviceFormat &d = p->fmt;
    size_t dev_bytes = d.tc_ptr.size() * 4 + d.kent.size() * 4 + d.wfrag.size() * 2 + d.vg_ptr.size() * 4 +
                       d.vg_f0.size() * 4 + d.vkent.size() * 4 + d.vw.size() * 4;
    if (p->ring.present) // the format the run calls use for this layer
        dev_bytes = p->ring.rg_ptr.size() * 4 + p->ring.rg_chunk.size() * 4 + p->ring.wimg.size() * 2;
    int64_t v[16] = {p->scheme, p->dtype, p->F, p->C, p->KH, p->KW, p->Bf, p->Bc, p->G,
                     (int64_t)p->k_pos.size(), p->n_pat, p->dev.device >= 0, d.variant,
                     (int64_t)dev_bytes, (int64_t)p->w_compact.size(), 0};
    memcpy(info, v, sizeof(v));
    return NPAS_OK;
}

int npas_packed_export(const npas_packed *p, int32_t *grp_ptr, int32_t *k_pos, void *w_compact, uint8_t *pat_id,
                       void *w4)
{
    if (!p) {
        set_error("NULL handle");
        return NPAS_E_NULL;
    }
    if (grp_ptr) memcpy(grp_ptr, p->grp_ptr.data(), p->grp_ptr.size() * sizeof(int32_t));
    if (k_pos && !p->k_pos.empty()) memcpy(k_pos, p->k_pos.data(), p->k_pos.size() * sizeof(int32_t));
    if (w_compact && !p->w_compact.empty()) memcpy(w_compact, p->w_compact.data(), p->w_compact.size());
    if (pat_id || w4) {
        if (p->scheme != NPAS_SCHEME_PATTERN) {
            set_error("pat_id / w4 requested from a layer that is not pattern-pruned");
            return NPAS_E_SHAPE;
        }
        if (pat_id) memcpy(pat_id, p->pat_id.data(), p->pat_id.size());
        if (w4) memcpy(w4, p->w4.data(), p->w4.size());
    }
    return NPAS_OK;
}

void npas_free(npas_packed *p)
{
    if (!p) return;
    if (p->dev.blob) (void)hipFree(p->dev.blob);
    delete p;
}

} // extern "C"
