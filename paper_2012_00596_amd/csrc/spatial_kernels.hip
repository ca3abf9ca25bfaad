// gfx950 kernels of libnpas for k x k layers with whole 64-channel chunks: spatial_ring (weights streamed through an
// LDS ring, 3 x 3 at stride 2 as four phase planes) and spatial_resident (at most 64 filters: all weights stay in LDS).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>

#include "npas_internal.h"
#include "device_util.h"

namespace npas {

// ------------------------------------------------------------------------------
// spatial_ring: k x k layers at stride 1 (3 x 3 at stride 2: see S2 at the kernel) with C a multiple of 64.  A stage is one tap of one
// 64-channel chunk (two MFMA steps); its 16 weight images (16 KB) go through a ring of `depth`
// LDS slots.  The activations of a chunk are the halo patch of the output tile
// ([patch pixel][64 channels], 128 B per pixel, XOR-swizzled by the patch pixel index),
// double-buffered: while the KH*KW taps of chunk c are multiplied out of one buffer, the
// patch of chunk c+1 is fetched into the other.  Padding pixels are fetched from a block of
// zeros.  A tile is NI images x TH x TW output pixels (several images per tile keep the 256
// MFMA columns busy on 7x7 and 14x14 maps).
//
// The workgroup has three kinds of waves, because a wave's vector-memory operations retire
// in order: a patch load (HBM latency) issued ahead of a weight load (L2 latency) would
// hold it back, and either would hold back a multiplying wave.
//   waves 0-7   multiply: 4 pixel groups x 2 filter groups, 64 x 64 outputs each; no
//               global loads in their main loop
//   wave 8      fetches the weight stages, depth-1 stages ahead
//   waves 9-15  fetch the patches, a few blocks per stage, finishing well before the chunk ends
// One s_barrier per stage, executed by all sixteen: a fetching wave first waits for the loads
// of the stage about to be multiplied; after the barrier the slot (or patch buffer) of the
// stage before is free to be refilled.
constexpr uint32_t kSpatialWStage = 16384;
// Tiles of 64 PG pixels x 128 filters.  PG == 4: eight multiplying waves, 4 pixel groups of 64 x 2 filter groups
// of 64.  PG == 2 (launches whose 256-pixel tiles would leave most CUs without one): also eight, 4 pixel
// groups of 32 x 2 filter groups of 64.
constexpr int spatial_waves(int pg) { return pg == 2 ? 8 : 2 * pg; } // multiplying waves
// Fetching waves: one brings the weight stages (its sixteen lane-linear loads per stage are issued in a few hundred
// cycles), seven the patch, whose loads cost their wave far more (pixel table entry from LDS behind the multiplying
// waves' reads, bounds, address arithmetic).  With four of each the patch waves of the stride-2 mode were the last at
// every second barrier by up to two stage times: 58.8 / 55.0 / 47.8 us on the three stride-2 layers of the 50-layer stack
// at batch 128, 57.8 / 53.2 / 47.6 with 3 + 5, 53.1 / 50.9 / 45.3 with 2 + 6, 51.2 / 49.6 / 45.2 with 1 + 7; the stride-1
// layers are the same with either split (38.5 / 34.1 / 39.4), and 2.5 % slower with 1 + 3 (twelve waves, 168 registers each).
constexpr int kSpatialFetchTotal = 8;
constexpr int spatial_threads(int pg) { return (spatial_waves(pg) + kSpatialFetchTotal) * 64; }

struct SpatialItem {
    int n0, ty0, tx0, fb;
};

__device__ __forceinline__ SpatialItem spatial_item(const SpatialRingArgs &a, uint32_t item)
{
    SpatialItem it;
    uint32_t rest = item / (uint32_t)a.nfb;
    it.fb = (int)(item - rest * (uint32_t)a.nfb);
    const uint32_t txi = rest % (uint32_t)a.tilesX;
    rest /= (uint32_t)a.tilesX;
    const uint32_t tyi = rest % (uint32_t)a.tilesY;
    it.n0 = (int)(rest / (uint32_t)a.tilesY) * a.NI;
    it.ty0 = (int)tyi * a.TH;
    it.tx0 = (int)txi * a.TW;
    return it;
}

// Output pixel table of a tile shape (the same for every item): entry m = image << 16 | row << 8 | column of tile
// pixel m inside the tile, ~0 past the tile's pixels.  1 KB of LDS (256 entries).
__device__ __forceinline__ void spatial_out_table(const SpatialRingArgs &a, uint32_t *tab, int npix, int tid, int nthreads)
{
    const int thtw = a.TH * a.TW;
    for (int m = tid; m < npix; m += nthreads) {
        const uint32_t img = fastdiv((uint32_t)m, a.div_thtw), r = (uint32_t)m - img * (uint32_t)thtw;
        const uint32_t ty = fastdiv(r, a.div_tw), tx = r - ty * (uint32_t)a.TW;
        tab[m] = m < a.NI * thtw ? (img << 16 | ty << 8 | tx) : 0xffffffffu;
    }
}

// Epilogue of a multiplying wave: bias, residual, activation, round, store.  Result register i of acc[j][s] is tile
// pixel m0 + 16 s + i (m0 = the wave's first pixel + 4 q), filter fcol + j: a lane writes 4 consecutive filters of a
// pixel, the 16 lanes of a quarter wave one whole 128-byte run of its row.  `ot` points at the lane's entry m0 of
// the output pixel table.  The activation kind and the residual are wave-uniform and compiled in (a branch per
// value and a pixel decode by division per store made this epilogue as long as five stages of the main loop).
template <int DT, int S, bool HS, bool RES>
__device__ __forceinline__ void spatial_store_tile(const SpatialRingArgs &a, const SpatialItem &it, const uint8_t *ot,
                                                   const f32x4 (&acc)[4][S], float4 b4, int fcol, Clamp cl)
{
    if (fcol >= a.F) return;
    const uint16_t *rp = reinterpret_cast<const uint16_t *>(a.residual);
    uint16_t *yp = reinterpret_cast<uint16_t *>(a.y);
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const uint4 e4 = *reinterpret_cast<const uint4 *>(ot + s * 64);
        const uint32_t ev[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t e = ev[i];
            const int n = it.n0 + (int)(e >> 16), oy = it.ty0 + (int)((e >> 8) & 255u), ox = it.tx0 + (int)(e & 255u);
            if (e == 0xffffffffu || n >= a.N || oy >= a.Ho || ox >= a.Wo) continue;
            const size_t o = (size_t)(uint32_t)((n * a.Ho + oy) * a.Wo + ox) * (size_t)(uint32_t)a.F + (size_t)(uint32_t)fcol;
            float v[4] = {acc[0][s][i] + b4.x, acc[1][s][i] + b4.y, acc[2][s][i] + b4.z, acc[3][s][i] + b4.w};
            if (RES) {
                const uint2 r2 = *reinterpret_cast<const uint2 *>(rp + o);
                v[0] += from_storage<DT>((uint16_t)(r2.x & 0xffffu));
                v[1] += from_storage<DT>((uint16_t)(r2.x >> 16));
                v[2] += from_storage<DT>((uint16_t)(r2.y & 0xffffu));
                v[3] += from_storage<DT>((uint16_t)(r2.y >> 16));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = HS ? v[j] * __builtin_amdgcn_fmed3f(v[j] + 3.0f, 0.0f, 6.0f) * (1.0f / 6.0f) : __builtin_amdgcn_fmed3f(v[j], cl.lo, cl.hi);
            uint2 out;
            out.x = pack2<DT>(v[0], v[1]);
            out.y = pack2<DT>(v[2], v[3]);
            *reinterpret_cast<uint2 *>(yp + o) = out;
        }
    }
}
template <int DT, int S>
__device__ __forceinline__ void spatial_epilogue(const SpatialRingArgs &a, const SpatialItem &it, const uint8_t *ot,
                                                 const f32x4 (&acc)[4][S], float4 b4, int fcol, Clamp cl)
{
    if (cl.hs) {
        if (a.residual) spatial_store_tile<DT, S, true, true>(a, it, ot, acc, b4, fcol, cl);
        else spatial_store_tile<DT, S, true, false>(a, it, ot, acc, b4, fcol, cl);
    } else {
        if (a.residual) spatial_store_tile<DT, S, false, true>(a, it, ot, acc, b4, fcol, cl);
        else spatial_store_tile<DT, S, false, false>(a, it, ot, acc, b4, fcol, cl);
    }
}

// S2: stride 2, 3 x 3, pad 1.  The patch is kept as four phase planes (input rows and columns of one parity
// each), every plane a dense (TH + 1) x (TW + 1) grid, so that a tap reads one plane at an offset of 0 or 1
// rows / columns exactly as at stride 1.  The taps are walked plane by plane (4 + 2 + 2 + 1 stages); a plane's
// buffer is refilled with the next chunk's pixels as soon as its last tap is done, which leaves every refill
// at least five stages: one copy of the patch in LDS instead of two.
template <int DT, int PG, bool S2>
__global__ __launch_bounds__(spatial_threads(PG)) void spatial_ring_kernel(SpatialRingArgs a)
{
    // PG == 4: 8 waves of 64 pixels x 64 filters.  PG == 2: 8 waves of 32 x 64 (two per SIMD; four waves of
    // 64 x 64, one per SIMD, left the operand latency of every step exposed)
    constexpr int NCW = spatial_waves(PG), S = PG == 2 ? 2 : 4, NB = 2 * S;
    constexpr int kSpatialThreads = spatial_threads(PG);
    constexpr int kWeightWaves = 1, kPatchWaves = kSpatialFetchTotal - kWeightWaves;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lbase = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint32_t nwg = gridDim.x;
    const uint32_t nitems = (uint32_t)(a.tilesN * a.tilesY * a.tilesX * a.nfb);
    const int T = a.KH * a.KW, nch = a.C >> 6;
    const uint32_t ppb = (uint32_t)a.npb * 1024u;      // bytes of one patch buffer
    const uint32_t wring = (S2 ? 4u : 2u) * ppb;       // LDS offset of the weight ring (after two patch buffers, or four planes)
    const uint32_t D = (uint32_t)a.depth;              // weight stages in the ring
    const uint32_t lbias = wring + D * kSpatialWStage; // two 1 KB bias buffers (item parity)
    const uint32_t ltab = lbias + 2048u;               // patch pixel -> (image, row, column), 4 B each
    const uint32_t lotab = ltab + (S2 ? 4u : 1u) * (uint32_t)a.npb * 32u; // tile pixel -> (image, row, column) inside the tile
    uint32_t c_item = xcd_remap(blockIdx.x, nwg);
    if (c_item >= nitems) return;
    SpatialItem it = spatial_item(a, c_item);
    const int phpw = a.PH * a.PW;

    // patch pixel table (the same for every item): img << 20 | row << 10 | column, ~0 past the end
    // (at stride 2: per plane; rows 2 py - ph + 1 and columns 2 px - pw + 1 of the tile's input window, where
    // planes 0, 1 hold the odd rows (ph = 1: taps kh = 0, 2) and planes 0, 2 the odd columns (pw = 1: kw = 0, 2))
    for (int idx = tid; idx < a.npb * 8 * (S2 ? 4 : 1); idx += kSpatialThreads) {
        const int plane = S2 ? idx / (a.npb * 8) : 0, pp = idx - plane * (a.npb * 8);
        const uint32_t img = fastdiv((uint32_t)pp, a.div_phpw), r = (uint32_t)pp - img * (uint32_t)phpw;
        const uint32_t py = fastdiv(r, a.div_pw), px = r - py * (uint32_t)a.PW;
        uint32_t e = (int)img < a.NI ? (img << 20 | py << 10 | px) : 0xffffffffu;
        if (S2 && (int)img < a.NI) {
            const uint32_t ph = plane < 2 ? 1u : 0u, pw = (plane & 1) ? 0u : 1u;
            const bool used = (ph == 1u || (int)py < a.TH) && (pw == 1u || (int)px < a.TW);
            e = used ? (img << 20 | (2u * py - ph + 1u) << 10 | (2u * px - pw + 1u)) : 0xffffffffu;
        }
        reinterpret_cast<uint32_t *>(lds + ltab)[idx] = e;
    }
    spatial_out_table(a, reinterpret_cast<uint32_t *>(lds + lotab), 64 * PG, tid, kSpatialThreads);
    __syncthreads();

    if (wave >= NCW + kWeightWaves) {
        // ---- patch fetch ------------------------------------------------------------------
        const int wl = __builtin_amdgcn_readfirstlane(wave - NCW - kWeightWaves); // (the compiler cannot see that a wave index is uniform)
        const uint8_t *xb = reinterpret_cast<const uint8_t *>(a.x);
        const uint8_t *zb = reinterpret_cast<const uint8_t *>(a.zeros) + (uint32_t)(lane & 7) * 16u;
        const uint32_t pcv = (uint32_t)((lane & 7) ^ (lane >> 3)) * 16u;
        const int nblk = max(0, (a.npb - wl + kPatchWaves - 1) / kPatchWaves); // this wave's blocks: wl, wl + kPatchWaves, ...
        // blocks per stage, spread over all but the chunk's last stage
        const int per = (nblk + max(1, T - 1) - 1) / max(1, T - 1);
        // Blocks first + 4 k, k in [k0, k1), of the pixel table go to LDS at dst + 4096 k; (y0, x0) is the tile origin in
        // input coordinates.  Four at a time: the table entries are read first and the four address computations are
        // independent, so they overlap (the loads themselves are ordered against the table reads); one at a time a
        // load held the wave for some 500 cycles, measured around the barriers.  Keeping an item's offsets in
        // registers instead (they only move by 128 bytes per chunk) compiled to copies and branches and was slower.
        auto fetch_blocks = [&](const SpatialItem &pi, int y0, int x0, int cc, int first, uint32_t dst, int k0, int k1) __attribute__((always_inline)) {
            const uint32_t *tab = reinterpret_cast<const uint32_t *>(lds + ltab) + first * 8 + (lane >> 3);
            for (; k0 < k1; k0 += 4) {
                uint32_t e[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) e[j] = tab[min(k0 + j, k1 - 1) * (kPatchWaves * 8)];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (k0 + j >= k1) break;
                    const int n = pi.n0 + (int)(e[j] >> 20), iy = y0 + (int)((e[j] >> 10) & 1023u), ix = x0 + (int)(e[j] & 1023u);
                    const bool inb = e[j] != 0xffffffffu && n < a.N && (uint32_t)iy < (uint32_t)a.H && (uint32_t)ix < (uint32_t)a.W;
                    // the offset is formed for every lane (24-bit multiplies: the launcher checks N H W < 2^24) and the
                    // source selected afterwards, so that the loads of a group are straight-line code the compiler can
                    // interleave: behind a branch per load each was a chain of some 25 dependent operations
                    const uint32_t pix = __umul24(__umul24((uint32_t)n, (uint32_t)a.H) + (uint32_t)iy, (uint32_t)a.W) + (uint32_t)ix;
                    const uint32_t off = __umul24(pix & 0xffffffu, (uint32_t)a.C * 2u) + ((uint32_t)cc * 128u + pcv);
                    const uint64_t sx = (uint64_t)(uintptr_t)xb + off, sz = (uint64_t)(uintptr_t)zb;
                    const uint8_t *src = reinterpret_cast<const uint8_t *>(inb ? sx : sz);
                    lds_dma16(src, dst + (uint32_t)(k0 + j) * (kPatchWaves * 1024u));
                }
            }
        };
        // blocks [k0, k1) of this wave's share of the patch of (item pi, chunk cc)
        auto patch = [&](const SpatialItem &pi, int cc, uint32_t buf, int k0, int k1) __attribute__((always_inline)) {
            fetch_blocks(pi, pi.ty0 - a.pad, pi.tx0 - a.pad, cc, wl, lbase + buf * ppb + (uint32_t)wl * 1024u, k0, min(k1, nblk));
        };
        // stride 2: this wave's blocks of one plane of (item pi, chunk cc)
        auto plane_fetch = [&](const SpatialItem &pi, int cc, int plane) __attribute__((always_inline)) {
            fetch_blocks(pi, 2 * pi.ty0 - a.pad, 2 * pi.tx0 - a.pad, cc, plane * a.npb + wl, lbase + (uint32_t)(plane * a.npb + wl) * 1024u, 0, nblk);
        };
        // bias of an item's 128 filters (512 B; lanes 32-63 fetch a copy that nobody reads)
        auto bias_block = [&](const SpatialItem &pi, uint32_t buf) __attribute__((always_inline)) {
            if (!a.bias || wl != 0) return;
            const int f = pi.fb * 128 + (lane & 31) * 4;
            lds_dma16(a.bias + (f < a.F ? f : 0), lbase + lbias + buf * 1024u);
        };
        if (S2) {
            // Stages 0-3 read plane 0, 4-5 plane 1, 6-7 plane 2, 8 plane 3.  Issue order, one burst of nblk loads
            // each: ... plane 3 of this chunk after barrier 0, then planes 0, 1, 2 of the next chunk after
            // barriers 4, 6, 8.  A plane is awaited at its first stage; two bursts were issued after it by then
            // (fewer at the very end), and a wave's loads complete in order.
            plane_fetch(it, 0, 0);
            plane_fetch(it, 0, 1);
            plane_fetch(it, 0, 2);
            bias_block(it, 0);
            uint32_t bbuf = 0;
            for (;;) {
                const bool more_items = c_item + nwg < nitems;
                SpatialItem nit = it;
                if (more_items) nit = spatial_item(a, c_item + nwg);
                for (int cc = 0; cc < nch; ++cc) {
                    const bool within = cc + 1 < nch, have_next = within || more_items;
                    const SpatialItem &ni = within ? it : nit;
                    const int ncc = within ? cc + 1 : 0;
                    for (int st = 0; st < 9; ++st) {
                        if (st == 0 || st == 4) wait_vmcnt((uint32_t)(2 * nblk));
                        else if (st == 6) wait_vmcnt((uint32_t)(have_next ? 2 * nblk : nblk));
                        else if (st == 8) wait_vmcnt((uint32_t)(have_next ? 2 * nblk : 0));
                        __builtin_amdgcn_s_barrier();
                        if (st == 0) {
                            plane_fetch(it, cc, 3);
                            if (!within && more_items) bias_block(nit, bbuf ^ 1u);
                        } else if (have_next && (st == 4 || st == 6 || st == 8)) plane_fetch(ni, ncc, (st - 4) >> 1);
                    }
                }
                if (!more_items) break;
                c_item += nwg;
                it = nit;
                bbuf ^= 1u;
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            return;
        }
        patch(it, 0, 0, 0, nblk);
        bias_block(it, 0);
        uint32_t pbuf = 0, bbuf = 0;
        for (;;) {
            const bool more_items = c_item + nwg < nitems;
            SpatialItem nit = it;
            if (more_items) nit = spatial_item(a, c_item + nwg);
            for (int cc = 0; cc < nch; ++cc) {
                const bool within = cc + 1 < nch;
                for (int tap = 0; tap < T; ++tap) {
                    if (tap == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this chunk's patch has landed
                    __builtin_amdgcn_s_barrier();
                    if (within) patch(it, cc + 1, pbuf ^ 1u, tap * per, (tap + 1) * per);
                    else if (more_items) {
                        patch(nit, 0, pbuf ^ 1u, tap * per, (tap + 1) * per);
                        if (tap == 0) bias_block(nit, bbuf ^ 1u);
                    }
                }
                pbuf ^= 1u;
            }
            if (!more_items) break;
            c_item += nwg;
            it = nit;
            bbuf ^= 1u;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    if (wave >= NCW) {
        // ---- weight stage fetch: this wave's share of the 16 images of every stage -----------
        const int wl = __builtin_amdgcn_readfirstlane(wave - NCW);
        const int img0 = 16 * wl / kWeightWaves, kImgs = 16 * (wl + 1) / kWeightWaves - img0; // 4 each, or 5, 5, 6
        const uint8_t *wb = reinterpret_cast<const uint8_t *>(a.wimg) + (uint32_t)img0 * 1024u + (uint32_t)lane * 16u;
        uint32_t p_item = c_item, p_slot = 0;
        int p_fb = it.fb, p_cc = 0, p_tap = 0;
        bool p_done = false;
        auto produce_w = [&]() __attribute__((always_inline)) { // always issues its 4 loads; past the end it repeats the last stage
            // stride 2: the taps in plane order (kh, kw both even; kw = 1; kh = 1; the centre)
            const int tapi = S2 ? (int)((0x453718620ull >> (4 * p_tap)) & 15ull) : p_tap;
            const uint8_t *wsrc = wb + (size_t)((p_fb * nch + p_cc) * T + tapi) * kSpatialWStage;
            const uint32_t dst = lbase + wring + p_slot * kSpatialWStage + (uint32_t)img0 * 1024u;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (i < kImgs) lds_dma16(wsrc + i * 1024, dst + (uint32_t)i * 1024u);
            if (++p_slot == D) p_slot = 0;
            if (!p_done) {
                if (++p_tap == T) {
                    p_tap = 0;
                    if (++p_cc == nch) {
                        p_cc = 0;
                        if (p_item + nwg < nitems) {
                            p_item += nwg;
                            p_fb = spatial_item(a, p_item).fb;
                        } else {
                            p_done = true;
                            p_cc = nch - 1;
                            p_tap = T - 1;
                        }
                    }
                }
            }
        };
        for (uint32_t i = 0; i + 1 < D; ++i) produce_w();
        for (;;) {
            const bool more_items = c_item + nwg < nitems;
            for (int st = 0; st < nch * T; ++st) {
                // at most the D-2 stages issued after the one about to be multiplied stay in flight
                wait_vmcnt((uint32_t)kImgs * (D - 2u)); // (at most 6 x 4: a wave can have 63 loads in flight)
                __builtin_amdgcn_s_barrier();
                produce_w(); // the stage D-1 ahead, into the slot the barrier freed
            }
            if (!more_items) break;
            c_item += nwg;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---- multiply ------------------------------------------------------------------------
    const int wp = wave >> 1, wf = wave & 1;
    const Clamp cl = clamp_of(a.act);
    const int thtw = a.TH * a.TW;
    // where this lane's operand rows (tile pixels 64 wp + 16 s + n16) sit in the patch (the same for every item)
    uint32_t pb0[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const uint32_t m = (uint32_t)(wp * (16 * S) + s * 16 + n16);
        const uint32_t img = fastdiv(m, a.div_thtw), r = m - img * (uint32_t)thtw;
        const uint32_t ty = fastdiv(r, a.div_tw), tx = r - ty * (uint32_t)a.TW;
        const bool valid = (int)m < a.NI * thtw;
        pb0[s] = valid ? img * (uint32_t)phpw + ty * (uint32_t)a.PW + tx : 0u;
    }
    uint32_t c_slot = 0, pbuf = 0, bbuf = 0;
    const uint32_t arow = (uint32_t)(wf * 4) * 1024u + (uint32_t)lane * 16u;

    for (;;) { // one item per iteration
        f32x4 acc[4][S];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int s = 0; s < S; ++s) acc[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};
        const bool more_items = c_item + nwg < nitems;

        for (int cc = 0; cc < nch; ++cc) {
            const uint8_t *pbp = lds + (S2 ? 0u : pbuf * ppb);
            uint32_t kh = 0, kw = 0;
            for (int tap = 0; tap < T; ++tap) {
                __builtin_amdgcn_s_barrier(); // this stage's weights (and, at its first stage, a chunk's patch or plane) are in LDS
                asm volatile("" ::: "memory");
                const uint8_t *wsp = lds + wring + c_slot * kSpatialWStage + arow;
                if (++c_slot == D) c_slot = 0;
                uint32_t toff = kh * (uint32_t)a.PW + kw;
                if (++kw == (uint32_t)a.KW) { kw = 0; ++kh; }
                if (S2) { // stage `tap` of the plane order: which plane, and 0 or 1 rows / columns into it
                    const uint32_t pl = (uint32_t)a.npb * 8u, st = (uint32_t)tap;
                    toff = st < 4u ? (st >> 1) * (uint32_t)a.PW + (st & 1u)
                         : st < 6u ? pl + (st - 4u) * (uint32_t)a.PW
                         : st < 8u ? 2u * pl + (st - 6u)
                                   : 3u * pl;
                }
                // Per step: its 4 + S fragments are asked for, then its 4 S MFMAs follow.  The scheduling barrier keeps
                // the reads together (left alone the compiler holds half of the pixel fragments back until just before
                // their use: 4 % slower).  Measured against this on 28 x 28 x 128 / 14 x 14 x 256 / 7 x 7 x 512 at batch 128
                // (38.0 / 34.0 / 39.1 us): all twelve fragments of a stage asked for at once and the weight tiles of the
                // second step rotated into the first step's registers 41.8 / 37.5 / 39.7; the first fragments of the
                // next stage read before its barrier and one pixel fragment in flight per wave 40.3 / 35.8 / 42.9, with
                // two in flight (spills) 48.4 / 41.1 / 51.8; pixel fragments three ahead of their use 46 / 39 / 52.
#pragma unroll
                for (int step = 0; step < 2; ++step) {
                    uint4 A[4], B[S];
#pragma unroll
                    for (int j = 0; j < 4; ++j) A[j] = *reinterpret_cast<const uint4 *>(wsp + step * 8192 + j * 1024);
#pragma unroll
                    for (int s2 = 0; s2 < S; ++s2) {
                        const uint32_t pp = pb0[s2] + toff;
                        B[s2] = *reinterpret_cast<const uint4 *>(pbp + pp * 128u + ((((uint32_t)(4 * step + q)) ^ (pp & 7u)) << 4));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int s2 = 0; s2 < S; ++s2)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[j][s2] = mfma16<DT>(B[s2], A[j], acc[j][s2]);
                }
            }
            pbuf ^= 1u;
        }
        // ---- bias (from LDS), residual, activation, round, store ------------------------------
        // The patch is the MFMA's row operand and the weight images its column operand, and row r of weight tile j
        // is filter 4r + j of the wave's 64: result register i of (j, s) is tile pixel 16 S wp + 16 s + 4q + i,
        // filter 4 n16 + j.
        {
            float4 b4 = float4{0.f, 0.f, 0.f, 0.f};
            if (a.bias) b4 = *reinterpret_cast<const float4 *>(lds + lbias + bbuf * 1024u + (uint32_t)(wf * 64 + 4 * n16) * 4u);
            spatial_epilogue<DT, S>(a, it, lds + lotab + (uint32_t)(wp * (16 * S) + 4 * q) * 4u, acc, b4, it.fb * 128 + wf * 64 + 4 * n16, cl);
        }
        if (!more_items) break;
        c_item += nwg;
        it = spatial_item(a, c_item);
        bbuf ^= 1u;
    }
}

template <int DT, int PG, bool S2 = false> static void launch_spatial_inst(const SpatialRingArgs &a, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    auto kern = spatial_ring_kernel<DT, PG, S2>;
    static std::once_flag once; // one per instantiation
    allow_lds_once(once, kern, 160 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(spatial_threads(PG)), lds_bytes, st, a);
}

int launch_spatial_ring(int dtype, const SpatialRingArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const bool s2 = a.stride == 2;
    const size_t lds_bytes = (size_t)(s2 ? 4 : 2) * a.npb * (1024 + (s2 ? 32 : 16)) + (size_t)a.depth * kSpatialWStage + 2048 + 1024;
    const long items = (long)a.tilesN * a.tilesY * a.tilesX * a.nfb;
    const unsigned grid = (unsigned)std::min<long>(items, 256);
    if (lds_bytes > 160 * 1024 || a.depth < 3 || a.depth > 6 || (long)a.N * a.H * a.W >= (1L << 24) /* 24-bit multiplies in the patch addresses */ || (a.pg != 4 && a.pg != 2) || a.NI * a.TH * a.TW > 64 * a.pg ||
        a.TH > 255 || a.TW > 255 || a.PH > 1023 || a.PW > 1023 || (a.stride != 1 && a.stride != 2) ||
        (s2 && (a.pg != 2 || a.KH != 3 || a.KW != 3 || a.pad != 1 || a.PH != a.TH + 1 || a.PW != a.TW + 1 || a.npb > 4 * 31))) {
        set_error("spatial_ring: tile plan does not fit the kernel");
        return NPAS_E_SHAPE;
    }
    if (dtype == NPAS_BF16) {
        if (s2) launch_spatial_inst<NPAS_BF16, 2, true>(a, grid, lds_bytes, st);
        else if (a.pg == 4) launch_spatial_inst<NPAS_BF16, 4>(a, grid, lds_bytes, st);
        else launch_spatial_inst<NPAS_BF16, 2>(a, grid, lds_bytes, st);
    } else if (dtype == NPAS_F16) {
        if (s2) launch_spatial_inst<NPAS_F16, 2, true>(a, grid, lds_bytes, st);
        else if (a.pg == 4) launch_spatial_inst<NPAS_F16, 4>(a, grid, lds_bytes, st);
        else launch_spatial_inst<NPAS_F16, 2>(a, grid, lds_bytes, st);
    } else {
        set_error("spatial_ring needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("spatial_ring launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
// spatial_resident: k x k layers at stride 1 with C a multiple of 64 and at most 64 filters, whose
// weight images (first filter half of every stage, 8 KB each) all fit in LDS next to two patch
// buffers: a 3 x 3 layer on 64 channels is 72 KB.  The workgroup fetches them once and then only
// streams patches: no weight traffic and no per-stage barrier, one barrier per (item, chunk).
//   waves 0-7   multiply: 32 pixels x 64 filters each (two waves per SIMD: one's operand reads
//               hide behind the other's MFMAs; four waves of 64 x 64, one per SIMD, with the next
//               step's operands read ahead by hand, read a third less from LDS and were slower:
//               54 against 42 us on 56 x 56 x 64 -> 64 at batch 128)
//   waves 8-15  fetch the next patch while the current one is multiplied (eight rather than four: 39.2 -> 38.5 us)
// Tile, patch layout, pixel table and epilogue are the spatial ring's.
constexpr int kResidentThreads = 16 * 64;
constexpr uint32_t kResidentWStage = 8192;

template <int DT>
__global__ __launch_bounds__(kResidentThreads) void spatial_resident_kernel(SpatialRingArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lbase = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint32_t nwg = gridDim.x;
    const uint32_t nitems = (uint32_t)(a.tilesN * a.tilesY * a.tilesX);
    const int T = a.KH * a.KW, nch = a.C >> 6, nst = nch * T;
    const uint32_t ppb = (uint32_t)a.npb * 1024u;                 // bytes of one patch buffer
    const uint32_t lw = 2u * ppb;                                 // the weights: nst stages of 8 KB
    const uint32_t lbias = lw + (uint32_t)nst * kResidentWStage;  // 64 floats (1 KB block)
    const uint32_t ltab = lbias + 1024u;                          // patch pixel -> (image, row, column), 4 B each
    const uint32_t lotab = ltab + (uint32_t)a.npb * 32u;          // tile pixel -> (image, row, column) inside the tile
    uint32_t c_item = xcd_remap(blockIdx.x, nwg);
    if (c_item >= nitems) return;
    SpatialItem it = spatial_item(a, c_item);
    const int phpw = a.PH * a.PW;

    for (int pp = tid; pp < a.npb * 8; pp += kResidentThreads) {
        const uint32_t img = fastdiv((uint32_t)pp, a.div_phpw), r = (uint32_t)pp - img * (uint32_t)phpw;
        const uint32_t py = fastdiv(r, a.div_pw), px = r - py * (uint32_t)a.PW;
        reinterpret_cast<uint32_t *>(lds + ltab)[pp] = (int)img < a.NI ? (img << 20 | py << 10 | px) : 0xffffffffu;
    }
    spatial_out_table(a, reinterpret_cast<uint32_t *>(lds + lotab), 256, tid, kResidentThreads);
    // weights: image i = stage * 8 + step * 4 + row tile, from [stage][step][8 tiles] in the packed format
    {
        const uint8_t *wb = reinterpret_cast<const uint8_t *>(a.wimg) + (uint32_t)lane * 16u;
        for (int i = wave; i < nst * 8; i += kResidentThreads / 64)
            lds_dma16(wb + (size_t)(i >> 3) * 16384u + (size_t)((i >> 2) & 1) * 8192u + (size_t)(i & 3) * 1024u, lbase + lw + (uint32_t)i * 1024u);
        if (wave == 0 && a.bias) { // lanes past the filters fetch a copy that nobody reads
            const int f = (lane & 15) * 4;
            lds_dma16(a.bias + (f < a.F ? f : 0), lbase + lbias);
        }
    }
    __syncthreads(); // the table

    if (wave >= 8) {
        // ---- patch fetch ------------------------------------------------------------------
        const int wl = wave - 8;
        const uint8_t *xb = reinterpret_cast<const uint8_t *>(a.x);
        const uint8_t *zb = reinterpret_cast<const uint8_t *>(a.zeros) + (uint32_t)(lane & 7) * 16u;
        const uint32_t pcv = (uint32_t)((lane & 7) ^ (lane >> 3)) * 16u;
        auto patch = [&](const SpatialItem &pi, int cc, uint32_t buf) __attribute__((always_inline)) {
            for (int blk = wl; blk < a.npb; blk += kResidentThreads / 64 - 8) {
                const uint32_t e = reinterpret_cast<const uint32_t *>(lds + ltab)[blk * 8 + (lane >> 3)];
                const int n = pi.n0 + (int)(e >> 20), iy = pi.ty0 - a.pad + (int)((e >> 10) & 1023u), ix = pi.tx0 - a.pad + (int)(e & 1023u);
                const bool inb = e != 0xffffffffu && n < a.N && (uint32_t)iy < (uint32_t)a.H && (uint32_t)ix < (uint32_t)a.W;
                const uint8_t *src = inb ? xb + ((uint32_t)((n * a.H + iy) * a.W + ix) * (uint32_t)a.C + (uint32_t)cc * 64u) * 2u + pcv : zb;
                lds_dma16(src, lbase + buf * ppb + (uint32_t)blk * 1024u);
            }
        };
        patch(it, 0, 0);
        uint32_t pbuf = 0;
        for (;;) {
            const bool more_items = c_item + nwg < nitems;
            SpatialItem nit = it;
            if (more_items) nit = spatial_item(a, c_item + nwg);
            for (int cc = 0; cc < nch; ++cc) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this chunk's patch (and, the first time, the weights) have landed
                __builtin_amdgcn_s_barrier();                    // ... and the other buffer has been multiplied
                if (cc + 1 < nch) patch(it, cc + 1, pbuf ^ 1u);
                else if (more_items) patch(nit, 0, pbuf ^ 1u);
                pbuf ^= 1u;
            }
            if (!more_items) break;
            c_item += nwg;
            it = nit;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---- multiply ------------------------------------------------------------------------
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wave's share of the weights
    const int wp = wave;
    const Clamp cl = clamp_of(a.act);
    const int thtw = a.TH * a.TW;
    uint32_t pb0[2]; // where this lane's operand rows (tile pixels 32 wp + 16 s + n16) sit in the patch
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t m = (uint32_t)(wp * 32 + s * 16 + n16);
        const uint32_t img = fastdiv(m, a.div_thtw), r = m - img * (uint32_t)thtw;
        const uint32_t ty = fastdiv(r, a.div_tw), tx = r - ty * (uint32_t)a.TW;
        pb0[s] = (int)m < a.NI * thtw ? img * (uint32_t)phpw + ty * (uint32_t)a.PW + tx : 0u;
    }
    uint32_t pbuf = 0;
    const uint32_t arow = (uint32_t)lane * 16u;

    for (;;) { // one item per iteration
        f32x4 acc[4][2];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int s = 0; s < 2; ++s) acc[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};
        const bool more_items = c_item + nwg < nitems;

        for (int cc = 0; cc < nch; ++cc) {
            __builtin_amdgcn_s_barrier(); // the chunk's patch is in LDS
            asm volatile("" ::: "memory");
            const uint8_t *pbp = lds + pbuf * ppb;
            const uint8_t *wsp = lds + lw + (uint32_t)(cc * T) * kResidentWStage + arow;
            uint32_t kh = 0, kw = 0;
            for (int tap = 0; tap < T; ++tap) {
                const uint32_t toff = kh * (uint32_t)a.PW + kw;
                if (++kw == (uint32_t)a.KW) { kw = 0; ++kh; }
#pragma unroll
                for (int step = 0; step < 2; ++step) {
                    uint4 A[4], B[2];
#pragma unroll
                    for (int j = 0; j < 4; ++j) A[j] = *reinterpret_cast<const uint4 *>(wsp + (uint32_t)(step * 4 + j) * 1024u);
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const uint32_t pp = pb0[s] + toff;
                        B[s] = *reinterpret_cast<const uint4 *>(pbp + pp * 128u + ((((uint32_t)(step * 4 + q)) ^ (pp & 7u)) << 4));
                    }
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[j][s] = mfma16<DT>(B[s], A[j], acc[j][s]);
                }
                wsp += kResidentWStage;
            }
            pbuf ^= 1u;
        }
        // ---- bias (from LDS), residual, activation, round, store: result register i of (j, s) is tile
        // pixel 32 wp + 16 s + 4q + i, filter 4 n16 + j
        {
            float4 b4 = float4{0.f, 0.f, 0.f, 0.f};
            if (a.bias) b4 = *reinterpret_cast<const float4 *>(lds + lbias + (uint32_t)(4 * n16) * 4u);
            spatial_epilogue<DT, 2>(a, it, lds + lotab + (uint32_t)(wp * 32 + 4 * q) * 4u, acc, b4, 4 * n16, cl);
        }
        if (!more_items) break;
        c_item += nwg;
        it = spatial_item(a, c_item);
    }
}

template <int DT> static void launch_resident_inst(const SpatialRingArgs &a, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    auto kern = spatial_resident_kernel<DT>;
    static std::once_flag once; // one per instantiation
    allow_lds_once(once, kern, 160 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kResidentThreads), lds_bytes, st, a);
}

size_t spatial_resident_lds_bytes(int npb, int nst) { return (size_t)2 * npb * 1024 + (size_t)nst * kResidentWStage + 1024 + (size_t)npb * 32 + 1024; }

int launch_spatial_resident(int dtype, const SpatialRingArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int nst = (a.C / 64) * a.KH * a.KW;
    const size_t lds_bytes = spatial_resident_lds_bytes(a.npb, nst);
    const long items = (long)a.tilesN * a.tilesY * a.tilesX;
    const unsigned grid = (unsigned)std::min<long>(items, 256);
    if (lds_bytes > 160 * 1024 || a.F > 64 || a.C % 64 != 0 || a.nfb != 1 || a.NI * a.TH * a.TW > 256 || a.npb > 4 * 60 ||
        a.TH > 255 || a.TW > 255 || a.PH > 1023 || a.PW > 1023) {
        set_error("spatial_resident: tile plan does not fit the kernel");
        return NPAS_E_SHAPE;
    }
    if (dtype == NPAS_BF16) launch_resident_inst<NPAS_BF16>(a, grid, lds_bytes, st);
    else if (dtype == NPAS_F16) launch_resident_inst<NPAS_F16>(a, grid, lds_bytes, st);
    else {
        set_error("spatial_resident needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("spatial_resident launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

} // namespace npas
