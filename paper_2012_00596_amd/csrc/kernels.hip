// gfx950 kernels of libnpas for one layer per launch (k x k layers on whole 64-channel chunks: spatial_kernels.hip; exact lists
// for sparse FC and small fp32 blocks: small_kernels.hip; fused pairs / blocks and the depthwise layer: block_kernels.hip).
//
// conv_gather_mfma: block-punched / block-based / pattern layers in bf16 or fp16.
//   The surviving (channel, kh, kw) positions of a 16-filter tile form the K
//   dimension of a dense sub-GEMM (paper section 3: the kept weights of a block
//   share their positions, so the remaining work is regular).  The activation
//   patch of an output tile is staged once in LDS ([pixel][channel chunk]); for
//   each 32 list entries a wave gathers the B operand (8 entries x its pixel per
//   lane) from LDS and issues one v_mfma_f32_16x16x32 per 16 output pixels with
//   the pre-swizzled weight image as the A operand.
// conv_valu_f32: fp32 layers, one thread per (output pixel, sub-group of <= 8
//   filters), weights broadcast from scalar loads, exact per-group skipping.
// maxpool3x3s2 / global_avgpool: glue layers of residual stacks.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "npas_internal.h"
#include "device_util.h"

namespace npas {

// Copies the input patch of one output tile, channels [cc*CC, cc*CC + CC), into LDS as
// [patch pixel][channel] with `pitch` bytes per pixel; out-of-image pixels become zeros.
// WIDE: 16-byte LDS writes (pitch is a multiple of 16), else two 8-byte writes.
template <bool WIDE>
__device__ __forceinline__ void stage_patch(const ConvMfmaArgs &a, uint8_t *lds, const uint16_t *x16, int n, int iy0,
                                            int ix0, int cc, int tid)
{
    const ConvGeom &g = a.g;
    const int c0 = cc * a.CC, ccount = min(a.CC, g.C - c0);
    if (g.vec) {
        const uint32_t nvv = (uint32_t)ccount >> 3;
        const uint32_t total = (uint32_t)(g.PH * g.PW) * nvv;
        const uint32_t dv = (nvv == (uint32_t)(a.CC >> 3)) ? g.div_vec : 0xffffffffu;
        for (uint32_t v = tid; v < total; v += 256) {
            uint32_t pix = dv == 0xffffffffu ? v / nvv : fastdiv(v, dv);
            uint32_t cv = v - pix * nvv;
            uint32_t py = fastdiv(pix, g.div_pw), px = pix - py * (uint32_t)g.PW;
            int iy = iy0 + (int)py * g.pstep, ix = ix0 + (int)px * g.pstep;
            uint4 val = uint4{0u, 0u, 0u, 0u};
            if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
                val = *reinterpret_cast<const uint4 *>(x16 + ((size_t)((n * g.H + iy) * g.W + ix) * g.C + c0 + cv * 8));
            if (WIDE) {
                *reinterpret_cast<uint4 *>(lds + pix * (uint32_t)g.pitch + cv * 16) = val;
            } else {
                uint2 *dst = reinterpret_cast<uint2 *>(lds + pix * (uint32_t)g.pitch + cv * 16);
                dst[0] = uint2{val.x, val.y};
                dst[1] = uint2{val.z, val.w};
            }
        }
    } else {
        const uint32_t total = (uint32_t)(g.PH * g.PW * ccount);
        for (uint32_t v = tid; v < total; v += 256) {
            uint32_t pix = v / (uint32_t)ccount, c = v - pix * (uint32_t)ccount;
            uint32_t py = fastdiv(pix, g.div_pw), px = pix - py * (uint32_t)g.PW;
            int iy = iy0 + (int)py * g.pstep, ix = ix0 + (int)px * g.pstep;
            uint16_t val = 0;
            if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W) val = x16[(size_t)((n * g.H + iy) * g.W + ix) * g.C + c0 + c];
            *reinterpret_cast<uint16_t *>(lds + pix * (uint32_t)g.pitch + c * 2) = val;
        }
    }
}

template <int DT, int S, bool HSW>
__device__ __forceinline__ void conv_gather_mfma_kernel_body(ConvMfmaArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const ConvGeom &g = a.g;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;

    const uint32_t logical = xcd_remap(blockIdx.x, gridDim.x);
    const uint32_t fsplit = logical % (uint32_t)g.nfsplit, ptile = logical / (uint32_t)g.nfsplit;
    const uint32_t tiles_img = (uint32_t)(g.tilesY * g.tilesX);
    const int n = (int)(ptile / tiles_img);
    const uint32_t trem = ptile % tiles_img;
    const int ty0 = (int)(trem / (uint32_t)g.tilesX) * g.TH, tx0 = (int)(trem % (uint32_t)g.tilesX) * g.TW;

    const uint32_t patch_bytes = ((uint32_t)(g.PH * g.PW * g.pitch) + 15u) & ~15u;
    uint32_t *koff = reinterpret_cast<uint32_t *>(lds + patch_bytes) + wave * g.koff_cap;

    // Which output pixel each of this lane's S MFMA columns is, where its patch
    // origin sits in LDS, and where its outputs go.
    const int npix_tile = g.TH * g.TW;
    const int ns = (npix_tile + 15) >> 4;
    uint32_t pixbase[S];
    int32_t outoff[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        uint32_t m = (uint32_t)(s * 16 + n16);
        uint32_t ty = fastdiv(m, g.div_tw), tx = m - ty * (uint32_t)g.TW;
        int oy = ty0 + (int)ty, ox = tx0 + (int)tx;
        bool valid = (int)m < npix_tile && oy < g.Ho && ox < g.Wo;
        pixbase[s] = valid ? ((ty * g.lstep) * g.PW + tx * g.lstep) * (uint32_t)g.pitch : 0u;
        outoff[s] = valid ? ((n * g.Ho + oy) * g.Wo + ox) * g.F : -1;
    }

    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    // input coordinate of patch pixel (0, 0)
    const int iy0 = (g.pstep > 1 ? ty0 * g.pstep : ty0 * g.stride) - g.pad;
    const int ix0 = (g.pstep > 1 ? tx0 * g.pstep : tx0 * g.stride) - g.pad;

    const int ft_begin = (int)fsplit * g.tiles_per_split;
    const int ft_end = min(ft_begin + g.tiles_per_split, a.ntiles);
    bool staged = false;

    for (int ftb = ft_begin; ftb < ft_end; ftb += 4) {
        const int ft = ftb + wave;
        const bool active = ft < ft_end;
        f32x4 acc[S];
#pragma unroll
        for (int s = 0; s < S; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int cc = 0; cc < a.nchunks; ++cc) {
            if (a.nchunks > 1 || !staged) {
                // ---- stage the activation patch of channel chunk cc -------------
                __syncthreads();
                stage_patch<false>(a, lds, x16, n, iy0, ix0, cc, tid);
                staged = true;
                __syncthreads();
            }
            if (!active) continue;

            const int e0 = a.tc_ptr[ft * a.nchunks + cc], e1 = a.tc_ptr[ft * a.nchunks + cc + 1];
            for (int eb = e0; eb < e1; eb += g.koff_cap) {
                const int nb = min(g.koff_cap, e1 - eb);
                // ---- list entries -> LDS byte offsets, once per wave -------------
                __builtin_amdgcn_wave_barrier();
                for (int i = lane; i < nb; i += 64) {
                    uint32_t ent = a.kent[eb + i];
                    uint32_t kh = ent >> 24, kw = (ent >> 16) & 255u, c = ent & 0xffffu;
                    koff[i] = (kh * (uint32_t)g.PW + kw) * (uint32_t)g.pitch + c * 2u;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

                const uint4 *wf = reinterpret_cast<const uint4 *>(a.wfrag) + (size_t)(eb >> 5) * 64 + lane;
                for (int j = 0; j < nb; j += 32, wf += 64) {
                    const uint4 wa = *wf;
                    const uint4 k0 = *reinterpret_cast<const uint4 *>(koff + j + 8 * q);
                    const uint4 k1 = *reinterpret_cast<const uint4 *>(koff + j + 8 * q + 4);
#pragma unroll
                    for (int s = 0; s < S; ++s) {
                        {
                            const uint8_t *pb = lds + pixbase[s];
                            uint4 b;
                            b.x = (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k0.x) |
                                  (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k0.y) << 16;
                            b.y = (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k0.z) |
                                  (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k0.w) << 16;
                            b.z = (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k1.x) |
                                  (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k1.y) << 16;
                            b.w = (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k1.z) |
                                  (uint32_t)*reinterpret_cast<const uint16_t *>(pb + k1.w) << 16;
                            acc[s] = mfma16<DT>(wa, b, acc[s]);
                        }
                    }
                }
            }
        }

        // ---- epilogue: bias, residual, activation, round, store -----------------
        if (active) {
            const int f0 = ft * 16 + 4 * q;
            if (f0 < g.F) {
                float bv[4] = {0.f, 0.f, 0.f, 0.f};
                if (a.bias) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (f0 + i < g.F) bv[i] = a.bias[f0 + i];
                }
                uint16_t *y16 = reinterpret_cast<uint16_t *>(a.y);
                const uint16_t *r16 = reinterpret_cast<const uint16_t *>(a.residual);
                const bool vec4 = (g.F & 3) == 0;
                const Clamp cl = clamp_of(g.act);
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    if (s < ns && outoff[s] >= 0) {
                        const size_t o = (size_t)outoff[s] + f0;
                        float v[4] = {acc[s][0] + bv[0], acc[s][1] + bv[1], acc[s][2] + bv[2], acc[s][3] + bv[3]};
                        if (vec4) {
                            if (r16) {
                                uint2 r = *reinterpret_cast<const uint2 *>(r16 + o);
                                v[0] += from_storage<DT>((uint16_t)(r.x & 0xffffu));
                                v[1] += from_storage<DT>((uint16_t)(r.x >> 16));
                                v[2] += from_storage<DT>((uint16_t)(r.y & 0xffffu));
                                v[3] += from_storage<DT>((uint16_t)(r.y >> 16));
                            }
                            uint2 out;
                            out.x = pack2<DT>(clampf<HSW>(v[0], cl), clampf<HSW>(v[1], cl));
                            out.y = pack2<DT>(clampf<HSW>(v[2], cl), clampf<HSW>(v[3], cl));
                            *reinterpret_cast<uint2 *>(y16 + o) = out;
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (f0 + i < g.F) {
                                    float t = v[i];
                                    if (r16) t += from_storage<DT>(r16[o + i]);
                                    y16[o + i] = (uint16_t)(pack2<DT>(clampf<HSW>(t, cl), 0.f) & 0xffffu);
                                }
                        }
                    }
                }
            }
        }
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT, int S>
__global__ __launch_bounds__(256) void conv_gather_mfma_kernel(ConvMfmaArgs a)
{
    if (a.g.act == NPAS_ACT_HARDSWISH) conv_gather_mfma_kernel_body<DT, S, true>(a);
    else conv_gather_mfma_kernel_body<DT, S, false>(a);
}

// ------------------------------------------------------------------------------
// conv_slab_mfma: the same layers, gathered at 8-channel granularity.  A list entry is
// an 8-channel slab at one tap; four slabs make one 32-deep MFMA step, and the B operand
// of a step is one 16-byte LDS read per lane (lane quarter q reads slab 4*step+q of its
// pixel).  The 4 waves of a workgroup form a WGF x (4/WGF) grid over a tile of
// 16*WT*WGF filters x 16*WB*(4/WGF) output pixels; a wave reuses each gathered
// activation fragment for its WT filter tiles and each weight fragment for its WB
// pixel blocks.
//
// Workgroups are persistent: each walks work items (pixel tile, filter block) and,
// inside an item, the layer's channel chunks.  The activation patch of the NEXT stage
// is fetched from global memory into registers while the current one is multiplied out
// of LDS, then written to the other LDS buffer: one barrier per stage, and global loads
// in flight all the time (what an HBM-bound layer needs).

template <int WT, int WB, int WGF> struct SlabShape {
    static constexpr int WGP = 4 / WGF;         // waves along pixels
    static constexpr int TPB = WB * WGP;        // pixel blocks per workgroup tile
    static constexpr int TFT = WT * WGF;        // filter tiles per workgroup tile
};

struct SlabItem {
    int n, ty0, tx0, fb;
};

__device__ __forceinline__ SlabItem slab_item(const ConvGeom &g, uint32_t item)
{
    SlabItem it;
    const uint32_t nfb = (uint32_t)g.nfsplit;
    const uint32_t ptile = item / nfb;
    it.fb = (int)(item - ptile * nfb);
    const uint32_t tiles_img = (uint32_t)(g.tilesY * g.tilesX);
    it.n = (int)(ptile / tiles_img);
    const uint32_t trem = ptile - (uint32_t)it.n * tiles_img;
    const uint32_t tyi = trem / (uint32_t)g.tilesX;
    it.ty0 = (int)tyi * g.TH;
    it.tx0 = (int)(trem - tyi * (uint32_t)g.tilesX) * g.TW;
    return it;
}

// What one thread moves of every staged patch chunk: NPF 16-byte vectors.
// Computed once per kernel (the patch geometry never changes), so that a stage costs an
// add per vector instead of divisions: grel = element offset of the vector relative to
// the patch origin pixel and the chunk's first channel, loff = byte offset in the LDS
// buffer.  Vectors past the end of the patch repeat the last one (same load, same
// store: harmless).
template <int NPF> struct SlabDesc { // NPF = 16-byte vectors of a patch chunk one thread moves
    int32_t grel[NPF];
    uint32_t loff[NPF];
};

template <int NPF> __device__ __forceinline__ void slab_desc_init(const ConvMfmaArgs &a, int tid, SlabDesc<NPF> &d)
{
    const ConvGeom &g = a.g;
    const uint32_t nvv = (uint32_t)a.CC >> 3;
    const uint32_t total = (uint32_t)(g.PH * g.PW) * nvv;
#pragma unroll
    for (int i = 0; i < NPF; ++i) {
        const uint32_t v = min((uint32_t)tid + 256u * i, total - 1u);
        const uint32_t pix = fastdiv(v, g.div_vec), cv = v - pix * nvv;
        const uint32_t py = fastdiv(pix, g.div_pw), px = pix - py * (uint32_t)g.PW;
        d.grel[i] = (int32_t)(((py * g.pstep) * g.W + px * g.pstep) * g.C + cv * 8);
        d.loff[i] = pix * (uint32_t)g.pitch + cv * 16;
    }
}

// Issues the global loads of one patch chunk.  interior: the whole patch lies inside the
// image and the chunk has all CC channels, so no vector needs a test.
template <int NPF>
__device__ __forceinline__ void slab_patch_load(const ConvMfmaArgs &a, const uint8_t *xb, const SlabItem &it, int cc,
                                                const SlabDesc<NPF> &d, uint4 (&pf)[NPF])
{
    const ConvGeom &g = a.g;
    const int c0 = cc * a.CC, ccount = min(a.CC, g.C - c0);
    const int iy0 = (g.pstep > 1 ? it.ty0 * g.pstep : it.ty0 * g.stride) - g.pad;
    const int ix0 = (g.pstep > 1 ? it.tx0 * g.pstep : it.tx0 * g.stride) - g.pad;
    const int32_t base = ((it.n * g.H + iy0) * g.W + ix0) * g.C + c0; // may point before the image: only used where valid
    const bool interior = ccount == a.CC && iy0 >= 0 && ix0 >= 0 && iy0 + (g.PH - 1) * g.pstep < g.H &&
                          ix0 + (g.PW - 1) * g.pstep < g.W;
    if (interior) {
#pragma unroll
        for (int i = 0; i < NPF; ++i)
            pf[i] = *reinterpret_cast<const uint4 *>(xb + (uint32_t)(base + d.grel[i]) * 2u);
    } else {
#pragma unroll
        for (int i = 0; i < NPF; ++i) {
            // border items only: recover the patch pixel from the LDS offset
            const uint32_t pix = fastdiv(d.loff[i], g.div_pitch), cb = d.loff[i] - pix * (uint32_t)g.pitch;
            const uint32_t py = fastdiv(pix, g.div_pw), px = pix - py * (uint32_t)g.PW;
            const int iy = iy0 + (int)py * g.pstep, ix = ix0 + (int)px * g.pstep;
            const bool ok = (uint32_t)iy < (uint32_t)g.H && (uint32_t)ix < (uint32_t)g.W && (int)(cb >> 1) < ccount;
            pf[i] = uint4{0u, 0u, 0u, 0u};
            if (ok) pf[i] = *reinterpret_cast<const uint4 *>(xb + (uint32_t)(base + d.grel[i]) * 2u);
        }
    }
}

template <int NPF>
__device__ __forceinline__ void slab_patch_store(uint8_t *buf, const SlabDesc<NPF> &d, const uint4 (&pf)[NPF])
{
#pragma unroll
    for (int i = 0; i < NPF; ++i) *reinterpret_cast<uint4 *>(buf + d.loff[i]) = pf[i];
}

template <int DT, int WT, int WB, int WGF, int NPF, int OCC, bool HSW>
__device__ __forceinline__ void conv_slab_mfma_kernel_body(ConvMfmaArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const ConvGeom &g = a.g;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const int wf = wave % WGF, wp = wave / WGF;
    const uint32_t nwg = gridDim.x;
    const uint32_t nitems = (uint32_t)(g.N * g.tilesY * g.tilesX * g.nfsplit);
    const uint32_t buf_bytes = ((uint32_t)(g.PH * g.PW * g.pitch) + 15u) & ~15u;
    const uint8_t *xb = reinterpret_cast<const uint8_t *>(a.x);
    uint8_t *yb = reinterpret_cast<uint8_t *>(a.y);
    const uint8_t *rb = reinterpret_cast<const uint8_t *>(a.residual);
    const int npix_tile = g.TH * g.TW;
    const Clamp cl = clamp_of(g.act); // F is a multiple of 4 on this path: a lane's 4 outputs are one 8-byte store

    uint32_t item = xcd_remap(blockIdx.x, nwg);
    if (item >= nitems) return;
    SlabDesc<NPF> desc;
    slab_desc_init(a, tid, desc);
    SlabItem it = slab_item(g, item);
    uint4 pf[NPF];
    slab_patch_load(a, xb, it, 0, desc, pf);
    slab_patch_store(lds, desc, pf);
    __syncthreads();
    uint32_t bufoff = 0;

    for (;;) { // one work item per iteration
        const int st = it.fb * WGF + wf; // this wave's super-tile
        const bool active = st < a.ntiles;
        const int fl = (st * WT) * 16 + 4 * q; // this lane's first filter in row tile 0
        // Where this lane's pixel columns sit in the patch and in the output; accumulators
        // start from the bias.
        uint32_t pixbase[WB], obyte[WB];
        f32x4 acc[WT][WB];
#pragma unroll
        for (int s = 0; s < WB; ++s) {
            const uint32_t m = (uint32_t)((wp * WB + s) * 16 + n16);
            const uint32_t ty = fastdiv(m, g.div_tw), tx = m - ty * (uint32_t)g.TW;
            const int oy = it.ty0 + (int)ty, ox = it.tx0 + (int)tx;
            const bool valid = (int)m < npix_tile && oy < g.Ho && ox < g.Wo;
            pixbase[s] = valid ? ((ty * g.lstep) * g.PW + tx * g.lstep) * (uint32_t)g.pitch : 0u;
            obyte[s] = valid ? (uint32_t)(((it.n * g.Ho + oy) * g.Wo + ox) * g.F + fl) * 2u : 0xffffffffu;
        }
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            f32x4 b0 = f32x4{0.f, 0.f, 0.f, 0.f};
            if (a.bias && active) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (fl + 16 * j + i < g.F) b0[i] = a.bias[fl + 16 * j + i];
            }
#pragma unroll
            for (int s = 0; s < WB; ++s) acc[j][s] = b0;
        }

        uint32_t nitem = item + nwg;
        bool more = nitem < nitems; // another item after this one?
        SlabItem nit = it;
        for (int cc = 0; cc < a.nchunks; ++cc) {
            // ---- next stage's patch: global loads go out now, land while we multiply ----
            const bool last = cc == a.nchunks - 1;
            const bool has_next = !last || more;
            if (has_next) {
                if (last) nit = slab_item(g, nitem);
                slab_patch_load(a, xb, last ? nit : it, last ? 0 : cc + 1, desc, pf);
            }
            // ---- residual: fetched ahead of the item's last chunk, added after it -----------
            uint2 res[WT][WB];
            if (last && rb && active) {
#pragma unroll
                for (int j = 0; j < WT; ++j)
#pragma unroll
                    for (int s = 0; s < WB; ++s) {
                        res[j][s] = uint2{0u, 0u};
                        if (obyte[s] != 0xffffffffu && fl + 16 * j < g.F)
                            res[j][s] = *reinterpret_cast<const uint2 *>(rb + obyte[s] + 32u * j);
                    }
            }
            // ---- multiply the current stage out of LDS ---------------------------------
            if (active) {
                const int e0 = a.tc_ptr[st * a.nchunks + cc], e1 = a.tc_ptr[st * a.nchunks + cc + 1];
                if (e0 < e1) {
                    const uint8_t *wfb = reinterpret_cast<const uint8_t *>(a.wfrag);
                    const uint8_t *keb = reinterpret_cast<const uint8_t *>(a.kent);
                    uint32_t wby = (uint32_t)(e0 >> 2) * (WT * 1024u) + (uint32_t)lane * 16u, kby = (uint32_t)(e0 + q) * 4u;
                    uint32_t ent = *reinterpret_cast<const uint32_t *>(keb + kby);
                    uint4 wa[WT];
#pragma unroll
                    for (int j = 0; j < WT; ++j) wa[j] = *reinterpret_cast<const uint4 *>(wfb + wby + j * 1024u);
                    for (int e = e0; e < e1; e += 4) {
                        const uint32_t koff = bufoff + ((ent >> 24) * (uint32_t)g.PW + ((ent >> 16) & 255u)) * (uint32_t)g.pitch +
                                              (ent & 0xffffu) * 2u;
                        uint4 wc[WT];
#pragma unroll
                        for (int j = 0; j < WT; ++j) wc[j] = wa[j];
                        if (e + 4 < e1) { // fetch the next step's entry and weight fragments during this step
                            kby += 16u;
                            wby += WT * 1024u;
                            ent = *reinterpret_cast<const uint32_t *>(keb + kby);
#pragma unroll
                            for (int j = 0; j < WT; ++j) wa[j] = *reinterpret_cast<const uint4 *>(wfb + wby + j * 1024u);
                        }
                        uint4 b[WB];
#pragma unroll
                        for (int s = 0; s < WB; ++s) b[s] = *reinterpret_cast<const uint4 *>(lds + pixbase[s] + koff);
#pragma unroll
                        for (int s = 0; s < WB; ++s)
#pragma unroll
                            for (int j = 0; j < WT; ++j) acc[j][s] = mfma16<DT>(wc[j], b[s], acc[j][s]);
                    }
                }
            }
            if (has_next) slab_patch_store(lds + (bufoff ^ buf_bytes), desc, pf);
            if (last && active) {
                // ---- clamp (activation), round, store --------------------------------------
#pragma unroll
                for (int j = 0; j < WT; ++j) {
                    const int f0 = fl + 16 * j;
                    if (f0 >= g.F) continue;
#pragma unroll
                    for (int s = 0; s < WB; ++s) {
                        if (obyte[s] == 0xffffffffu) continue;
                        if (rb) {
                            acc[j][s][0] += from_storage<DT>((uint16_t)(res[j][s].x & 0xffffu));
                            acc[j][s][1] += from_storage<DT>((uint16_t)(res[j][s].x >> 16));
                            acc[j][s][2] += from_storage<DT>((uint16_t)(res[j][s].y & 0xffffu));
                            acc[j][s][3] += from_storage<DT>((uint16_t)(res[j][s].y >> 16));
                        }
                        uint2 out;
                        out.x = pack2<DT>(clampf<HSW>(acc[j][s][0], cl), clampf<HSW>(acc[j][s][1], cl));
                        out.y = pack2<DT>(clampf<HSW>(acc[j][s][2], cl), clampf<HSW>(acc[j][s][3], cl));
                        *reinterpret_cast<uint2 *>(yb + obyte[s] + 32u * j) = out;
                    }
                }
            }
            __syncthreads();
            bufoff ^= buf_bytes;
        }
        if (!more) break;
        item = nitem;
        it = nit;
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT, int WT, int WB, int WGF, int NPF, int OCC>
__global__ __launch_bounds__(256, OCC) void conv_slab_mfma_kernel(ConvMfmaArgs a)
{
    if (a.g.act == NPAS_ACT_HARDSWISH) conv_slab_mfma_kernel_body<DT, WT, WB, WGF, NPF, OCC, true>(a);
    else conv_slab_mfma_kernel_body<DT, WT, WB, WGF, NPF, OCC, false>(a);
}

template <int DT, int WT, int WB, int WGF, int NPF, int OCC>
static int launch_slab_inst(const ConvMfmaArgs &a, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    auto kern = conv_slab_mfma_kernel<DT, WT, WB, WGF, NPF, OCC>;
    static std::once_flag once; // one per instantiation
    allow_lds_once(once, kern, 96 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds_bytes, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_slab_mfma launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// Workgroup shapes (filter tiles per wave, pixel blocks per wave, waves along filters):
//   0: 4 x 4 x 2 -> 128 filters x 128 pixels     2: 2 x 2 x 1 -> 32 filters x 128 pixels
//   1: 4 x 2 x 1 ->  64 filters x 128 pixels     3: 4 x 2 x 2 -> 128 filters x  64 pixels
// Each with 4 or 8 staged vectors per thread (patch chunk of up to 1024 / 2048 vectors).
template <int DT> static int launch_slab_dt(const ConvMfmaArgs &a, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    const bool small = a.g.PH * a.g.PW * (a.CC / 8) <= 1024;
    switch (a.g.shape) {
    case 0: return small ? launch_slab_inst<DT, 4, 4, 2, 4, 2>(a, grid, lds_bytes, st) : launch_slab_inst<DT, 4, 4, 2, 8, 2>(a, grid, lds_bytes, st);
    case 1: return small ? launch_slab_inst<DT, 4, 2, 1, 4, 3>(a, grid, lds_bytes, st) : launch_slab_inst<DT, 4, 2, 1, 8, 2>(a, grid, lds_bytes, st);
    case 2: return small ? launch_slab_inst<DT, 2, 2, 1, 4, 4>(a, grid, lds_bytes, st) : launch_slab_inst<DT, 2, 2, 1, 8, 3>(a, grid, lds_bytes, st);
    case 3: return small ? launch_slab_inst<DT, 4, 2, 2, 4, 3>(a, grid, lds_bytes, st) : launch_slab_inst<DT, 4, 2, 2, 8, 2>(a, grid, lds_bytes, st);
    }
    set_error("conv_slab_mfma: unknown workgroup shape %d", a.g.shape);
    return NPAS_E_SHAPE;
}

// ------------------------------------------------------------------------------
// pointwise_ring: 1x1 layers (and FC) with C a multiple of 64, streamed through a ring of
// LDS stages that are filled by direct global->LDS loads (global_load_lds_dwordx4): no
// registers hold data in flight, so whole stages are always on their way while one is
// multiplied — what an HBM-bound layer with little work per byte needs.
//
// Tile (PW * 64) pixels x (FW * 64) filters.  Stage = 64 channels: 128 B per pixel of
// activations + FW * 8 weight images of 1 KB.  A load writes 64 lanes x 16 B lane-linearly
// into one 1 KB LDS block.  Activations are stored unpadded with an XOR swizzle: 16-byte
// vector cv of pixel p sits at p*128 + (cv ^ (p & 7))*16, so that the MFMA operand reads
// (16 consecutive pixels, same cv) spread over the banks.
//
// Waves 0 .. PW*FW-1 multiply (PW pixel groups x FW filter groups, 64 x 64 outputs each), the
// next WW fetch the weight images, the last XW the activations.  The loads are inline assembly
// (the compiler would otherwise drain the whole ring before every LDS read) and a fetching
// wave tracks their completion by hand: a wave's vector-memory operations return in order, so
// "at most D-2 stages' worth outstanding" means the stage about to be multiplied has landed.
// The multiplying waves issue no such loads; their residual / bias loads and their stores are
// ordinary code the compiler waits for exactly.  One s_barrier per stage, executed by all.
//
// Three configurations: 256 x 128 tiles with a 3-stage ring (throughput: most bytes in flight
// per CU, most reuse of the weights); 64 x 64 tiles with an 8-stage ring for launches that
// would leave most CUs without a tile (small batches): more, smaller items, and a whole
// layer's channel loop in flight at once instead of one load latency per stage (its tile is
// multiplied by four waves of 16 pixels x 64 filters, one per SIMD: such a launch is a chain of
// stage latencies, and four short chains of 8 MFMAs beat one of 32); 128 x 128
// tiles with a 4-stage ring in between, when the 256 x 128 items divide badly over the CUs.
// S: 16-pixel blocks of a multiplying wave (4: 64 pixels x 64 filters; fewer: more, narrower waves per tile)
template <int PW_, int FW_, int XW_, int WW_, int D_, int S_ = 4> struct PointwiseCfg {
    static constexpr int PW = PW_, FW = FW_, XW = XW_, WW = WW_, D = D_, S = S_;
    static constexpr int kComputeWaves = PW * FW * (4 / S);
    static constexpr int kThreads = (kComputeWaves + XW + WW) * 64;
    static constexpr uint32_t kXBytes = PW * 8192, kWBytes = FW * 8192, kStageBytes = kXBytes + kWBytes;
    static constexpr int kXBlocks = PW * 8, kWImages = FW * 8;             // 1 KB loads per stage
    static constexpr int kXLoads = (kXBlocks + XW - 1) / XW, kWLoads = (kWImages + WW - 1) / WW; // per fetch wave, at most
    static constexpr size_t kLdsBytes = (size_t)D * kStageBytes + 2048;    // + two bias buffers
    static_assert(D >= 3 && kXLoads * (D - 1) <= 63 && kWLoads * (D - 1) <= 63, "a wave can have 63 loads in flight");
};
using PointwiseBig = PointwiseCfg<4, 2, 3, 1, 3>;
using PointwiseSmall = PointwiseCfg<1, 1, 4, 4, 8, 1>;
using PointwiseMedium = PointwiseCfg<2, 2, 2, 1, 4, 2>; // 128 x 128 tiles, 4-stage ring: half-size items for layers whose 256 x 128 items divide badly over the CUs

struct PointwiseItem {
    uint32_t ptile, fb; // pixel tile, filter block (in units of the configuration's tile)
};

__device__ __forceinline__ PointwiseItem pointwise_item(uint32_t nfb, uint32_t item)
{
    PointwiseItem it;
    it.ptile = item / nfb;
    it.fb = item - it.ptile * nfb;
    return it;
}

// Epilogue of a multiplying wave of the pointwise ring: bias, residual, activation, round, store.  Result register i
// of acc[j][s] is the pixel 16 s + i rows after the lane's first one (row pitch `pitch` bytes, first row at yb0),
// filter j of the lane's 4.  The activation kind, the residual and "every row of the wave is inside the map" are
// wave-uniform and compiled in: with a branch per value and a mask per store this epilogue was longer than the
// main loop of a 64-channel layer.
template <int DT, int S, bool HS, bool RES, bool FULL>
__device__ __forceinline__ void pointwise_store_tile(uint8_t *yb0, uint32_t pitch, uint32_t rows_left, const f32x4 (&acc)[4][S],
                                                     const uint2 (&res)[S][4], float4 bv, Clamp cl)
{
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (!FULL && (uint32_t)(16 * s + i) >= rows_left) continue;
            float v[4] = {acc[0][s][i] + bv.x, acc[1][s][i] + bv.y, acc[2][s][i] + bv.z, acc[3][s][i] + bv.w};
            if (RES) {
                v[0] += from_storage<DT>((uint16_t)(res[s][i].x & 0xffffu));
                v[1] += from_storage<DT>((uint16_t)(res[s][i].x >> 16));
                v[2] += from_storage<DT>((uint16_t)(res[s][i].y & 0xffffu));
                v[3] += from_storage<DT>((uint16_t)(res[s][i].y >> 16));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = HS ? v[j] * __builtin_amdgcn_fmed3f(v[j] + 3.0f, 0.0f, 6.0f) * (1.0f / 6.0f) : __builtin_amdgcn_fmed3f(v[j], cl.lo, cl.hi);
            uint2 out;
            out.x = pack2<DT>(v[0], v[1]);
            out.y = pack2<DT>(v[2], v[3]);
            store_stream8(yb0 + (uint32_t)(16 * s + i) * pitch, out);
        }
}
template <int DT, int S, bool HS, bool RES>
__device__ __forceinline__ void pointwise_store_rows(uint8_t *yb0, uint32_t pitch, uint32_t rows_left, const f32x4 (&acc)[4][S],
                                                     const uint2 (&res)[S][4], float4 bv, Clamp cl)
{
    if (__all(rows_left >= (uint32_t)(16 * S))) pointwise_store_tile<DT, S, HS, RES, true>(yb0, pitch, rows_left, acc, res, bv, cl);
    else pointwise_store_tile<DT, S, HS, RES, false>(yb0, pitch, rows_left, acc, res, bv, cl);
}
template <int DT, int S>
__device__ __forceinline__ void pointwise_epilogue(uint8_t *yb0, uint32_t pitch, uint32_t rows_left, bool has_res, const f32x4 (&acc)[4][S],
                                                   const uint2 (&res)[S][4], float4 bv, Clamp cl)
{
    if (cl.hs) {
        if (has_res) pointwise_store_rows<DT, S, true, true>(yb0, pitch, rows_left, acc, res, bv, cl);
        else pointwise_store_rows<DT, S, true, false>(yb0, pitch, rows_left, acc, res, bv, cl);
    } else {
        if (has_res) pointwise_store_rows<DT, S, false, true>(yb0, pitch, rows_left, acc, res, bv, cl);
        else pointwise_store_rows<DT, S, false, false>(yb0, pitch, rows_left, acc, res, bv, cl);
    }
}

template <int DT, typename Cfg>
__global__ __launch_bounds__(Cfg::kThreads) void pointwise_ring_kernel(RingArgs a)
{
    constexpr int PW = Cfg::PW, FW = Cfg::FW, XW = Cfg::XW, WW = Cfg::WW, D = Cfg::D, NC = Cfg::kComputeWaves, S = Cfg::S;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lbase = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint32_t nwg = gridDim.x, nitems = (uint32_t)(a.nptiles * a.nfb);
    const int nst = a.C >> 6; // stages (64-channel chunks) per item
    const uint32_t nfb = (uint32_t)a.nfb;
    const uint32_t lbias = (uint32_t)D * Cfg::kStageBytes; // two 1 KB bias buffers (item parity)
    uint32_t c_item = xcd_remap(blockIdx.x, nwg);
    if (c_item >= nitems) return;

    if (wave >= NC + WW) {
        // ---- activation fetch: blocks wl, wl + XW, wl + 2 XW, ... (8 pixels each) of every stage ----
        const int wl = wave - NC - WW;
        const int nblocks = (a.P + 7) >> 3;                 // 8-pixel blocks of a tile that hold pixels of it
        const int nld = max(0, (nblocks - wl + XW - 1) / XW); // this wave's loads per stage
        const uint8_t *xb = reinterpret_cast<const uint8_t *>(a.x);
        const uint32_t pcv = (uint32_t)((lane & 7) ^ (lane >> 3)) * 16u; // which 16-byte vector of its pixel this lane fetches
        auto in_byte = [&](uint32_t m) __attribute__((always_inline)) -> uint32_t { // byte offset in x of output pixel m's input pixel
            m = min(m, (uint32_t)a.M - 1u);
            if (a.flat) return m * (uint32_t)a.C * 2u;
            const uint32_t n = fastdiv(m, a.div_howo), r = m - n * (uint32_t)(a.Ho * a.Wo);
            const uint32_t oy = fastdiv(r, a.div_wo), ox = r - oy * (uint32_t)a.Wo;
            return ((n * a.H + oy * a.stride) * a.W + ox * a.stride) * (uint32_t)a.C * 2u;
        };
        uint32_t p_item = c_item, p_slot = 0, ppix[Cfg::kXLoads];
        int p_t = 0;
        bool p_done = false;
        auto producer_item = [&]() __attribute__((always_inline)) {
            const PointwiseItem pi = pointwise_item(nfb, p_item);
            p_t = 0;
#pragma unroll
            for (int i = 0; i < Cfg::kXLoads; ++i) ppix[i] = in_byte(pi.ptile * (uint32_t)a.P + (uint32_t)((wl + XW * i) * 8 + (lane >> 3))) + pcv;
        };
        producer_item();
        auto produce = [&]() __attribute__((always_inline)) { // always issues its nld loads; past the end it repeats the last stage
            const uint32_t dst = lbase + p_slot * Cfg::kStageBytes + (uint32_t)wl * 1024u;
#pragma unroll
            for (int i = 0; i < Cfg::kXLoads; ++i)
                if (i < nld) lds_dma16(xb + ppix[i] + (uint32_t)p_t * 128u, dst + (uint32_t)(XW * i) * 1024u);
            if (++p_slot == (uint32_t)D) p_slot = 0;
            if (!p_done) {
                if (p_t + 1 < nst) ++p_t;
                else if (p_item + nwg < nitems) {
                    p_item += nwg;
                    producer_item();
                } else p_done = true;
            }
        };
        for (int i = 0; i + 1 < D; ++i) produce();
        const uint32_t allow = (uint32_t)(nld * (D - 2)); // the D-2 stages issued after the awaited one may stay in flight
        for (;;) {
            for (int t = 0; t < nst; ++t) {
                wait_vmcnt(allow);
                __builtin_amdgcn_s_barrier();
                produce(); // D-1 stages ahead, into the slot the barrier freed
            }
            if (c_item + nwg >= nitems) break;
            c_item += nwg;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    if (wave >= NC) {
        // ---- weight fetch: images wl, wl + WW, ... of every stage, and each item's bias --------------
        // A stage's images in the packed format are [step 0..1][filter half 0..1][row tile 0..3]; a
        // 64-filter tile (FW == 1) takes the four row tiles of its half in each step.
        const int wl = wave - NC;
        const int nld = (Cfg::kWImages - wl + WW - 1) / WW;
        const uint8_t *wb = reinterpret_cast<const uint8_t *>(a.wimg) + (uint32_t)lane * 16u;
        uint32_t p_item = c_item, p_slot = 0;
        PointwiseItem pi = pointwise_item(nfb, p_item);
        int p_t = 0;
        bool p_done = false;
        auto produce = [&]() __attribute__((always_inline)) { // always issues its loads; past the end it repeats the last stage
            const uint32_t fb128 = FW == 2 ? pi.fb : pi.fb >> 1, half = FW == 2 ? 0u : pi.fb & 1u;
            const uint8_t *wsrc = wb + (size_t)(fb128 * (uint32_t)nst + (uint32_t)p_t) * 16384u;
            const uint32_t dst = lbase + p_slot * Cfg::kStageBytes + Cfg::kXBytes;
#pragma unroll
            for (int i = 0; i < Cfg::kWLoads; ++i) {
                const int img = wl + WW * i; // local image: step * (FW * 4) + (filter group) * 4 + row tile
                if (i < nld) {
                    const uint32_t src_img = FW == 2 ? (uint32_t)img : (uint32_t)((img >> 2) * 8 + (img & 3)) + half * 4u;
                    lds_dma16(wsrc + src_img * 1024u, dst + (uint32_t)img * 1024u);
                }
            }
            if (++p_slot == (uint32_t)D) p_slot = 0;
            if (!p_done) {
                if (p_t + 1 < nst) ++p_t;
                else if (p_item + nwg < nitems) {
                    p_item += nwg;
                    pi = pointwise_item(nfb, p_item);
                    p_t = 0;
                } else p_done = true;
            }
        };
        // bias of an item's filters (lanes past the tile fetch a copy that nobody reads)
        auto bias_block = [&](uint32_t fb, uint32_t buf) __attribute__((always_inline)) {
            if (!a.bias || wl != 0) return;
            const int f = (int)fb * (FW * 64) + (lane & (FW * 16 - 1)) * 4;
            lds_dma16(a.bias + (f < a.F ? f : 0), lbase + lbias + buf * 1024u);
        };
        uint32_t bbuf = 0;
        bias_block(pi.fb, 0);
        for (int i = 0; i + 1 < D; ++i) produce();
        // a bias load in between only makes the wait stricter (one more completion than needed)
        const uint32_t allow = (uint32_t)(nld * (D - 2));
        for (;;) {
            const bool more = c_item + nwg < nitems;
            for (int t = 0; t < nst; ++t) {
                wait_vmcnt(allow);
                __builtin_amdgcn_s_barrier();
                // the other bias buffer was last read in the epilogue before this item's first barrier
                if (t == 0 && more) bias_block(pointwise_item(nfb, c_item + nwg).fb, bbuf ^ 1u);
                produce();
            }
            if (!more) break;
            c_item += nwg;
            bbuf ^= 1u;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---- multiply ------------------------------------------------------------------------
    const int wp = wave / FW, wf = wave % FW;
    uint8_t *yb = reinterpret_cast<uint8_t *>(a.y);
    const uint8_t *rb = reinterpret_cast<const uint8_t *>(a.residual);
    const Clamp cl = clamp_of(a.act);
    const uint32_t brow = (uint32_t)((wp * (16 * S) + n16) * 128), arow = (uint32_t)(wf * 4) * 1024u + (uint32_t)lane * 16u;
    uint32_t c_slot = 0, bbuf = 0;
    for (;;) { // one item per iteration
        const PointwiseItem it = pointwise_item(nfb, c_item);
        // The activations are the MFMA's row operand and the weight images its column operand, and
        // row r of weight tile j is filter 4r + j of the wave's 64: result register i of (j, s)
        // is pixel 16s + 4q + i, filter 4 n16 + j.  A lane therefore owns 4 consecutive filters
        // of a pixel, and the 16 lanes of a quarter wave one whole 128-byte run of its row.
        const int fcol = (int)it.fb * (FW * 64) + wf * 64 + 4 * n16;
        const uint32_t ml = (uint32_t)(wp * (16 * S) + 4 * q), m0 = it.ptile * (uint32_t)a.P + ml; // first pixel: in the tile, of all
        const uint32_t obase = (m0 * (uint32_t)a.F + (uint32_t)fcol) * 2u; // byte offset of (pixel m0, filter fcol)
        // valid pixels from m0 on: to the end of the tile's P pixels (rows past them hold other tiles' pixels or stale data) and of the map
        const uint32_t rows_left = fcol < a.F && m0 < (uint32_t)a.M && ml < (uint32_t)a.P ? min((uint32_t)a.M - m0, (uint32_t)a.P - ml) : 0u;
        f32x4 acc[4][S];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int s = 0; s < S; ++s) acc[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};
        uint2 res[S][4]; // [s][i]
        for (int t = 0; t < nst; ++t) {
            __builtin_amdgcn_s_barrier(); // this stage has landed; everyone is done with the stage before
            asm volatile("" ::: "memory");
            if (rb && t == 0) { // residual: asked for at the item's first stage, used after its last
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    uint32_t ob = obase;
                    asm volatile("" : "+v"(ob)); // keeps the 16 addresses from being formed (and held) outside the loop
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bool ok = (uint32_t)(16 * s + i) < rows_left;
                        res[s][i] = load_stream8(rb + (ok ? ob + (uint32_t)(16 * s + i) * (uint32_t)a.F * 2u : 0u));
                    }
                }
            }
            const uint8_t *sb = lds + c_slot * Cfg::kStageBytes;
            if (++c_slot == (uint32_t)D) c_slot = 0;
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                uint4 A[4], B[S];
                const uint8_t *ap = sb + Cfg::kXBytes + (uint32_t)(step * FW * 4) * 1024u + arow;
                const uint8_t *bp = sb + brow + (uint32_t)(((step * 4 + q) ^ (n16 & 7)) * 16);
#pragma unroll
                for (int j = 0; j < 4; ++j) A[j] = *reinterpret_cast<const uint4 *>(ap + j * 1024);
#pragma unroll
                for (int s = 0; s < S; ++s) B[s] = *reinterpret_cast<const uint4 *>(bp + s * 2048);
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j][s] = mfma16<DT>(B[s], A[j], acc[j][s]);
            }
        }
        // ---- bias, residual, activation, round, store --------------------------------------
        {
            float4 bv = float4{0.f, 0.f, 0.f, 0.f};
            if (a.bias) bv = *reinterpret_cast<const float4 *>(lds + lbias + bbuf * 1024u + (uint32_t)(wf * 64 + 4 * n16) * 4u);
            pointwise_epilogue<DT, S>(yb + obase, (uint32_t)a.F * 2u, rows_left, rb != nullptr, acc, res, bv, cl);
        }
        if (c_item + nwg >= nitems) break;
        c_item += nwg;
        bbuf ^= 1u;
    }
}

template <int DT, typename Cfg> static void launch_pointwise_cfg(const RingArgs &a, hipStream_t st)
{
    static std::once_flag once; // one per instantiation
    auto kern = pointwise_ring_kernel<DT, Cfg>;
    allow_lds_once(once, kern, (int)Cfg::kLdsBytes);
    const unsigned grid = (unsigned)std::min<long>((long)a.nptiles * a.nfb, 256);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::kThreads), Cfg::kLdsBytes, st, a);
}

// a.small: 0 = 256 x 128 tiles, 1 = 64 x 64, 2 = 128 x 128; a.nptiles / a.nfb count that configuration's tiles.
int launch_pointwise_ring(int dtype, const RingArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (dtype == NPAS_BF16) {
        if (a.small == 1) launch_pointwise_cfg<NPAS_BF16, PointwiseSmall>(a, st);
        else if (a.small == 2) launch_pointwise_cfg<NPAS_BF16, PointwiseMedium>(a, st);
        else launch_pointwise_cfg<NPAS_BF16, PointwiseBig>(a, st);
    } else if (dtype == NPAS_F16) {
        if (a.small == 1) launch_pointwise_cfg<NPAS_F16, PointwiseSmall>(a, st);
        else if (a.small == 2) launch_pointwise_cfg<NPAS_F16, PointwiseMedium>(a, st);
        else launch_pointwise_cfg<NPAS_F16, PointwiseBig>(a, st);
    } else {
        set_error("pointwise_ring needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("pointwise_ring launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

template <int DT, int S>
static int launch_mfma_inst(const ConvMfmaArgs &a, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    auto kern = conv_gather_mfma_kernel<DT, S>;
    static std::once_flag once; // one per instantiation
    allow_lds_once(once, kern, 64 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds_bytes, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_gather_mfma launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

int launch_conv_mfma(int dtype, int variant, const ConvMfmaArgs &a, unsigned grid, size_t lds_bytes, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (variant == V_MFMA_SLAB) {
        if (dtype == NPAS_BF16) return launch_slab_dt<NPAS_BF16>(a, grid, lds_bytes, st);
        if (dtype == NPAS_F16) return launch_slab_dt<NPAS_F16>(a, grid, lds_bytes, st);
        set_error("conv_slab_mfma needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    const bool s8 = a.g.TH * a.g.TW > 64;
    if (dtype == NPAS_BF16)
        return s8 ? launch_mfma_inst<NPAS_BF16, 8>(a, grid, lds_bytes, st) : launch_mfma_inst<NPAS_BF16, 4>(a, grid, lds_bytes, st);
    if (dtype == NPAS_F16)
        return s8 ? launch_mfma_inst<NPAS_F16, 8>(a, grid, lds_bytes, st) : launch_mfma_inst<NPAS_F16, 4>(a, grid, lds_bytes, st);
    set_error("conv_gather_mfma needs a 16-bit storage type");
    return NPAS_E_DTYPE;
}

// ------------------------------------------------------------------------------
// conv_smallc_mfma: k x k layers with fewer than 8 input channels (the stem of an image network)
// and at most 64 filters.  The reduction index k = (kh*KW + kw)*C + c runs over the whole patch of
// an output pixel (147 for 7 x 7 x 3), so the layer is NS = ceil(K / 32) MFMA steps and its weight
// images (NS x 4 of 1 KB, the column operand) stay in registers for the life of a wave.  The
// activations are the row operand: a workgroup stages the input patch of a 256-pixel output tile
// in LDS as rows of PW*C contiguous values, and a lane gathers its 8 values of a step with eight
// 2-byte reads at pixel base + per-lane offset (consecutive k are consecutive addresses within one
// patch row).  Each gathered fragment feeds the four 16-filter tiles.  Result register i of tile j
// is pixel 4q + i of the 16-pixel block, filter 4 n16 + j: a lane writes four consecutive filters
// of a pixel, a quarter wave one contiguous 2F-byte output row.  Pruned weights are zeros in the
// images: with so few channels every position is kept by some filter of the 64 anyway.
// The patch of the next tile is fetched into registers (kSmallCLoads values per thread at most)
// while the current one is multiplied: fetched inside the tile loop without that, every tile paid
// one load latency per 256 values.  WIDE (an input row is an even number of values, so all rows
// of a patch start at the same 4-byte phase): the patch is fetched and staged as aligned 4-byte
// words, one value of slack in front of each LDS row when the tile starts on an odd value;
// otherwise value by value.
constexpr int kSmallCLoads = 24;

// POOL: the layer is followed by a 3 x 3 / stride 2 / pad 1 max pool.  The tile's conv outputs (after bias,
// activation and rounding; positions outside the conv output as -inf) go to LDS instead of memory, and the
// workgroup then writes the pooled pixels that lie wholly inside the tile: the conv output never reaches HBM.
template <int DT, int NS, bool WIDE, bool POOL, bool HSW>
__device__ __forceinline__ void conv_smallc_mfma_kernel_body(SmallCArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    uint16_t *lds16 = reinterpret_cast<uint16_t *>(lds);
    uint8_t *ctile = lds + (((uint32_t)(a.PH * a.pitch) + 15u) & ~15u); // POOL: the tile's conv outputs, 256 x 128 B
    const Clamp cl = clamp_of(a.act);

    uint4 wreg[NS][4];
#pragma unroll
    for (int st = 0; st < NS; ++st)
#pragma unroll
        for (int j = 0; j < 4; ++j) wreg[st][j] = reinterpret_cast<const uint4 *>(a.wimg)[(st * 4 + j) * 64 + lane];
    // byte offset of this lane's value i of step st from its pixel's patch origin, two to a
    // register (the patch is below 64 KB); slots past K alias the last real one (their weights are zero)
    uint32_t koff2[NS][4];
    const uint32_t kwc = (uint32_t)(a.KW * a.C);
#pragma unroll
    for (int st = 0; st < NS; ++st)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t k = min((uint32_t)(32 * st + 8 * q + i), (uint32_t)a.K - 1u);
            const uint32_t kh = fastdiv(k, a.div_kwc);
            const uint32_t off = kh * (uint32_t)a.pitch + (k - kh * kwc) * 2u;
            if (i & 1) koff2[st][i >> 1] |= off << 16;
            else koff2[st][i >> 1] = off;
        }
    const int fcol = 4 * n16;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.bias && fcol < a.F) {
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = a.bias[fcol + j];
    }
    const uint32_t rowlen = (uint32_t)(a.PW * a.C), patch_elems = (uint32_t)a.PH * rowlen;
    const uint32_t tiles_img = (uint32_t)(a.tilesY * a.tilesX);

    constexpr int NPV = WIDE ? kSmallCLoads / 2 : kSmallCLoads;
    using PV = typename std::conditional<WIDE, uint32_t, uint16_t>::type;
    PV pv[NPV];
    const uint32_t row2 = (uint32_t)a.row2, patch_words = (uint32_t)a.PH * row2;
    auto fetch_patch = [&](uint32_t item) __attribute__((always_inline)) {
        const uint32_t n = fastdiv(item, a.div_tiles), trem = item - n * tiles_img;
        const uint32_t tyi = fastdiv(trem, a.div_tx), txi = trem - tyi * (uint32_t)a.tilesX;
        const int fy0 = POOL ? 2 * (int)tyi * a.PTH - 1 : (int)tyi * a.TH, fx0 = POOL ? 2 * (int)txi * a.PTW - 1 : (int)txi * a.TW; // the tile's first conv pixel
        const int iy0 = fy0 * a.stride - a.pad, ixe0 = (fx0 * a.stride - a.pad) * a.C; // first row, first value of a row
        const uint16_t *xn = x16 + (size_t)n * a.H * (size_t)(a.W * a.C);
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            const uint32_t e = (uint32_t)tid + 256u * i;
            pv[i] = 0; // zero padding
            if (WIDE) {
                const uint32_t py = fastdiv(e, a.div_row2), pd = e - py * row2;
                const int iy = iy0 + (int)py, ixe = (ixe0 & ~1) + 2 * (int)pd; // an even value index: both of the pair in the row or neither
                if (e < patch_words && iy >= 0 && iy < a.H && ixe >= 0 && ixe < a.W * a.C)
                    pv[i] = (PV) * reinterpret_cast<const uint32_t *>(xn + (uint32_t)(iy * (a.W * a.C) + ixe));
            } else {
                const uint32_t py = fastdiv(e, a.div_rowlen), pe = e - py * rowlen;
                const int iy = iy0 + (int)py, ixe = ixe0 + (int)pe;
                if (e < patch_elems && iy >= 0 && iy < a.H && ixe >= 0 && ixe < a.W * a.C) pv[i] = (PV)xn[(uint32_t)(iy * (a.W * a.C) + ixe)];
            }
        }
    };
    uint32_t item = blockIdx.x;
    if (item < a.nitems) fetch_patch(item);
    while (item < a.nitems) {
        const uint32_t n = fastdiv(item, a.div_tiles), trem = item - n * tiles_img;
        const uint32_t tyi = fastdiv(trem, a.div_tx), txi = trem - tyi * (uint32_t)a.tilesX;
        const int ty0 = POOL ? 2 * (int)tyi * a.PTH - 1 : (int)tyi * a.TH, tx0 = POOL ? 2 * (int)txi * a.PTW - 1 : (int)txi * a.TW;
        __syncthreads(); // the tile before has been read
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            const uint32_t e = (uint32_t)tid + 256u * i;
            if (WIDE) {
                const uint32_t py = fastdiv(e, a.div_row2), pd = e - py * row2;
                if (e < patch_words) reinterpret_cast<uint32_t *>(lds)[py * (uint32_t)(a.pitch >> 2) + pd] = (uint32_t)pv[i];
            } else {
                const uint32_t py = fastdiv(e, a.div_rowlen), pe = e - py * rowlen;
                if (e < patch_elems) lds16[py * (uint32_t)(a.pitch >> 1) + pe] = (uint16_t)pv[i];
            }
        }
        __syncthreads();
        // WIDE: the tile's first value sits one value into its LDS rows when it is an odd one
        const uint32_t phase2 = WIDE ? (uint32_t)(((tx0 * a.stride - a.pad) * a.C) & 1) * 2u : 0u;
        const uint32_t next = item + gridDim.x;
        if (next < a.nitems) fetch_patch(next); // lands while this tile is multiplied
#pragma unroll 1
        for (int s = 0; s < 4; ++s) {
            const uint32_t m = (uint32_t)((wave * 4 + s) * 16 + n16); // this lane's operand row
            const uint32_t ty = fastdiv(m, a.div_tw), tx = m - ty * (uint32_t)a.TW;
            const uint8_t *pp = lds + (ty * (uint32_t)a.stride) * (uint32_t)a.pitch + (tx * (uint32_t)(a.stride * a.C)) * 2u + phase2;
            f32x4 acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = f32x4{bv[j], bv[j], bv[j], bv[j]};
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                uint4 af;
                uint32_t h[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    h[i] = *reinterpret_cast<const uint16_t *>(pp + ((i & 1) ? koff2[st][i >> 1] >> 16 : koff2[st][i >> 1] & 0xffffu));
                af.x = h[0] | h[1] << 16;
                af.y = h[2] | h[3] << 16;
                af.z = h[4] | h[5] << 16;
                af.w = h[6] | h[7] << 16;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = mfma16<DT>(af, wreg[st][j], acc[j]);
            }
            // ---- residual, clamp (activation), round, store -------------------------------------
            const uint32_t m0 = (uint32_t)((wave * 4 + s) * 16 + 4 * q);
            uint32_t oty = fastdiv(m0, a.div_tw), otx = m0 - oty * (uint32_t)a.TW;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i > 0 && ++otx == (uint32_t)a.TW) { // the next pixel of the tile, row-major
                    otx = 0;
                    ++oty;
                }
                const int oy = ty0 + (int)oty, ox = tx0 + (int)otx;
                if (POOL) { // to the tile in LDS: [tile pixel][64 filters]
                    const bool valid = (int)oty < a.TH && (uint32_t)oy < (uint32_t)a.Ho && (uint32_t)ox < (uint32_t)a.Wo && fcol < a.F;
                    const uint32_t ninf = DT == NPAS_BF16 ? 0xff80ff80u : 0xfc00fc00u; // -inf, -inf
                    uint2 out{ninf, ninf};
                    if (valid) {
                        out.x = pack2<DT>(clampf<HSW>(acc[0][i], cl), clampf<HSW>(acc[1][i], cl));
                        out.y = pack2<DT>(clampf<HSW>(acc[2][i], cl), clampf<HSW>(acc[3][i], cl));
                    }
                    *reinterpret_cast<uint2 *>(ctile + (m0 + (uint32_t)i) * 128u + (uint32_t)n16 * 8u) = out;
                    continue;
                }
                if (oy >= a.Ho || ox >= a.Wo || fcol >= a.F) continue;
                const size_t o = (((size_t)n * a.Ho + (size_t)oy) * a.Wo + (size_t)ox) * (size_t)a.F + (size_t)fcol;
                float v[4] = {acc[0][i], acc[1][i], acc[2][i], acc[3][i]};
                if (a.residual) {
                    const uint2 r2 = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.residual) + o);
                    v[0] += from_storage<DT>((uint16_t)(r2.x & 0xffffu));
                    v[1] += from_storage<DT>((uint16_t)(r2.x >> 16));
                    v[2] += from_storage<DT>((uint16_t)(r2.y & 0xffffu));
                    v[3] += from_storage<DT>((uint16_t)(r2.y >> 16));
                }
                uint2 out;
                out.x = pack2<DT>(clampf<HSW>(v[0], cl), clampf<HSW>(v[1], cl));
                out.y = pack2<DT>(clampf<HSW>(v[2], cl), clampf<HSW>(v[3], cl));
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(a.y) + o) = out;
            }
        }
        if (POOL) {
            __syncthreads(); // the tile's conv outputs are in LDS
            // thread = (pooled pixel of the tile, 16 filters): the maximum over its 3 x 3 window of conv pixels
            const uint32_t pp = (uint32_t)tid >> 2, f0 = (uint32_t)(tid & 3) * 16u;
            const uint32_t pty = fastdiv(pp, a.div_ptw), ptx = pp - pty * (uint32_t)a.PTW;
            const int py = (int)tyi * a.PTH + (int)pty, px = (int)txi * a.PTW + (int)ptx;
            if ((int)pty < a.PTH && py < a.PHo && px < a.PWo) {
                uint16_t *dst = reinterpret_cast<uint16_t *>(a.y) + (((size_t)n * a.PHo + (size_t)py) * a.PWo + (size_t)px) * (size_t)a.F + f0;
#pragma unroll 1
                for (uint32_t hf = 0; hf < 2; ++hf) { // 8 filters at a time: the main loop's registers stay live across this
                    if ((int)(f0 + 8u * hf) >= a.F) break;
                    float mx[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) mx[e] = -INFINITY;
#pragma unroll
                    for (int d = 0; d < 9; ++d) {
                        const uint32_t cm = (2u * pty + (uint32_t)(d / 3)) * (uint32_t)a.TW + 2u * ptx + (uint32_t)(d % 3);
                        const uint4 v = *reinterpret_cast<const uint4 *>(ctile + cm * 128u + f0 * 2u + hf * 16u);
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            mx[2 * e] = fmaxf(mx[2 * e], from_storage<DT>((uint16_t)(w[e] & 0xffffu)));
                            mx[2 * e + 1] = fmaxf(mx[2 * e + 1], from_storage<DT>((uint16_t)(w[e] >> 16)));
                        }
                    }
                    uint2 o0, o1; // F is a multiple of 4: the second 4 filters may lie past it
                    o0.x = pack2<DT>(mx[0], mx[1]);
                    o0.y = pack2<DT>(mx[2], mx[3]);
                    o1.x = pack2<DT>(mx[4], mx[5]);
                    o1.y = pack2<DT>(mx[6], mx[7]);
                    *reinterpret_cast<uint2 *>(dst + 8 * hf) = o0;
                    if ((int)(f0 + 8u * hf + 4u) < a.F) *reinterpret_cast<uint2 *>(dst + 8 * hf + 4) = o1;
                }
            }
        }
        item = next;
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT, int NS, bool WIDE, bool POOL>
__global__ __launch_bounds__(256, POOL ? 2 : 1) void conv_smallc_mfma_kernel(SmallCArgs a) // (two waves per SIMD: 256 registers; left alone the pooled variant takes 264 and one workgroup per CU)
{
    if (a.act == NPAS_ACT_HARDSWISH) conv_smallc_mfma_kernel_body<DT, NS, WIDE, POOL, true>(a);
    else conv_smallc_mfma_kernel_body<DT, NS, WIDE, POOL, false>(a);
}

// Persistent workgroups, exactly as many as are resident at once (a workgroup that had to wait for
// a free slot would start its share of the tiles when the others are done with theirs).
template <typename K> static void launch_smallc_inst(K kern, const SmallCArgs &a, size_t lds_bytes, hipStream_t st)
{
    // the occupancy query is kept per instantiation and LDS size (a stack repeats the same launch)
    static std::mutex mu;
    static size_t known_lds = (size_t)-1;
    static int known_per_cu = 1;
    int per_cu;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (known_lds != lds_bytes) {
            int v = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, kern, 256, lds_bytes) != hipSuccess || v < 1) v = 1;
            known_lds = lds_bytes;
            known_per_cu = v;
        }
        per_cu = known_per_cu;
    }
    const unsigned grid = (unsigned)std::min<uint32_t>(a.nitems, 256u * (unsigned)std::min(per_cu, 4));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds_bytes, st, a);
}

template <int DT> static int launch_smallc_dt(const SmallCArgs &a, size_t lds_bytes, hipStream_t st)
{
    const bool wide = (a.W * a.C) % 2 == 0;
#define NPAS_SC(N_)                                                                        \
    case N_:                                                                               \
        if (a.pool) {                                                                      \
            if (wide) launch_smallc_inst(conv_smallc_mfma_kernel<DT, N_, true, true>, a, lds_bytes, st); \
            else launch_smallc_inst(conv_smallc_mfma_kernel<DT, N_, false, true>, a, lds_bytes, st);     \
        } else if (wide) launch_smallc_inst(conv_smallc_mfma_kernel<DT, N_, true, false>, a, lds_bytes, st); \
        else launch_smallc_inst(conv_smallc_mfma_kernel<DT, N_, false, false>, a, lds_bytes, st);     \
        break;
    switch (a.nsteps) {
        NPAS_SC(1) NPAS_SC(2) NPAS_SC(3) NPAS_SC(4) NPAS_SC(5)
    default: set_error("conv_smallc_mfma: %d reduction steps (at most 5)", a.nsteps); return NPAS_E_SHAPE;
    }
#undef NPAS_SC
    return NPAS_OK;
}

int launch_conv_smallc(int dtype, const SmallCArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t patch_bytes = (size_t)a.PH * a.pitch;
    const size_t lds_bytes = a.pool ? ((patch_bytes + 15) & ~(size_t)15) + 256 * 128 : patch_bytes;
    const bool pool_ok = !a.pool || (a.TH == 2 * a.PTH + 1 && a.TW == 2 * a.PTW + 1 && a.TH * a.TW <= 256 && a.PTH * a.PTW <= 64 &&
                                    !a.residual && a.PHo > 0 && a.PWo > 0);
    if ((a.pool ? !pool_ok : a.TH * a.TW != 256) || patch_bytes > 48 * 1024 || a.PH * a.PW * a.C > 256 * kSmallCLoads ||
        a.PH * a.row2 > 128 * kSmallCLoads || a.row2 * 4 > a.pitch || a.F > 64 || a.F % 4 != 0 || a.K > 32 * a.nsteps || a.K < 1) {
        set_error("conv_smallc_mfma: plan does not fit the kernel");
        return NPAS_E_SHAPE;
    }
    int rc;
    if (dtype == NPAS_BF16) rc = launch_smallc_dt<NPAS_BF16>(a, lds_bytes, st);
    else if (dtype == NPAS_F16) rc = launch_smallc_dt<NPAS_F16>(a, lds_bytes, st);
    else {
        set_error("conv_smallc_mfma needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    if (rc) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_smallc_mfma launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
// conv_smallm_mfma: k x k layers (C a multiple of 64, ring-format weights) on few output pixels:
// batch 1, the late stages of a network.  The tiled kernels then run a handful of workgroups that
// each walk the whole reduction (C*KH*KW / 32 MFMA steps) alone, one load latency after the
// other.  Here a workgroup owns 64 output pixels x 16 filters (one weight image per step) and its
// sixteen waves split the reduction: a wave takes a contiguous run of steps, fetches each step's
// weight image (1 KB, coalesced) and its four activation fragments (lane = pixel n16 of a block,
// 8 channels = 16 bytes at the tap's input pixel; zero padding by predicate) straight from
// memory, three steps in flight, and accumulates 4 MFMA tiles.  The sixteen partial sums meet in
// LDS; waves 0-3 add them up (always in the same order), add bias / residual, clamp, round and
// store.  Stride and kernel size are free (every address is formed per lane).
struct SmallMPix {
    int n, iy0, ix0; // image and input coordinates of tap (0, 0); n < 0: no such pixel
};

template <int DT, bool HSW>
__device__ __forceinline__ void conv_smallm_mfma_kernel_body(SmallMArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint32_t ptile = blockIdx.x % (uint32_t)a.nptiles, img = blockIdx.x / (uint32_t)a.nptiles;
    const uint32_t fb = img >> 3, tile8 = img & 7u;
    if ((int)(fb * 128u + (tile8 >> 2) * 64u) >= a.F) return; // an image of padding filters only (whole workgroup)
    const int T = a.KH * a.KW, nch = a.C >> 6, S = nch * T * 2;
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    const uint8_t *wb = reinterpret_cast<const uint8_t *>(a.wimg) + (size_t)fb * nch * T * 16384u + tile8 * 1024u + (uint32_t)lane * 16u;

    SmallMPix px[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t m = ptile * 64u + (uint32_t)(s * 16 + n16);
        const uint32_t n = fastdiv(m, a.div_howo), r = m - n * (uint32_t)(a.Ho * a.Wo);
        const uint32_t oy = fastdiv(r, a.div_wo), ox = r - oy * (uint32_t)a.Wo;
        px[s].n = m < (uint32_t)a.M ? (int)n : -1;
        px[s].iy0 = (int)oy * a.stride - a.pad;
        px[s].ix0 = (int)ox * a.stride - a.pad;
    }
    f32x4 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int st0 = wave * S / 16, st1 = (wave + 1) * S / 16; // this wave's steps
    constexpr int NB = 3;                                      // steps in flight
    for (int sb = st0; sb < st1; sb += NB) {
        uint4 wf[NB], xf[NB][4];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int st = sb + u;
            if (st < st1) { // wave-uniform
                // step st = (chunk * T + tap) * 2 + half
                const uint32_t ct = (uint32_t)st >> 1, hs = (uint32_t)st & 1u;
                const uint32_t cc = fastdiv(ct * 2u, a.div_T2), tap = ct - cc * (uint32_t)T;
                const uint32_t kh = fastdiv(tap, a.div_kw), kw = tap - kh * (uint32_t)a.KW;
                wf[u] = *reinterpret_cast<const uint4 *>(wb + (size_t)ct * 16384u + hs * 8192u);
                const uint32_t coff = cc * 64u + hs * 32u + 8u * (uint32_t)q;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int iy = px[s].iy0 + (int)kh, ix = px[s].ix0 + (int)kw;
                    const bool ok = px[s].n >= 0 && (uint32_t)iy < (uint32_t)a.H && (uint32_t)ix < (uint32_t)a.W;
                    xf[u][s] = uint4{0u, 0u, 0u, 0u};
                    if (ok) xf[u][s] = *reinterpret_cast<const uint4 *>(x16 + ((size_t)(px[s].n * a.H + iy) * a.W + ix) * a.C + coff);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            if (sb + u < st1) {
#pragma unroll
                for (int s = 0; s < 4; ++s) acc[s] = mfma16<DT>(wf[u], xf[u][s], acc[s]);
            }
        }
    }
    // ---- the sixteen partial sums meet in LDS: [wave][block][lane] ----------------------------------
    f32x4 *red = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
    for (int s = 0; s < 4; ++s) red[(wave * 4 + s) * 64 + lane] = acc[s];
    __syncthreads();
    if (wave >= 4) return;
    f32x4 sum = red[wave * 64 + lane]; // block s = wave
    for (int w = 1; w < 16; ++w) {
        const f32x4 t = red[(w * 4 + wave) * 64 + lane];
        sum[0] += t[0]; sum[1] += t[1]; sum[2] += t[2]; sum[3] += t[3];
    }
    // row 4q + i of the image is filter 128 fb + 64 (tile8 / 4) + 4 (4q + i) + tile8 % 4; column n16 is pixel 16 wave + n16
    const uint32_t m = ptile * 64u + (uint32_t)(wave * 16 + n16);
    if (m >= (uint32_t)a.M) return;
    const Clamp cl = clamp_of(a.act);
    uint16_t *y16 = reinterpret_cast<uint16_t *>(a.y);
    const uint16_t *r16 = reinterpret_cast<const uint16_t *>(a.residual);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int f = (int)(fb * 128u + (tile8 >> 2) * 64u + 4u * (uint32_t)(4 * q + i) + (tile8 & 3u));
        if (f >= a.F) continue;
        float v = sum[i];
        if (a.bias) v += a.bias[f];
        const size_t o = (size_t)m * a.F + (size_t)f;
        if (r16) v += from_storage<DT>(r16[o]);
        y16[o] = to_storage<DT>(clampf<HSW>(v, cl));
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT>
__global__ __launch_bounds__(1024) void conv_smallm_mfma_kernel(SmallMArgs a)
{
    if (a.act == NPAS_ACT_HARDSWISH) conv_smallm_mfma_kernel_body<DT, true>(a);
    else conv_smallm_mfma_kernel_body<DT, false>(a);
}

int launch_conv_smallm(int dtype, const SmallMArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t lds_bytes = 16 * 4 * 64 * 16;
    const long grid = (long)a.nptiles * a.nimg;
    if (a.C % 64 != 0 || a.M <= 0 || grid > 0x7fffffffL || (double)a.N * a.H * a.W * a.C >= 2147483648.0) {
        set_error("conv_smallm_mfma: unsupported shape");
        return NPAS_E_SHAPE;
    }
    static std::once_flag once[2];
    if (dtype == NPAS_BF16) {
        auto kern = conv_smallm_mfma_kernel<NPAS_BF16>;
        allow_lds_once(once[0], kern, (int)lds_bytes);
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(1024), lds_bytes, st, a);
    } else if (dtype == NPAS_F16) {
        auto kern = conv_smallm_mfma_kernel<NPAS_F16>;
        allow_lds_once(once[1], kern, (int)lds_bytes);
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(1024), lds_bytes, st, a);
    } else {
        set_error("conv_smallm_mfma needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_smallm_mfma launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
template <int VB>
__global__ __launch_bounds__(256) void conv_valu_f32_kernel(ConvValuArgs a)
{
    const int vg = blockIdx.y;
    const uint32_t pix = blockIdx.x * 256u + threadIdx.x;
    const uint32_t npix = (uint32_t)(a.N * a.Ho * a.Wo);
    if (pix >= npix) return;
    const uint32_t ox = pix % (uint32_t)a.Wo, t = pix / (uint32_t)a.Wo;
    const uint32_t oy = t % (uint32_t)a.Ho, n = t / (uint32_t)a.Ho;
    const int f0 = a.vg_f0[vg];
    // fp32 storage, fp64 accumulation: products of two fp32 values are exact in fp64,
    // so the only rounding of note is the final one to fp32 (keeps small outputs of
    // cancelling sums within 1e-5 of the exact result).
    double acc[VB];
#pragma unroll
    for (int j = 0; j < VB; ++j) acc[j] = (a.bias && f0 + j < a.F) ? (double)a.bias[f0 + j] : 0.0;
    const int k0 = a.vg_ptr[vg], k1 = a.vg_ptr[vg + 1];
    const int by = (int)oy * a.stride - a.pad, bx = (int)ox * a.stride - a.pad;
    const float *xn = a.x + (size_t)n * a.H * a.W * a.C;
    // eight positions at a time: their entries and activations are all asked for before the first
    // multiply-add (one at a time, every position cost one load latency); the sums keep their order
    constexpr int U = 8;
    int k = k0;
    for (; k + U <= k1; k += U) {
        float xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t ent = a.vkent[k + u];
            const int iy = by + (int)(ent >> 24), ix = bx + (int)((ent >> 16) & 255u);
            xv[u] = 0.0f;
            if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) xv[u] = xn[(size_t)(iy * a.W + ix) * a.C + (ent & 0xffffu)];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *w = a.vw + (size_t)(k + u) * VB;
#pragma unroll
            for (int j = 0; j < VB; ++j) acc[j] = fma((double)w[j], (double)xv[u], acc[j]);
        }
    }
    for (; k < k1; ++k) {
        const uint32_t ent = a.vkent[k];
        const int iy = by + (int)(ent >> 24), ix = bx + (int)((ent >> 16) & 255u);
        float xv = 0.0f;
        if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) xv = xn[(size_t)(iy * a.W + ix) * a.C + (ent & 0xffffu)];
        const float *w = a.vw + (size_t)k * VB;
#pragma unroll
        for (int j = 0; j < VB; ++j) acc[j] = fma((double)w[j], (double)xv, acc[j]);
    }
    const size_t o = (size_t)pix * a.F + f0;
#pragma unroll
    for (int j = 0; j < VB; ++j)
        if (f0 + j < a.F) {
            double v = acc[j];
            if (a.residual) v += (double)a.residual[o + j];
            a.y[o + j] = act_apply((float)v, a.act);
        }
}

int launch_conv_valu(const ConvValuArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const uint32_t npix = (uint32_t)(a.N * a.Ho * a.Wo);
    dim3 grid((npix + 255) / 256, (unsigned)a.nvg), block(256);
    if (a.nvg > 65535) {
        set_error("too many filter sub-groups (%d) for one launch", a.nvg);
        return NPAS_E_SHAPE;
    }
    switch (a.VB) {
    case 1: hipLaunchKernelGGL(conv_valu_f32_kernel<1>, grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL(conv_valu_f32_kernel<2>, grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL(conv_valu_f32_kernel<4>, grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL(conv_valu_f32_kernel<8>, grid, block, 0, st, a); break;
    default: set_error("unsupported sub-group width %d", a.VB); return NPAS_E_SHAPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_valu_f32 launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------

template <int DT>
__global__ __launch_bounds__(256) void maxpool3x3s2_kernel(const void *x, void *y, int N, int H, int W, int C, int Ho, int Wo)
{
    const size_t total = (size_t)N * Ho * Wo * C;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        int c = (int)(i % C);
        size_t t = i / C;
        int ox = (int)(t % Wo);
        t /= Wo;
        int oy = (int)(t % Ho), n = (int)(t / Ho);
        float m = -INFINITY;
        for (int kh = 0; kh < 3; ++kh) {
            int iy = 2 * oy + kh - 1;
            if (iy < 0 || iy >= H) continue;
            for (int kw = 0; kw < 3; ++kw) {
                int ix = 2 * ox + kw - 1;
                if (ix < 0 || ix >= W) continue;
                m = fmaxf(m, ld_act<DT>(x, ((size_t)(n * H + iy) * W + ix) * C + c));
            }
        }
        st_act<DT>(y, i, m);
    }
}

// 16-bit storage, C a multiple of 8: one thread owns 8 channels of one output pixel
// (16-byte loads and stores).  Values are compared as floats; the winner's bits are kept.
template <int DT>
__global__ __launch_bounds__(256) void maxpool3x3s2_vec8_kernel(const uint4 *x, uint4 *y, int N, int H, int W, int C8,
                                                                int Ho, int Wo)
{
    const uint32_t total = (uint32_t)(N * Ho * Wo * C8);
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < total; i += gridDim.x * 256u) {
        const uint32_t c = i % (uint32_t)C8;
        uint32_t t = i / (uint32_t)C8;
        const int ox = (int)(t % (uint32_t)Wo);
        t /= (uint32_t)Wo;
        const int oy = (int)(t % (uint32_t)Ho), n = (int)(t / (uint32_t)Ho);
        float m[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) m[k] = -INFINITY;
        for (int kh = 0; kh < 3; ++kh) {
            const int iy = 2 * oy + kh - 1;
            if (iy < 0 || iy >= H) continue;
            for (int kw = 0; kw < 3; ++kw) {
                const int ix = 2 * ox + kw - 1;
                if (ix < 0 || ix >= W) continue;
                const uint4 v = x[(uint32_t)((n * H + iy) * W + ix) * (uint32_t)C8 + c];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    m[2 * k] = fmaxf(m[2 * k], from_storage<DT>((uint16_t)(w[k] & 0xffffu)));
                    m[2 * k + 1] = fmaxf(m[2 * k + 1], from_storage<DT>((uint16_t)(w[k] >> 16)));
                }
            }
        }
        uint4 o;
        o.x = pack2<DT>(m[0], m[1]);
        o.y = pack2<DT>(m[2], m[3]);
        o.z = pack2<DT>(m[4], m[5]);
        o.w = pack2<DT>(m[6], m[7]);
        y[i] = o;
    }
}

template <int DT>
__global__ __launch_bounds__(256) void global_avgpool_kernel(const void *x, void *y, int N, int HW, int C)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N * C) return;
    const int n = i / C, c = i % C;
    double s = 0.0; // fp64 sum: the mean of an fp32 map stays within 1e-5 of the exact one
    for (int p = 0; p < HW; ++p) s += (double)ld_act<DT>(x, ((size_t)n * HW + p) * C + c);
    st_act<DT>(y, (size_t)i, (float)(s / (double)HW));
}

// 16-bit storage, C a multiple of 4: a thread averages 4 channels (8-byte loads, a wave reads 512
// contiguous bytes of a pixel), seven loads in flight, fp32 sum (exact to ~1e-6 for a map of a few
// thousand 16-bit values, far inside the storage type's rounding).
template <int DT>
__global__ __launch_bounds__(256) void global_avgpool_vec4_kernel(const void *x, void *y, int N, int HW, int C)
{
    const int C4 = C >> 2;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N * C4) return;
    const int n = i / C4, c4 = i - n * C4;
    const uint2 *xp = reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(x) + (size_t)n * HW * C) + c4;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 7
    for (int p = 0; p < HW; ++p) {
        const uint2 v = xp[(size_t)p * C4];
        s0 += from_storage<DT>((uint16_t)(v.x & 0xffffu));
        s1 += from_storage<DT>((uint16_t)(v.x >> 16));
        s2 += from_storage<DT>((uint16_t)(v.y & 0xffffu));
        s3 += from_storage<DT>((uint16_t)(v.y >> 16));
    }
    const float r = 1.0f / (float)HW;
    uint2 out;
    out.x = pack2<DT>(s0 * r, s1 * r);
    out.y = pack2<DT>(s2 * r, s3 * r);
    reinterpret_cast<uint2 *>(y)[i] = out;
}


__global__ void empty_kernel() {}

int launch_empty(int count, void *stream)
{
    for (int i = 0; i < count; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("empty launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

int launch_maxpool(const void *x, void *y, int N, int H, int W, int C, int dt, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
    size_t total = (size_t)N * Ho * Wo * C;
    unsigned grid = (unsigned)std::min<size_t>((total + 255) / 256, 256 * 64);
    if (dt != NPAS_F32 && C % 8 == 0) {
        grid = (unsigned)std::min<size_t>((total / 8 + 255) / 256, 256 * 32);
        if (dt == NPAS_BF16)
            hipLaunchKernelGGL(maxpool3x3s2_vec8_kernel<NPAS_BF16>, dim3(grid), dim3(256), 0, st, (const uint4 *)x, (uint4 *)y, N, H, W, C / 8, Ho, Wo);
        else
            hipLaunchKernelGGL(maxpool3x3s2_vec8_kernel<NPAS_F16>, dim3(grid), dim3(256), 0, st, (const uint4 *)x, (uint4 *)y, N, H, W, C / 8, Ho, Wo);
    } else if (dt == NPAS_F32) hipLaunchKernelGGL(maxpool3x3s2_kernel<NPAS_F32>, dim3(grid), dim3(256), 0, st, x, y, N, H, W, C, Ho, Wo);
    else if (dt == NPAS_BF16) hipLaunchKernelGGL(maxpool3x3s2_kernel<NPAS_BF16>, dim3(grid), dim3(256), 0, st, x, y, N, H, W, C, Ho, Wo);
    else hipLaunchKernelGGL(maxpool3x3s2_kernel<NPAS_F16>, dim3(grid), dim3(256), 0, st, x, y, N, H, W, C, Ho, Wo);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("maxpool launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

int launch_avgpool(const void *x, void *y, int N, int H, int W, int C, int dt, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned grid = (unsigned)((N * C + 255) / 256);
    if (dt != NPAS_F32 && C % 4 == 0) {
        grid = (unsigned)((N * (C / 4) + 255) / 256);
        if (dt == NPAS_BF16) hipLaunchKernelGGL(global_avgpool_vec4_kernel<NPAS_BF16>, dim3(grid), dim3(256), 0, st, x, y, N, H * W, C);
        else hipLaunchKernelGGL(global_avgpool_vec4_kernel<NPAS_F16>, dim3(grid), dim3(256), 0, st, x, y, N, H * W, C);
    } else if (dt == NPAS_F32) hipLaunchKernelGGL(global_avgpool_kernel<NPAS_F32>, dim3(grid), dim3(256), 0, st, x, y, N, H * W, C);
    else if (dt == NPAS_BF16) hipLaunchKernelGGL(global_avgpool_kernel<NPAS_BF16>, dim3(grid), dim3(256), 0, st, x, y, N, H * W, C);
    else hipLaunchKernelGGL(global_avgpool_kernel<NPAS_F16>, dim3(grid), dim3(256), 0, st, x, y, N, H * W, C);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("avgpool launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

} // namespace npas
