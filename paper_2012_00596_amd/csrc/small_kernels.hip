// gfx950 kernels of libnpas for the two cases where the pruned structure itself, not a dense tile, is the unit of work:
//
// fc_gather_mfma: block-based sparse FC layers (and sparse 1x1 layers on few pixels).  The columns a 16-row block
//   keeps are shared by its rows (paper section 3, block-based pruning: whole columns go inside a block), so they
//   are the K dimension of a dense 16 x K sub-GEMM on the matrix cores: nothing pruned is multiplied, and the
//   weights are read in compact form.
// conv_wave_f32: fp32 block-punched layers with small blocks.  The kept positions of a filter group are split
//   over eight lanes and the partial sums meet in a fixed-order cross-lane reduction: the launch is bound by
//   latency, and a reduction walked by one lane is eight load latencies deep.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "npas_internal.h"
#include "device_util.h"

namespace npas {

// ------------------------------------------------------------------------------
// One workgroup (8 waves) owns 16 output pixels (one MFMA column block) and `tiles_per_wg` (1, 2, 4 or 8) 16-filter
// tiles; the list of a tile is cut into 8 / tiles_per_wg runs of steps, one wave per (tile, run).  The workgroup
// stages the pixels' whole activation rows in LDS (16 x C values, coalesced 16-byte loads; row pitch 2 C + 8 bytes
// so that the sixteen rows start on different banks); a wave then walks its run: per 32 list entries the entries'
// byte offsets (16 bytes per lane, the same for the 16 pixels of a quarter wave) and the weight image (1 KB,
// coalesced) come from memory (the first kFcSteps steps are asked for before the staging, so that their latency and
// the staging's overlap), its pixel's 8 activations from eight 2-byte LDS reads, then one MFMA.  The partial tiles of
// a tile's runs meet in LDS and are added in a fixed order.  The weights are the row operand: result register i of
// lane (pixel n, quarter q) is filter 16 t + 4 q + i.
constexpr int kFcSteps = 4; // list steps whose loads are issued together

template <int DT, bool HSW>
__device__ __forceinline__ void fc_gather_mfma_kernel_body(FcGatherArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const uint32_t nptiles = (uint32_t)(a.M + 15) >> 4;
    const uint32_t ptile = blockIdx.x % nptiles, tg = blockIdx.x / nptiles;
    const uint8_t *xb = reinterpret_cast<const uint8_t *>(a.x);
    f32x4 *red = reinterpret_cast<f32x4 *>(lds + 16u * (uint32_t)a.pitch); // [wave][lane] partial tiles

    // ---- this wave's unit: tile t, run `seg` of `ksplit` -----------------------------------------
    const int ksplit = 8 / a.tiles_per_wg, seg = wave % ksplit;
    const int t = (int)tg * a.tiles_per_wg + wave / ksplit;
    const bool have = t < a.ntiles;
    int s0 = 0, s1 = 0;
    if (have) {
        const int b0 = a.tptr[t], n = a.tptr[t + 1] - b0;
        s0 = b0 + n * seg / ksplit;
        s1 = b0 + n * (seg + 1) / ksplit;
    }
    uint4 ko[kFcSteps], wa[kFcSteps];
    auto fetch = [&](int sb) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kFcSteps; ++u) {
            const int s = min(sb + u, s1 - 1); // past the end: the last step again (not multiplied)
            ko[u] = *reinterpret_cast<const uint4 *>(a.koff + (size_t)s * 32 + 8 * q);
            wa[u] = reinterpret_cast<const uint4 *>(a.wimg)[(size_t)s * 64 + lane];
        }
    };
    if (s0 < s1) fetch(s0);

    // ---- stage the 16 activation rows -------------------------------------------------------
    const uint32_t cv = (uint32_t)a.C >> 3, total = 16u * cv;
    for (uint32_t v = (uint32_t)tid; v < total; v += 512u) {
        const uint32_t pix = v / cv, vec = v - pix * cv;
        const uint32_t m = ptile * 16u + pix;
        uint4 val = uint4{0u, 0u, 0u, 0u};
        if (m < (uint32_t)a.M) {
            uint32_t ipix = m; // input pixel of output pixel m
            if (a.stride != 1) {
                const uint32_t n = fastdiv(m, a.div_howo), r = m - n * (uint32_t)(a.Ho * a.Wo);
                const uint32_t oy = fastdiv(r, a.div_wo), ox = r - oy * (uint32_t)a.Wo;
                ipix = (n * (uint32_t)a.H + oy * (uint32_t)a.stride) * (uint32_t)a.W + ox * (uint32_t)a.stride;
            }
            val = *reinterpret_cast<const uint4 *>(xb + ((size_t)ipix * (size_t)a.C + (size_t)vec * 8u) * 2u);
        }
        uint2 *dst = reinterpret_cast<uint2 *>(lds + pix * (uint32_t)a.pitch + vec * 16u);
        dst[0] = uint2{val.x, val.y};
        dst[1] = uint2{val.z, val.w};
    }
    __syncthreads();

    const uint8_t *row = lds + (uint32_t)n16 * (uint32_t)a.pitch;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int sb = s0; sb < s1; sb += kFcSteps) {
        if (sb != s0) fetch(sb);
#pragma unroll
        for (int u = 0; u < kFcSteps; ++u) {
            if (sb + u < s1) { // wave-uniform
                const uint32_t o[4] = {ko[u].x, ko[u].y, ko[u].z, ko[u].w};
                uint32_t b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    b[i] = (uint32_t)*reinterpret_cast<const uint16_t *>(row + (o[i] & 0xffffu)) |
                           (uint32_t)*reinterpret_cast<const uint16_t *>(row + (o[i] >> 16)) << 16;
                acc = mfma16<DT>(wa[u], uint4{b[0], b[1], b[2], b[3]}, acc);
            }
        }
    }
    if (ksplit > 1) { // the runs of a tile meet in LDS; the wave of run 0 adds them in run order
        red[wave * 64 + lane] = acc;
        __syncthreads();
        if (seg != 0) return;
        for (int r = 1; r < ksplit; ++r) {
            const f32x4 p = red[(wave + r) * 64 + lane];
            acc[0] += p[0]; acc[1] += p[1]; acc[2] += p[2]; acc[3] += p[3];
        }
    }
    // ---- bias, residual, activation, round, store: 4 consecutive filters of this lane's pixel --------
    const uint32_t m = ptile * 16u + (uint32_t)n16;
    const int f0 = 16 * t + 4 * q;
    if (!have || m >= (uint32_t)a.M || f0 >= a.F) return;
    const Clamp cl = clamp_of(a.act);
    float v[4] = {acc[0], acc[1], acc[2], acc[3]};
    if (a.bias) {
        const float4 bv = *reinterpret_cast<const float4 *>(a.bias + f0);
        v[0] += bv.x; v[1] += bv.y; v[2] += bv.z; v[3] += bv.w;
    }
    const size_t o = (size_t)m * (size_t)a.F + (size_t)f0;
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
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT>
__global__ __launch_bounds__(512) void fc_gather_mfma_kernel(FcGatherArgs a)
{
    if (a.act == NPAS_ACT_HARDSWISH) fc_gather_mfma_kernel_body<DT, true>(a);
    else fc_gather_mfma_kernel_body<DT, false>(a);
}

int launch_fc_gather(int dtype, const FcGatherArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t lds_bytes = (size_t)16 * a.pitch + 8 * 1024; // the rows, and eight partial tiles
    const bool tpw_ok = a.tiles_per_wg == 1 || a.tiles_per_wg == 2 || a.tiles_per_wg == 4 || a.tiles_per_wg == 8;
    const long nptiles = ((long)a.M + 15) / 16, ngroups = tpw_ok ? (a.ntiles + a.tiles_per_wg - 1) / a.tiles_per_wg : 0;
    if (a.M <= 0 || a.C % 8 != 0 || a.F % 4 != 0 || a.pitch < 2 * a.C + 8 || a.pitch % 16 != 8 || 2 * a.C > 65535 ||
        lds_bytes > 160 * 1024 || !tpw_ok || nptiles * ngroups > 0x7fffffffL || (double)a.M * a.F >= 2147483648.0) {
        set_error("fc_gather_mfma: unsupported shape (M %d, C %d, F %d)", a.M, a.C, a.F);
        return NPAS_E_SHAPE;
    }
    const unsigned grid = (unsigned)(nptiles * ngroups), block = 512u;
    static std::once_flag once[2];
    if (dtype == NPAS_BF16) {
        auto kern = fc_gather_mfma_kernel<NPAS_BF16>;
        allow_lds_once(once[0], kern, 160 * 1024);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(block), lds_bytes, st, a);
    } else if (dtype == NPAS_F16) {
        auto kern = fc_gather_mfma_kernel<NPAS_F16>;
        allow_lds_once(once[1], kern, 160 * 1024);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(block), lds_bytes, st, a);
    } else {
        set_error("fc_gather_mfma needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("fc_gather_mfma launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
// conv_wave_f32: eight consecutive lanes own one (output pixel, filter sub-group of VB <= 8 filters).  Lane l takes
// list entries l, l + 8, l + 16, ... of the group's kept positions (the lists are padded to multiples of 8 with
// zero weights), all its loads in flight at once, and accumulates in fp64 (products of two fp32 values are exact
// there).  The eight partial sums per filter are added across lanes in a fixed tree (lane pairs 1, 2, 4 apart), so
// the result does not vary from run to run; lanes 0 .. VB-1 then each finish one filter (bias, residual, activation)
// and store it.
constexpr int kWaveLanes = 8;

__device__ __forceinline__ double lane_xor_add(double v, int mask)
{
    return v + __shfl_xor(v, mask, 64);
}

template <int VB>
__global__ __launch_bounds__(256) void conv_wave_f32_kernel(WaveF32Args a)
{
    const int vg = blockIdx.y;
    const uint32_t slot = blockIdx.x * 256u + threadIdx.x;
    const uint32_t l8 = slot & (kWaveLanes - 1), pix = slot >> 3;
    const uint32_t npix = (uint32_t)(a.N * a.Ho * a.Wo);
    const bool live = pix < npix; // (all eight lanes of a pixel agree; dead lanes still take part in the shuffles)
    const uint32_t pc = live ? pix : 0u;
    const uint32_t ox = pc % (uint32_t)a.Wo, t = pc / (uint32_t)a.Wo;
    const uint32_t oy = t % (uint32_t)a.Ho, n = t / (uint32_t)a.Ho;
    const int f0 = a.vg_f0[vg];
    const int k0 = a.wg_ptr[vg], k1 = a.wg_ptr[vg + 1];
    const int by = (int)oy * a.stride - a.pad, bx = (int)ox * a.stride - a.pad;
    const float *xn = a.x + (size_t)n * a.H * a.W * a.C;
    double acc[VB];
#pragma unroll
    for (int j = 0; j < VB; ++j) acc[j] = 0.0;
    constexpr int U = 3; // list rounds in flight
    for (int kb = k0 + (int)l8; kb < k1; kb += kWaveLanes * U) {
        float xv[U];
        float wv[U][VB];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = kb + kWaveLanes * u;
            xv[u] = 0.0f;
#pragma unroll
            for (int j = 0; j < VB; ++j) wv[u][j] = 0.0f;
            if (k < k1) {
                const uint32_t ent = a.kent[k];
                const int iy = by + (int)(ent >> 24), ix = bx + (int)((ent >> 16) & 255u);
                if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) xv[u] = xn[(size_t)(iy * a.W + ix) * a.C + (ent & 0xffffu)];
                const float *w = a.w + (size_t)k * VB;
#pragma unroll
                for (int j = 0; j < VB; ++j) wv[u][j] = w[j];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < VB; ++j) acc[j] = fma((double)wv[u][j], (double)xv[u], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < VB; ++j) {
        acc[j] = lane_xor_add(acc[j], 1);
        acc[j] = lane_xor_add(acc[j], 2);
        acc[j] = lane_xor_add(acc[j], 4);
    }
    double mine = acc[0]; // lane j finishes filter j
#pragma unroll
    for (int j = 1; j < VB; ++j)
        if (l8 == (uint32_t)j) mine = acc[j];
    const int f = f0 + (int)l8;
    if (!live || (int)l8 >= VB || f >= a.F) return;
    if (a.bias) mine += (double)a.bias[f];
    const size_t o = (size_t)pix * a.F + (size_t)f;
    if (a.residual) mine += (double)a.residual[o];
    a.y[o] = act_apply((float)mine, a.act);
}

int launch_conv_wave_f32(const WaveF32Args &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const double slots = (double)a.N * a.Ho * a.Wo * kWaveLanes;
    if (a.nvg > 65535 || slots > 2147483647.0 || a.VB > kWaveLanes) {
        set_error("conv_wave_f32: unsupported shape (%d filter sub-groups, %.0f lanes)", a.nvg, slots);
        return NPAS_E_SHAPE;
    }
    dim3 grid((unsigned)(((long)slots + 255) / 256), (unsigned)a.nvg), block(256);
    switch (a.VB) {
    case 1: hipLaunchKernelGGL(conv_wave_f32_kernel<1>, grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL(conv_wave_f32_kernel<2>, grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL(conv_wave_f32_kernel<4>, grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL(conv_wave_f32_kernel<8>, grid, block, 0, st, a); break;
    default: set_error("unsupported sub-group width %d", a.VB); return NPAS_E_SHAPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("conv_wave_f32 launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

} // namespace npas
