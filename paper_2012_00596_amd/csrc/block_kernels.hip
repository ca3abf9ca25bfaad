// gfx950 kernels of libnpas that run more than one layer, or the depthwise layer between two of them: the fused 1x1 pair,
// the fused 1x1 -> depthwise 3x3 -> 1x1 block, and the depthwise 3x3 layer on its own.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "npas_internal.h"
#include "device_util.h"

namespace npas {

// ------------------------------------------------------------------------------
// Fused pointwise pair: y = act2(W2 * act1(W1 * x + b1) + b2) for two 1x1 layers
// whose intermediate tensor has no other reader (the expand -> project pair of an
// inverted-residual bottleneck).  HBM-bound: x is read once and y written once,
// the F1-channel intermediate never leaves registers.
//
// One wave owns 16 pixels at a time.  Layer 1: the B operand is the pixel's C1
// (<= 32) channels straight from global memory, one MFMA per 16 intermediate
// channels.  The 16x16 result tile of MFMA t holds, in lane (pixel n, quarter q),
// channels 16t + 4q .. 4q+3 of that pixel; two such tiles, activated and rounded
// to the storage type, are exactly the B operand of a 32-deep MFMA of layer 2
// whose K slots are ordered  slot 8q+i <-> channel 16(2j) + 4q + i      (i < 4)
//                            slot 8q+4+i <-> channel 16(2j+1) + 4q + i
// and layer 2's weights are stored pre-permuted to that order.  All weights live
// in registers for the life of the wave.
//
// Pruning shows up twice.  An intermediate channel that no filter of layer 2 keeps
// is dead and layer 1 never computes it; the live channels are renumbered ("slots")
// so that the ones each 16-filter tile of layer 2 needs are contiguous and dead
// channels cost nothing (use[u] records which 32-slot chunks tile u really needs).
struct FppArgs {
    const void *x;
    void *y;
    const void *wblob;   // [NT1 + NT2*NCH][64 lanes][8] 16-bit weight images
    int M, C1, F2;       // pixels, input channels, output channels
    int act1, act2;
    uint32_t use[2];     // per layer-2 tile: which 32-slot chunks it needs
};

constexpr int kFppBlocksPerWave = 8; // 16-pixel blocks a wave owns; all their loads are issued up front

// Straight-line body for a wave that owns exactly CNT blocks starting at block b0.
// No branch between the loads and their uses, so the compiler can wait for block k's
// activations alone (s_waitcnt vmcnt(n)) while later blocks are still in flight.
template <int DT, int NT1, int NT2, int CNT, bool HSW>
__device__ __forceinline__ void fpp_body(const FppArgs &a, int b0, int n16, int q, int lane)
{
    constexpr int NCH = NT1 / 2;
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    uint16_t *y16 = reinterpret_cast<uint16_t *>(a.y);
    const bool ld_on = 8 * q < a.C1;
    const Clamp c1 = clamp_of(a.act1), c2 = clamp_of(a.act2);
    const uint4 *wb = reinterpret_cast<const uint4 *>(a.wblob) + lane;
    uint4 A1[NT1], A2[NT2][NCH];
#pragma unroll
    for (int t = 0; t < NT1; ++t) A1[t] = wb[t * 64];
#pragma unroll
    for (int u = 0; u < NT2; ++u)
#pragma unroll
        for (int j = 0; j < NCH; ++j) A2[u][j] = wb[(NT1 + u * NCH + j) * 64];
    // Rows of a partial last output tile repeat its valid rows (the weight image is built
    // that way), so every lane holds real outputs and stores them, some twice, unpredicated.
    int fst[NT2];
#pragma unroll
    for (int u = 0; u < NT2; ++u) {
        const int nvq = min(4, (a.F2 - 16 * u) >> 2); // valid groups of 4 rows in tile u
        const int q1 = q - nvq, q2 = q1 - nvq;         // q mod nvq without a division
        fst[u] = 16 * u + 4 * (q < nvq ? q : (q1 < nvq ? q1 : (nvq == 1 ? 0 : q2)));
    }
    // Pixels past M are clamped to pixel M-1 for the load AND the store: such a lane
    // recomputes pixel M-1 and writes the same bytes again, which needs no branch.
    uint4 xin[CNT];
    const int cq = ld_on ? 8 * q : 0;
    const uint32_t lmask = ld_on ? 0xffffffffu : 0u;
#pragma unroll
    for (int k = 0; k < CNT; ++k) {
        const int pix = min((b0 + k) * 16 + n16, a.M - 1);
        xin[k] = load_stream16(x16 + (size_t)pix * a.C1 + cq);
    }
    __builtin_amdgcn_sched_barrier(0); // keep every load above the first use (memory-level parallelism)
    // A layer-2 tile that keeps nothing in a chunk has an all-zero image there; it is multiplied
    // anyway rather than branched around (the MFMA pipe has slack, and a branch here would
    // make every load wait).
#pragma unroll
    for (int k = 0; k < CNT; ++k) {
        uint4 xb = xin[k];
        xb.x &= lmask; xb.y &= lmask; xb.z &= lmask; xb.w &= lmask; // K slots past C1 are zero
        f32x4 d1[NT1];
#pragma unroll
        for (int t = 0; t < NT1; ++t) d1[t] = mfma16<DT>(A1[t], xb, f32x4{0.f, 0.f, 0.f, 0.f});
        f32x4 d2[NT2];
#pragma unroll
        for (int u = 0; u < NT2; ++u) d2[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            uint4 b;
            b.x = pack2<DT>(clampf<HSW>(d1[2 * j][0], c1), clampf<HSW>(d1[2 * j][1], c1));
            b.y = pack2<DT>(clampf<HSW>(d1[2 * j][2], c1), clampf<HSW>(d1[2 * j][3], c1));
            b.z = pack2<DT>(clampf<HSW>(d1[2 * j + 1][0], c1), clampf<HSW>(d1[2 * j + 1][1], c1));
            b.w = pack2<DT>(clampf<HSW>(d1[2 * j + 1][2], c1), clampf<HSW>(d1[2 * j + 1][3], c1));
#pragma unroll
            for (int u = 0; u < NT2; ++u) d2[u] = mfma16<DT>(A2[u][j], b, d2[u]);
        }
        const int pix = min((b0 + k) * 16 + n16, a.M - 1);
#pragma unroll
        for (int u = 0; u < NT2; ++u) {
            uint2 o;
            o.x = pack2<DT>(clampf<HSW>(d2[u][0], c2), clampf<HSW>(d2[u][1], c2));
            o.y = pack2<DT>(clampf<HSW>(d2[u][2], c2), clampf<HSW>(d2[u][3], c2));
            store_stream8(y16 + (size_t)pix * a.F2 + fst[u], o); // written once, read by nobody in this launch
        }
    }
}

template <int DT, int NT1, int NT2>
__global__ __launch_bounds__(256, 2) void fused_pointwise_pair_kernel(FppArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n16 = lane & 15, q = lane >> 4;
    const int nblk = (a.M + 15) >> 4;
    const int nw = gridDim.x * 4, gw = blockIdx.x * 4 + wave;
    // contiguous run of blocks per wave, remainder spread over the first waves
    const int base = nblk / nw, extra = nblk % nw;
    const int b0 = gw * base + min(gw, extra), cnt = base + (gw < extra ? 1 : 0);
    // (the activation kinds compiled in: see clampf)
    auto run = [&](auto hsw) __attribute__((always_inline)) {
        constexpr bool H = decltype(hsw)::value;
        switch (cnt) { // wave-uniform
        case 1: fpp_body<DT, NT1, NT2, 1, H>(a, b0, n16, q, lane); break;
        case 2: fpp_body<DT, NT1, NT2, 2, H>(a, b0, n16, q, lane); break;
        case 3: fpp_body<DT, NT1, NT2, 3, H>(a, b0, n16, q, lane); break;
        case 4: fpp_body<DT, NT1, NT2, 4, H>(a, b0, n16, q, lane); break;
        case 5: fpp_body<DT, NT1, NT2, 5, H>(a, b0, n16, q, lane); break;
        case 6: fpp_body<DT, NT1, NT2, 6, H>(a, b0, n16, q, lane); break;
        case 7: fpp_body<DT, NT1, NT2, 7, H>(a, b0, n16, q, lane); break;
        case 8: fpp_body<DT, NT1, NT2, 8, H>(a, b0, n16, q, lane); break;
        default: break;
        }
    };
    if (a.act1 == NPAS_ACT_HARDSWISH || a.act2 == NPAS_ACT_HARDSWISH) run(std::true_type{});
    else run(std::false_type{});
}

template <int DT, int NT1, int NT2> static void fpp_launch(const FppArgs &a, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((fused_pointwise_pair_kernel<DT, NT1, NT2>), dim3(grid), dim3(256), 0, st, a);
}

// nt1 = live intermediate tiles rounded up to an even count, nt2 = output tiles
bool fpp_supported(int nt1, int nt2) { return nt1 >= 2 && nt1 <= 12 && nt1 % 2 == 0 && (nt2 == 1 || nt2 == 2); }

int launch_fused_pointwise_pair(int dtype, const void *x, void *y, const void *wblob, int M, int C1, int nt1, int F2,
                                int act1, int act2, uint32_t use0, uint32_t use1, void *stream)
{
    FppArgs a{x, y, wblob, M, C1, F2, act1, act2, {use0, use1}};
    hipStream_t st = (hipStream_t)stream;
    const int nt2 = (F2 + 15) / 16;
    const int nblk = (M + 15) / 16;
    // two workgroups per CU when the batch allows it, more when a wave would otherwise own
    // more than kFppBlocksPerWave blocks
    const int min_grid = (nblk + 4 * kFppBlocksPerWave - 1) / (4 * kFppBlocksPerWave);
    unsigned grid = (unsigned)std::max(min_grid, std::min((nblk + 3) / 4, 512));
#define NPAS_FPP_CASE(N1, N2)                                                              \
    if (nt1 == N1 && nt2 == N2) {                                                          \
        if (dtype == NPAS_BF16) fpp_launch<NPAS_BF16, N1, N2>(a, grid, st);                \
        else fpp_launch<NPAS_F16, N1, N2>(a, grid, st);                                    \
    } else
    NPAS_FPP_CASE(2, 1) NPAS_FPP_CASE(2, 2) NPAS_FPP_CASE(4, 1) NPAS_FPP_CASE(4, 2) NPAS_FPP_CASE(6, 1)
    NPAS_FPP_CASE(6, 2) NPAS_FPP_CASE(8, 1) NPAS_FPP_CASE(8, 2) NPAS_FPP_CASE(10, 1) NPAS_FPP_CASE(10, 2)
    NPAS_FPP_CASE(12, 1) NPAS_FPP_CASE(12, 2)
    {
        set_error("fused pointwise pair: unsupported tile counts %d, %d", nt1, nt2);
        return NPAS_E_SHAPE;
    }
#undef NPAS_FPP_CASE
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("fused_pointwise_pair launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
// fused_inverted_residual: y = act3(W3 . act2(DW3x3(act1(W1 . x + b1)) + b2) + b3 [+ x]) for the cascade
// 1x1 -> 3x3 depthwise (stride 1 or 2) -> 1x1 of the search space (section 5.1.1) when the two wide
// tensors between the layers have no other reader.  They never leave the CU: HBM sees x once and y once.
// The block input is added at stride 1 only (at stride 2 the shapes differ); the biases are optional.
//
// A workgroup (4 waves) owns an output tile of TH x TW pixels.
//   1. Expansion: for the input pixels under the tile plus a one-pixel halo ((TH-1) stride + 3 rows),
//      16 pixels at a time, layer 1's MFMAs
//      (K = C1 <= 32 in one step) produce 16 x 16 output tiles that get their bias, are clamped, rounded and
//      written to LDS as [halo pixel][slot] in the storage type.  Halo pixels outside the image are written
//      as zero, as the padding of the depthwise
//      layer must be.  A slot is an intermediate channel some filter of layer 3 keeps; channels
//      nobody keeps are dead and are never computed (the pruning of layer 3 pays in layers 1 and 2).
//   2. Depthwise + projection, 16 output pixels at a time: lane (q, n) forms the depthwise output
//      of pixel n for 8 slots (nine 16-byte LDS reads of activations, weights from an LDS table,
//      one dot2 instruction per multiply-add on the packed pairs, fp32 accumulate, clamp, round):
//      exactly the B operand of layer 3's MFMA step for
//      those 32 slots.  After all steps: residual (x again, 8 bytes per lane), clamp, round, store.
// Bound: vector ALUs (the depthwise arithmetic and the unpacking of 16-bit pairs), not HBM.
// c + x.lo * w.lo + x.hi * w.hi on two packed 16-bit pairs (v_dot2c_f32_bf16 / v_dot2_f32_f16).  With one half of
// w zero this is a multiply-add on the other half without unpacking it (the zero half adds an exact zero as long
// as the activation beside it is finite).
template <int DT> __device__ __forceinline__ float dot2acc(uint32_t x, uint32_t w, float c)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    if (DT == NPAS_BF16) return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x), __builtin_bit_cast(bf16x2, w), c, false);
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, x), __builtin_bit_cast(f16x2, w), c, false);
}

// Padding of a halo pixel's row in LDS: 32 bytes measured best among 16 .. 144 for 96 slots (a 256-byte row
// pitch, i.e. 64, is the worst case: every pixel on the same banks).
constexpr uint32_t kIrPad = 32;

struct IrArgs {
    const void *x;
    void *y;
    const void *w1;      // [nt1][64 lanes][8] layer-1 A-operand images, rows in slot order
    const void *w3;      // [nt3][nk][64 lanes][8] layer-3 A-operand images, K in slot order
    const uint32_t *wdw; // [9][nslots] depthwise weights in slot order, each alone in its half of a 16-bit pair
                         // (even slots low, odd slots high, the other half zero)
    const int *perm;     // [nslots] intermediate channel of each slot, -1: padding slot
    const float *b1, *b2, *b3; // biases of the three layers in channel order, or null
    int N, H, W, C1, F3;
    int stride, Ho, Wo;  // of the depthwise layer; output map
    int nt1, nk, nt3;    // slots / 16, slots / 32, ceil(F3 / 16)
    int TH, TW, tilesY, tilesX;
    int act1, act2, act3;
    int residual;        // 1: add the block input (needs F3 == C1 and stride 1)
    uint32_t div_tw, div_pw;
};

// BIAS: some layer of the block has one (bias tables in LDS, halo pixels outside the image zeroed explicitly: the
// padding of the depthwise layer is zero, not act1(b1)).  Without, x = 0 there already gives zero, and the kernel
// keeps the registers that let three workgroups share a CU.
template <int DT, bool BIAS, bool HSW>
__device__ __forceinline__ void fused_inverted_residual_kernel_body(IrArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n16 = lane & 15, q = lane >> 4;
    const int PH = (a.TH - 1) * a.stride + 3, PW = (a.TW - 1) * a.stride + 3, nslots = a.nt1 * 16;
    const int nhb = (PH * PW + 15) >> 4, nob = (a.TH * a.TW + 15) >> 4; // 16-pixel blocks of the halo tile / the tile
    const uint32_t pitch = (uint32_t)nslots * 2u + kIrPad;               // bytes per halo pixel
    uint8_t *y1 = lds;
    uint32_t *dww = reinterpret_cast<uint32_t *>(lds + (size_t)nhb * 16 * pitch);
    float *lb1 = reinterpret_cast<float *>(dww + 9 * nslots), *lb2 = lb1 + nslots; // biases of layers 1 and 2 in slot order

    uint32_t tile = blockIdx.x;
    const int txi = (int)(tile % (uint32_t)a.tilesX);
    tile /= (uint32_t)a.tilesX;
    const int tyi = (int)(tile % (uint32_t)a.tilesY), n = (int)(tile / (uint32_t)a.tilesY);
    const int ty0 = tyi * a.TH, tx0 = txi * a.TW;             // in the output map
    const int iy0 = ty0 * a.stride - 1, ix0 = tx0 * a.stride - 1; // input pixel of halo pixel (0, 0)

    for (int i = tid; i < 9 * nslots; i += 256) dww[i] = a.wdw[i];

    // ---- 1. expansion into LDS ------------------------------------------------------------
    const Clamp cl1 = clamp_of(a.act1);
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    const uint4 *w1 = reinterpret_cast<const uint4 *>(a.w1) + lane;
    // every load of this phase is issued before the first MFMA: the wave's activation vectors (up to four
    // 16-pixel blocks) and layer 1's images, so that one memory latency is paid instead of one per block and image
    uint4 xv[4], w1r[12];
    bool inside[4]; // the lane's halo pixel of round r lies in the image
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int hb = wave + 4 * r;
        const uint32_t hp = (uint32_t)(hb * 16 + n16);
        const uint32_t py = fastdiv(hp, a.div_pw), px = hp - py * (uint32_t)PW;
        const int iy = iy0 + (int)py, ix = ix0 + (int)px;
        inside[r] = hb < nhb && (int)py < PH && (uint32_t)iy < (uint32_t)a.H && (uint32_t)ix < (uint32_t)a.W;
        xv[r] = uint4{0u, 0u, 0u, 0u};
        if (inside[r] && 8 * q < a.C1) xv[r] = *reinterpret_cast<const uint4 *>(x16 + ((size_t)(n * a.H + iy) * a.W + ix) * a.C1 + 8 * q);
    }
#pragma unroll
    for (int t = 0; t < 12; ++t) w1r[t] = t < a.nt1 ? w1[t * 64] : uint4{0u, 0u, 0u, 0u};
    if (BIAS) {
        for (int i = tid; i < nslots; i += 256) { // bias tables, asked for behind the loads above
            const int c = a.b1 || a.b2 ? a.perm[i] : -1;
            lb1[i] = a.b1 && c >= 0 ? a.b1[c] : 0.f;
            lb2[i] = a.b2 && c >= 0 ? a.b2[c] : 0.f;
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int hb = wave + 4 * r;
        uint8_t *dst = y1 + (size_t)(hb * 16 + n16) * pitch + (uint32_t)(4 * q) * 2u;
#pragma unroll
        for (int t = 0; t < 12; ++t) {
            if (hb < nhb && t < a.nt1) {
                const f32x4 d = mfma16<DT>(w1r[t], xv[r], f32x4{0.f, 0.f, 0.f, 0.f});
                float4 bb = float4{0.f, 0.f, 0.f, 0.f};
                if (BIAS) bb = *reinterpret_cast<const float4 *>(lb1 + 16 * t + 4 * q); // result register i: slot 16 t + 4 q + i
                uint2 o;
                o.x = pack2<DT>(clampf<HSW>(d[0] + bb.x, cl1), clampf<HSW>(d[1] + bb.y, cl1));
                o.y = pack2<DT>(clampf<HSW>(d[2] + bb.z, cl1), clampf<HSW>(d[3] + bb.w, cl1));
                if (BIAS && !inside[r]) o = uint2{0u, 0u}; // padding of the depthwise layer, whatever the bias
                *reinterpret_cast<uint2 *>(dst + t * 32) = o;
            }
        }
    }
    __syncthreads();

    // ---- 2. depthwise + projection ---------------------------------------------------------
    const Clamp cl2 = clamp_of(a.act2), cl3 = clamp_of(a.act3);
    const uint4 *w3 = reinterpret_cast<const uint4 *>(a.w3) + lane;
    uint16_t *y16 = reinterpret_cast<uint16_t *>(a.y);
    for (int ob = wave; ob < nob; ob += 4) {
        const uint32_t m = (uint32_t)(ob * 16 + n16);
        const uint32_t ty = fastdiv(m, a.div_tw), tx = m - ty * (uint32_t)a.TW;
        const int oy = ty0 + (int)ty, ox = tx0 + (int)tx;
        const bool valid = (int)ty < a.TH && oy < a.Ho && ox < a.Wo;
        const uint8_t *base = y1 + (valid ? (size_t)((ty * (uint32_t)PW + tx) * (uint32_t)a.stride) * pitch : 0) + (uint32_t)(8 * q) * 2u;
        f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < a.nk; ++k) {
            const uint4 w3a = w3[k * 64], w3b = a.nt3 == 2 ? w3[(a.nk + k) * 64] : uint4{0u, 0u, 0u, 0u}; // asked for before the taps
            float4 ba = float4{0.f, 0.f, 0.f, 0.f}, bb = ba;
            if (BIAS) {
                ba = *reinterpret_cast<const float4 *>(lb2 + 32 * k + 8 * q);
                bb = *reinterpret_cast<const float4 *>(lb2 + 32 * k + 8 * q + 4);
            }
            float s[8] = {ba.x, ba.y, ba.z, ba.w, bb.x, bb.y, bb.z, bb.w};
            uint4 vt[9]; // all nine taps asked for before the first is used
#pragma unroll
            for (int tap = 0; tap < 9; ++tap)
                vt[tap] = *reinterpret_cast<const uint4 *>(base + (size_t)((tap / 3) * PW + tap % 3) * pitch + k * 64);
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const uint4 v = vt[tap];
                const uint4 wa = *reinterpret_cast<const uint4 *>(dww + tap * nslots + 32 * k + 8 * q);
                const uint4 wb = *reinterpret_cast<const uint4 *>(dww + tap * nslots + 32 * k + 8 * q + 4);
                s[0] = dot2acc<DT>(v.x, wa.x, s[0]);
                s[1] = dot2acc<DT>(v.x, wa.y, s[1]);
                s[2] = dot2acc<DT>(v.y, wa.z, s[2]);
                s[3] = dot2acc<DT>(v.y, wa.w, s[3]);
                s[4] = dot2acc<DT>(v.z, wb.x, s[4]);
                s[5] = dot2acc<DT>(v.z, wb.y, s[5]);
                s[6] = dot2acc<DT>(v.w, wb.z, s[6]);
                s[7] = dot2acc<DT>(v.w, wb.w, s[7]);
            }
            uint4 b;
            b.x = pack2<DT>(clampf<HSW>(s[0], cl2), clampf<HSW>(s[1], cl2));
            b.y = pack2<DT>(clampf<HSW>(s[2], cl2), clampf<HSW>(s[3], cl2));
            b.z = pack2<DT>(clampf<HSW>(s[4], cl2), clampf<HSW>(s[5], cl2));
            b.w = pack2<DT>(clampf<HSW>(s[6], cl2), clampf<HSW>(s[7], cl2));
            acc0 = mfma16<DT>(w3a, b, acc0);
            if (a.nt3 == 2) acc1 = mfma16<DT>(w3b, b, acc1);
        }
        if (!valid) continue;
        const size_t pix = (size_t)(n * a.Ho + oy) * a.Wo + ox;
        for (int u = 0; u < a.nt3; ++u) {
            const int f = 16 * u + 4 * q;
            if (f >= a.F3) continue;
            const f32x4 d = u == 0 ? acc0 : acc1;
            float v[4] = {d[0], d[1], d[2], d[3]};
            if (BIAS && a.b3) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] += a.b3[f + i];
            }
            if (a.residual) {
                const uint2 r = *reinterpret_cast<const uint2 *>(x16 + pix * a.C1 + f);
                v[0] += from_storage<DT>((uint16_t)(r.x & 0xffffu));
                v[1] += from_storage<DT>((uint16_t)(r.x >> 16));
                v[2] += from_storage<DT>((uint16_t)(r.y & 0xffffu));
                v[3] += from_storage<DT>((uint16_t)(r.y >> 16));
            }
            uint2 o;
            o.x = pack2<DT>(clampf<HSW>(v[0], cl3), clampf<HSW>(v[1], cl3));
            o.y = pack2<DT>(clampf<HSW>(v[2], cl3), clampf<HSW>(v[3], cl3));
            store_stream8(y16 + pix * a.F3 + f, o);
        }
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT, bool BIAS, bool HSW>
__global__ __launch_bounds__(256, 3) void fused_inverted_residual_kernel(IrArgs a) // three workgroups per CU: at most 168 registers
{
    fused_inverted_residual_kernel_body<DT, BIAS, HSW>(a); // (a kernel per activation class, chosen at the launch: registers are tight here)
}

size_t fused_ir_lds_bytes(int TH, int TW, int nslots, int stride)
{
    const int nhb = (((TH - 1) * stride + 3) * ((TW - 1) * stride + 3) + 15) / 16;
    return (size_t)nhb * 16 * ((size_t)nslots * 2 + kIrPad) + (size_t)9 * nslots * 4 + (size_t)2 * nslots * 4;
}

int launch_fused_inverted_residual(int dtype, const IrLaunch &l, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int N = l.N, H = l.H, W = l.W, C1 = l.C1, F3 = l.F3, nslots = l.nslots, TH = l.TH, TW = l.TW, stride = l.stride;
    IrArgs a;
    a.x = l.x; a.y = l.y; a.w1 = l.w1; a.w3 = l.w3; a.wdw = l.wdw; a.perm = l.perm;
    a.b1 = l.b1; a.b2 = l.b2; a.b3 = l.b3;
    a.N = N; a.H = H; a.W = W; a.C1 = C1; a.F3 = F3;
    a.stride = stride; a.Ho = (H - 1) / stride + 1; a.Wo = (W - 1) / stride + 1; // 3 x 3, padding 1
    a.nt1 = nslots / 16; a.nk = nslots / 32; a.nt3 = (F3 + 15) / 16;
    a.TH = TH; a.TW = TW; a.tilesY = (a.Ho + TH - 1) / TH; a.tilesX = (a.Wo + TW - 1) / TW;
    a.act1 = l.act1; a.act2 = l.act2; a.act3 = l.act3; a.residual = l.residual;
    const int PH = (TH - 1) * stride + 3, PW = (TW - 1) * stride + 3;
    a.div_tw = TW <= 1 ? 0u : (uint32_t)(((1ull << 32) + TW - 1) / TW);
    a.div_pw = (uint32_t)(((1ull << 32) + PW - 1) / PW);
    const size_t lds_bytes = fused_ir_lds_bytes(TH, TW, nslots, stride);
    if (nslots <= 0 || nslots % 32 || nslots > 192 || TH < 1 || TW < 1 || PH * PW > 256 || a.nt3 < 1 || a.nt3 > 2 || C1 > 32 || C1 % 8 || F3 % 4 ||
        lds_bytes > 160 * 1024 || (stride != 1 && stride != 2) || (l.residual && (F3 != C1 || stride != 1)) || !l.perm) {
        set_error("fused inverted residual: unsupported shape (slots %d, C1 %d, F3 %d, stride %d, LDS %zu)", nslots, C1, F3, stride, lds_bytes);
        return NPAS_E_SHAPE;
    }
    const long grid = (long)N * a.tilesY * a.tilesX;
    const bool bias = l.b1 || l.b2 || l.b3;
    const bool hsw = l.act1 == NPAS_ACT_HARDSWISH || l.act2 == NPAS_ACT_HARDSWISH || l.act3 == NPAS_ACT_HARDSWISH;
    static std::once_flag once[8];
    auto go = [&](auto kern, std::once_flag &flag) {
        allow_lds_once(flag, kern, 160 * 1024);
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds_bytes, st, a);
    };
    if (dtype == NPAS_BF16) {
        if (bias && hsw) go(fused_inverted_residual_kernel<NPAS_BF16, true, true>, once[0]);
        else if (bias) go(fused_inverted_residual_kernel<NPAS_BF16, true, false>, once[1]);
        else if (hsw) go(fused_inverted_residual_kernel<NPAS_BF16, false, true>, once[2]);
        else go(fused_inverted_residual_kernel<NPAS_BF16, false, false>, once[3]);
    } else if (dtype == NPAS_F16) {
        if (bias && hsw) go(fused_inverted_residual_kernel<NPAS_F16, true, true>, once[4]);
        else if (bias) go(fused_inverted_residual_kernel<NPAS_F16, true, false>, once[5]);
        else if (hsw) go(fused_inverted_residual_kernel<NPAS_F16, false, true>, once[6]);
        else go(fused_inverted_residual_kernel<NPAS_F16, false, false>, once[7]);
    } else {
        set_error("fused inverted residual needs a 16-bit storage type");
        return NPAS_E_DTYPE;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("fused_inverted_residual launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

// ------------------------------------------------------------------------------
// Depthwise 3x3, padding 1: one thread per (output pixel, vector of V channels); V * element
// size = 16 bytes when the channel count allows it, so every load and store is one 16-byte
// access, coalesced along the channels.  HBM-bound: the nine taps of a pixel come from L1 / L2.
// fp32 storage accumulates in fp64, like the fp32 convolution kernel (products of two fp32
// values are exact in fp64, so the stored result is the correctly rounded one).
template <int DT, int V>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const void *x, void *y, const void *w, const float *bias,
                                                           const void *residual, int N, int H, int W, int C, int Ho,
                                                           int Wo, int stride, int act)
{
    const int CV = C / V;
    const size_t total = (size_t)N * Ho * Wo * CV;
    const Clamp cl = clamp_of(act);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int cv = (int)(i % CV);
        size_t r = i / CV;
        const int ox = (int)(r % Wo);
        r /= Wo;
        const int oy = (int)(r % Ho), n = (int)(r / Ho);
        using Acc = typename std::conditional<DT == NPAS_F32, double, float>::type;
        Acc acc[V];
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] = bias ? (Acc)bias[cv * V + k] : (Acc)0;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int iy = oy * stride + kh - 1;
            if (iy < 0 || iy >= H) continue;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int ix = ox * stride + kw - 1;
                if (ix < 0 || ix >= W) continue;
                const size_t xo = ((size_t)(n * H + iy) * W + ix) * C + (size_t)cv * V;
                const size_t wo = (size_t)(kh * 3 + kw) * C + (size_t)cv * V;
                if (V == 8) { // 16-bit storage, 8 channels
                    const uint4 xv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(x) + xo);
                    const uint4 wv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(w) + wo);
                    const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w}, ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        acc[2 * k] += from_storage<DT>((uint16_t)(xs[k] & 0xffffu)) * from_storage<DT>((uint16_t)(ws[k] & 0xffffu));
                        acc[2 * k + 1] += from_storage<DT>((uint16_t)(xs[k] >> 16)) * from_storage<DT>((uint16_t)(ws[k] >> 16));
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < V; ++k) acc[k] += (Acc)ld_act<DT>(x, xo + k) * (Acc)ld_act<DT>(w, wo + k);
                }
            }
        }
        const size_t yo = ((size_t)(n * Ho + oy) * Wo + ox) * C + (size_t)cv * V;
        if (residual) {
#pragma unroll
            for (int k = 0; k < V; ++k) acc[k] += (Acc)ld_act<DT>(residual, yo + k);
        }
        if (V == 8) {
            uint4 out;
            out.x = pack2<DT>(clampf((float)acc[0], cl), clampf((float)acc[1], cl));
            out.y = pack2<DT>(clampf((float)acc[2], cl), clampf((float)acc[3], cl));
            out.z = pack2<DT>(clampf((float)acc[4], cl), clampf((float)acc[5], cl));
            out.w = pack2<DT>(clampf((float)acc[6], cl), clampf((float)acc[7], cl));
            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(y) + yo) = out;
        } else {
#pragma unroll
            for (int k = 0; k < V; ++k) st_act<DT>(y, yo + k, clampf((float)acc[k], cl));
        }
    }
}

// 16-bit storage, C a multiple of 8: one thread owns 8 channels of kDwRows consecutive output rows
// of one output column.  It walks down the input rows once (each input vector is loaded once per
// thread and feeds up to three output rows), keeps the 9 tap weights of its channels in registers
// for its whole life, and multiplies on packed pairs: dot2(x pair, weight pair with the other half
// zeroed) adds exactly one product in fp32, with no unpacking of the activations.  Consecutive
// lanes are consecutive 16-byte channel vectors of a pixel, then consecutive pixels of a row.
constexpr int kDwRows = 4;

struct DwArgs {
    const void *x;
    void *y;
    const void *w;        // [9][C] storage type, tap-major
    const float *bias;
    const void *residual;
    int N, H, W, C, Ho, Wo, act;
    uint32_t CV, nyb, total;            // channel vectors, row blocks per image, threads
    uint32_t div_cv, div_wo, div_nyb;   // fastdiv magics
};

template <int DT, int STRIDE, bool HSW>
__device__ __forceinline__ void depthwise3x3_rows_kernel_body(DwArgs a)
{
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= a.total) return;
    uint32_t t = fastdiv(idx, a.div_cv);
    const uint32_t cv = idx - t * a.CV;
    uint32_t t2 = fastdiv(t, a.div_wo);
    const int ox = (int)(t - t2 * (uint32_t)a.Wo);
    const uint32_t n = fastdiv(t2, a.div_nyb);
    const int oy0 = (int)(t2 - n * a.nyb) * kDwRows;
    const Clamp cl = clamp_of(a.act);
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(a.x);
    const uint16_t *w16 = reinterpret_cast<const uint16_t *>(a.w);

    uint32_t wlo[9][4], whi[9][4]; // each pair of weights with the upper / the lower one zeroed
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
        const uint4 wv = *reinterpret_cast<const uint4 *>(w16 + (size_t)tap * a.C + (size_t)cv * 8);
        const uint32_t ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            wlo[tap][k] = ws[k] & 0xffffu;
            whi[tap][k] = ws[k] & 0xffff0000u;
        }
    }
    float acc[kDwRows][8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float b = a.bias ? a.bias[cv * 8 + k] : 0.f;
#pragma unroll
        for (int j = 0; j < kDwRows; ++j) acc[j][k] = b;
    }
    constexpr int NR = (kDwRows - 1) * STRIDE + 3; // input rows this thread reads
    const int ix0 = ox * STRIDE - 1, iy0 = oy0 * STRIDE - 1;
    const size_t img = (size_t)n * a.H;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int iy = iy0 + r;
        const bool rowok = iy >= 0 && iy < a.H; // zero padding above and below the image
        uint4 xv[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int ix = ix0 + kw;
            const bool ok = rowok && ix >= 0 && ix < a.W;
            xv[kw] = uint4{0u, 0u, 0u, 0u};
            if (ok) xv[kw] = *reinterpret_cast<const uint4 *>(x16 + ((img + (size_t)iy) * a.W + (size_t)ix) * a.C + (size_t)cv * 8);
        }
#pragma unroll
        for (int j = 0; j < kDwRows; ++j) {
            const int kh = r - j * STRIDE; // compile-time after unrolling
            if (kh < 0 || kh > 2) continue;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const uint32_t xs[4] = {xv[kw].x, xv[kw].y, xv[kw].z, xv[kw].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    acc[j][2 * k] = dot2acc<DT>(xs[k], wlo[kh * 3 + kw][k], acc[j][2 * k]);
                    acc[j][2 * k + 1] = dot2acc<DT>(xs[k], whi[kh * 3 + kw][k], acc[j][2 * k + 1]);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kDwRows; ++j) {
        const int oy = oy0 + j;
        if (oy >= a.Ho) continue;
        const size_t yo = (((size_t)n * a.Ho + (size_t)oy) * a.Wo + (size_t)ox) * a.C + (size_t)cv * 8;
        if (a.residual) {
            const uint4 rv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(a.residual) + yo);
            const uint32_t rs[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                acc[j][2 * k] += from_storage<DT>((uint16_t)(rs[k] & 0xffffu));
                acc[j][2 * k + 1] += from_storage<DT>((uint16_t)(rs[k] >> 16));
            }
        }
        uint4 out;
        out.x = pack2<DT>(clampf<HSW>(acc[j][0], cl), clampf<HSW>(acc[j][1], cl));
        out.y = pack2<DT>(clampf<HSW>(acc[j][2], cl), clampf<HSW>(acc[j][3], cl));
        out.z = pack2<DT>(clampf<HSW>(acc[j][4], cl), clampf<HSW>(acc[j][5], cl));
        out.w = pack2<DT>(clampf<HSW>(acc[j][6], cl), clampf<HSW>(acc[j][7], cl));
        store_stream16(reinterpret_cast<uint16_t *>(a.y) + yo, out);
    }
}
// The activation kind is compiled in: hard-swish behind a (wave-uniform) branch per value kept the compiler from
// interleaving loads, MFMAs and epilogue arithmetic across values and cost the launches without it 15-50 %.
template <int DT, int STRIDE, bool HSW>
__global__ __launch_bounds__(256, 3) void depthwise3x3_rows_kernel(DwArgs a)
{
    depthwise3x3_rows_kernel_body<DT, STRIDE, HSW>(a); // (one body per kernel: with two behind a branch the stride-2 variant's spills moved into its row loop)
}

static uint32_t magic32(uint32_t d) { return d <= 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); }

int launch_depthwise3x3(int dt, const void *x, void *y, const void *w, const float *bias, const void *residual, int N, int H,
                        int W, int C, int stride, int act, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
    const bool vec = dt != NPAS_F32 && C % 8 == 0;
    if (vec && (stride == 1 || stride == 2)) {
        const uint32_t CV = (uint32_t)C / 8, nyb = (uint32_t)((Ho + kDwRows - 1) / kDwRows);
        const double threads = (double)N * nyb * Wo * CV;
        // the index decode divides by CV, Wo and nyb with 32-bit reciprocals: exact while index * divisor < 2^32
        if (threads * std::max({CV, (uint32_t)Wo, nyb}) < 4294967296.0) {
            DwArgs a{x, y, w, bias, residual, N, H, W, C, Ho, Wo, act, CV, nyb, (uint32_t)threads,
                     magic32(CV), magic32((uint32_t)Wo), magic32(nyb)};
            const unsigned grid = (a.total + 255u) / 256u;
            if (dt == NPAS_BF16) {
#define NPAS_DWR(DT_)                                                                                                           \
    do {                                                                                                                         \
        const bool hs = a.act == NPAS_ACT_HARDSWISH;                                                                            \
        if (stride == 1 && hs) hipLaunchKernelGGL((depthwise3x3_rows_kernel<DT_, 1, true>), dim3(grid), dim3(256), 0, st, a);   \
        else if (stride == 1) hipLaunchKernelGGL((depthwise3x3_rows_kernel<DT_, 1, false>), dim3(grid), dim3(256), 0, st, a);   \
        else if (hs) hipLaunchKernelGGL((depthwise3x3_rows_kernel<DT_, 2, true>), dim3(grid), dim3(256), 0, st, a);            \
        else hipLaunchKernelGGL((depthwise3x3_rows_kernel<DT_, 2, false>), dim3(grid), dim3(256), 0, st, a);                   \
    } while (0)
                NPAS_DWR(NPAS_BF16);
            } else {
                NPAS_DWR(NPAS_F16);
#undef NPAS_DWR
            }
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) {
                set_error("depthwise3x3_rows launch failed: %s", hipGetErrorString(e));
                return NPAS_E_HIP;
            }
            return NPAS_OK;
        }
    }
    const size_t total = (size_t)N * Ho * Wo * (vec ? C / 8 : C);
    const unsigned grid = (unsigned)std::min<size_t>((total + 255) / 256, 256 * 32);
#define NPAS_DW(DT, V) hipLaunchKernelGGL((depthwise3x3_kernel<DT, V>), dim3(grid), dim3(256), 0, st, x, y, w, bias, residual, N, H, W, C, Ho, Wo, stride, act)
    if (dt == NPAS_BF16) {
        if (vec) NPAS_DW(NPAS_BF16, 8);
        else NPAS_DW(NPAS_BF16, 1);
    } else if (dt == NPAS_F16) {
        if (vec) NPAS_DW(NPAS_F16, 8);
        else NPAS_DW(NPAS_F16, 1);
    } else NPAS_DW(NPAS_F32, 1);
#undef NPAS_DW
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("depthwise3x3 launch failed: %s", hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    return NPAS_OK;
}

} // namespace npas
