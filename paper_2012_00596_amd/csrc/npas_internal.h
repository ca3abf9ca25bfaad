// Internal structures of libnpas: the packed-layer handle (canonical compact
// form + device execution format) and the kernel argument blocks.
#pragma once
#include <cstddef>
#include <cstdint>
#include <array>
#include <memory>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "../../include/npas.h"

namespace npas {

void set_error(const char *fmt, ...);

inline int dtype_size(int dt) { return dt == NPAS_F32 ? 4 : 2; }

// Testing switches (NPAS_FORCE_VARIANT / NPAS_NO_BALANCE): read from the environment once, at load;
// npas_debug_set_switches replaces them.
enum ForceVariant { FV_NONE = 0, FV_GATHER, FV_SLAB, FV_NORING, FV_NOSMALLC, FV_SPATIAL, FV_NOSPATIAL2, FV_SMALLM,
                    FV_RESIDENT, FV_NORESIDENT, FV_NOFCGATHER, FV_VALU };
struct Switches {
    int force = FV_NONE;
    bool no_balance = false;
};
const Switches &switches();
inline bool valid_act(int act) { return act >= NPAS_ACT_NONE && act <= NPAS_ACT_HARDSWISH; }

// Kernel variants a packed layer can be executed with.
enum Variant {
    V_VALU_F32 = 0,    // fp32 storage: one thread per (pixel, filter sub-group), scalar-broadcast weights
    V_MFMA_GATHER = 1, // 16-bit storage: 16-filter tiles, element-gathered activations, MFMA 16x16x32
    V_MFMA_SLAB = 2,   // 16-bit storage: 16*NT-filter super-tiles, 8-channel slabs gathered with one 16-byte LDS read
    V_DEPTHWISE = 3,   // depthwise 3x3: weights tap-major [9][C] in the storage type (wfrag for 16-bit, vw for fp32)
};

// ---- device execution format for V_MFMA_GATHER -------------------------------
// Filters are cut into tiles of 16 (MFMA rows), channels into chunks of CC.
// For tile t and chunk cc the list kent[tc_ptr[t*nchunks+cc] .. tc_ptr[..+1])
// holds every (kh, kw, c) position of that chunk kept by ANY filter of the tile
// (the union of the tile's filter groups), tap-major then channel, padded to a
// multiple of 32 with copies of entry 0 whose weights are zero.
//   entry = kh << 24 | kw << 16 | (c - cc*CC)
// wfrag holds, per 32 entries, the MFMA A-operand image: 64 lanes x 8 values,
// lane = 16*q + r holds W[filter 16t + r][entries 8q .. 8q+7] (zero where that
// filter does not keep the position).
//
// ---- device execution format for V_MFMA_SLAB ---------------------------------
// Same arrays, coarser units.  Filters are cut into super-tiles of 16*NT (one wave
// owns a super-tile and reuses every gathered activation fragment for its NT MFMA
// row tiles).  A list entry is a slab: 8 consecutive channels (c multiple of 8) at
// one tap, kept if ANY filter of the super-tile keeps ANY of its 8 weights.
// Lists are padded to a multiple of 4 slabs (one 32-deep MFMA step).  wfrag holds
// per step and per row tile j < NT the A-operand image
//   [(step*NT + j)][lane = 16*q + r][i] = W[filter 16*(st*NT + j) + r][slab 4*step + q, channel c + i].
// `ntiles` counts super-tiles; tc_ptr is in slabs.
//
// ---- device execution format for V_VALU_F32 ----------------------------------
// Filter groups are cut into sub-groups of VB (<= 8) filters that share the
// group's list.  vg_ptr[v] .. vg_ptr[v+1] indexes vkent (same entry coding with
// the absolute channel) and vw[entry][VB] (fp32).  vg_f0[v] = first filter.
struct DeviceFormat {
    int variant = -1;
    // MFMA gather
    int CC = 0, nchunks = 0, ntiles = 0, NT = 1;
    std::vector<int32_t> tc_ptr;
    std::vector<uint32_t> kent;
    std::vector<uint16_t> wfrag;
    // VALU f32
    int VB = 0, nvg = 0;
    std::vector<int32_t> vg_ptr, vg_f0;
    std::vector<uint32_t> vkent;
    std::vector<float> vw;
    int max_list = 0; // longest per-(tile,chunk) list, entries
    double density = 1.0; // kept share of a 16-filter tile's (channel, tap) positions, union over its groups
};

// ---- ring format: extra execution format of 1x1 layers with C % 64 == 0 ---------
// (also built for k x k layers with C % 64 == 0, which run it at stride 1.)
// Filters in blocks of 128, channels in chunks of 64, taps kh*KW + kw; every (block,
// chunk, tap) present: the kernels walk them in that order, one ring stage each
// (rg_ptr / rg_chunk record the chunk order for inspection).  Per (block, chunk, tap) wimg
// holds 16 MFMA operand images of 1 KB: image step*8 + tile, lane 16*q + r, value i =
// W[128 fb + 64 (tile / 4) + 4 r + tile % 4][64 chunk + 32 step + 8 q + i][tap] (zero where pruned
// or past F): used as the column operand, the four tiles of a 64-filter half give every result
// column four consecutive filters.
struct RingFormat {
    bool present = false;
    int nfb = 0, taps = 1;
    std::vector<int32_t> rg_ptr;
    std::vector<uint32_t> rg_chunk;
    std::vector<uint16_t> wimg;
};

// ---- small-channel format: k x k layers with fewer than 8 input channels (an image stem), at
// most 64 filters and C*KH*KW <= 160.  The whole reduction, k = (kh*KW + kw)*C + c, is padded to
// nsteps * 32; wimg holds per step four column-operand images of 1 KB: image step*4 + j, lane
// 16*q + r, value i = W[4 r + j][k = 32 step + 8 q + i] (zero where pruned, past F or past K).
struct SmallCFormat {
    bool present = false;
    int nsteps = 0;
    std::vector<uint16_t> wimg;
};

// ---- exact-list format of sparse 1x1 / FC layers (fc_gather_mfma): per 16-filter tile the list of input channels
// kept by ANY filter of the tile, over all of C, ascending, padded to a multiple of 32 with copies of channel 0 whose
// weights are zero.  With 16-row blocks (the block-based FC scheme) a tile is one block row and the list is exactly
// the block's kept columns: the shared positions become the K dimension of a dense 16 x K sub-GEMM.
//   tptr[t] .. tptr[t+1]   the tile's 32-entry steps
//   koff[step][32]         byte offset (2 * channel) of each entry in a staged activation row
//   wimg[step][lane][8]    MFMA A-operand image: lane = 16 q + r holds W[16 t + r][entries 8 q .. 8 q + 7]
struct FcFormat {
    bool present = false;
    int ntiles = 0, max_steps = 0;
    std::vector<int32_t> tptr;
    std::vector<uint16_t> koff;
    std::vector<uint16_t> wimg;
};

// ---- lane-split format of fp32 layers (conv_wave_f32): the canonical group lists, each padded to a multiple of
// 8 entries (entry coding as vkent, weight rows [entry][VB] as vw; padding entries carry zero weights and repeat the
// group's first position, or position 0 of an empty group).  wg_ptr[v] .. wg_ptr[v+1] in entries.
struct WaveF32Format {
    bool present = false;
    std::vector<int32_t> wg_ptr;
    std::vector<uint32_t> kent;
    std::vector<float> w;
};

struct DeviceCopy {
    int device = -1;
    void *blob = nullptr; // one allocation holding everything below
    size_t bytes = 0;
    const int32_t *tc_ptr = nullptr;
    const uint32_t *kent = nullptr;
    const void *wfrag = nullptr;
    const int32_t *vg_ptr = nullptr, *vg_f0 = nullptr;
    const uint32_t *vkent = nullptr;
    const float *vw = nullptr;
    const int32_t *rg_ptr = nullptr;
    const uint32_t *rg_chunk = nullptr;
    const void *wimg = nullptr;
    const void *scimg = nullptr; // small-channel images
    const int32_t *fc_tptr = nullptr; // exact-list format
    const uint16_t *fc_koff = nullptr;
    const void *fc_wimg = nullptr;
    const int32_t *wv_ptr = nullptr;  // lane-split fp32 format
    const uint32_t *wv_kent = nullptr;
    const float *wv_w = nullptr;
    const void *zeros = nullptr; // 256 bytes of zeros
};

struct ConvPlan; // host-side plan of one conv launch, defined below

} // namespace npas

struct npas_packed {
    int scheme = 0, dtype = 0;
    int F = 0, C = 0, KH = 0, KW = 0, Bf = 0, Bc = 0, G = 0;
    // canonical compact form
    std::vector<int32_t> grp_ptr, k_pos;
    std::vector<uint8_t> w_compact; // storage type, [K_total][Bf]
    int n_pat = 0;
    std::vector<uint8_t> library, pat_id, w4;
    // execution format
    npas::DeviceFormat fmt;
    npas::RingFormat ring;
    npas::SmallCFormat smallc;
    npas::FcFormat fc;
    npas::WaveF32Format wavef;
    npas::DeviceCopy dev;
    // launch plans already computed for this layer, by geometry (filled by the run calls)
    mutable std::mutex plan_mu;
    mutable std::vector<std::pair<std::array<int, 5>, std::shared_ptr<const npas::ConvPlan>>> plans;
};

namespace npas {

// ---- kernel argument blocks (passed by value) ---------------------------------
struct ConvGeom {
    int N, H, W, C, F, Ho, Wo;
    int KH, KW, stride, pad;
    int TH, TW;           // output tile (TH*TW <= 16*S pixels)
    int tilesY, tilesX;   // tiles per image
    int PH, PW;           // LDS patch in pixels
    int pstep;            // input step between patch pixels (stride for 1x1, else 1)
    int lstep;            // patch step between neighbouring output pixels (1 for 1x1, else stride)
    int pitch;            // LDS bytes per patch pixel
    int act;
    int nfsplit;          // filter-tile splits (grid = pixel tiles x nfsplit)
    int tiles_per_split;  // filter tiles one workgroup walks through
    int koff_cap;         // per-wave capacity of the offset table, entries
    uint32_t div_tw, div_pw, div_vec, div_pitch; // magic reciprocals (see fastdiv)
    int vec;              // 1: 16-byte staging path (C and CC multiples of 8)
    int shape;            // slab path: workgroup shape index (see launch_slab_dt)
};

struct ConvMfmaArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const int32_t *tc_ptr;
    const uint32_t *kent;
    const void *wfrag;
    int CC, nchunks, ntiles, NT;
    ConvGeom g;
};

struct ConvValuArgs {
    const float *x;
    float *y;
    const float *residual;
    const float *bias;
    const int32_t *vg_ptr, *vg_f0;
    const uint32_t *vkent;
    const float *vw;
    int nvg, VB;
    int N, H, W, C, F, Ho, Wo, KH, KW, stride, pad, act;
};

struct SmallCArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const void *wimg;
    int N, H, W, C, F, Ho, Wo, KH, KW, stride, pad, act;
    int K, nsteps;                  // reduction length C*KH*KW and its 32-deep steps
    int TH, TW, tilesY, tilesX;     // output tile (TH*TW == 256) and tiles per image
    int PH, PW, pitch;              // LDS patch: rows, pixels per row, bytes per row
    int row2;                       // 4-byte words staged per patch row when rows are fetched as words
    uint32_t nitems;                // N * tilesY * tilesX
    uint32_t div_tw, div_kwc, div_rowlen, div_row2, div_tiles, div_tx; // fastdiv magics
    // pool != 0: a 3 x 3 / stride 2 / pad 1 max pool follows and is done in the same kernel; y is the pooled
    // tensor (N x PHo x PWo x F).  A tile is then PTH x PTW pooled pixels = (2 PTH + 1) x (2 PTW + 1) conv pixels
    // (TH x TW, at most 256) starting one conv row / column before 2 x the pooled origin.
    int pool, PTH, PTW, PHo, PWo;
    uint32_t div_ptw;
};

// k x k layer on few output pixels (small batch, small maps): see conv_smallm_mfma_kernel
struct SmallMArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const void *wimg;               // ring-format images
    int N, H, W, C, F, Ho, Wo, KH, KW, stride, pad, act;
    int M;                          // output pixels N*Ho*Wo
    int nptiles;                    // 64-pixel tiles
    int nimg;                       // 16-filter images: 8 per 128-filter block
    uint32_t div_howo, div_wo, div_kw, div_T2; // fastdiv magics (Ho*Wo, Wo, KW, 2*KH*KW)
};

struct RingArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const int32_t *rg_ptr;
    const uint32_t *rg_chunk;
    const void *wimg;
    int M;                      // output pixels N*Ho*Wo
    int C, F;
    int H, W, Ho, Wo, stride;   // input / output geometry (stride > 1: subsampled input pixels)
    int nptiles, nfb;           // pixel tiles and filter blocks of the chosen configuration
    int P;                      // pixels per tile actually used (<= the configuration's tile height): evens out the items over the workgroups
    int small;                  // 0: 256 x 128 tiles, 3-stage ring; 1: 64 x 64 tiles, 8-stage ring
    int act;
    int flat;                   // 1: stride 1, input pixel index == output pixel index
    uint32_t div_howo, div_wo;  // magic reciprocals of Ho*Wo and Wo
};

struct SpatialRingArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const void *wimg;
    const void *zeros;          // >= 16 bytes of zeros on the device (source of padding pixels)
    int N, H, W, C, F, Ho, Wo;
    int KH, KW, pad;
    int stride;                 // 1, or 2 (3 x 3, pad 1: the patch as four phase planes, PH = TH + 1, PW = TW + 1, npb per plane)
    int pg;                     // pixel groups of 64 a workgroup multiplies: 4 (256-pixel tiles) or 2 (128)
    int NI, TH, TW;             // tile: NI images x TH x TW output pixels (<= 64 pg)
    int PH, PW;                 // patch of one image of the tile
    int tilesN, tilesY, tilesX, nfb;
    int npb;                    // 1 KB blocks (8 pixels) of one patch chunk
    int depth;                  // weight stages in the LDS ring (3..6)
    int act;
    uint32_t div_tw, div_pw, div_thtw, div_phpw; // magic reciprocals
};

// Sparse 1x1 / FC layer on few pixels through the exact per-tile lists: see fc_gather_mfma_kernel
struct FcGatherArgs {
    const void *x;
    void *y;
    const void *residual;
    const float *bias;
    const int32_t *tptr;
    const uint16_t *koff;
    const void *wimg;
    int M, C, F, ntiles, act;
    int tiles_per_wg;   // filter tiles one workgroup (8 waves) walks
    int pitch;          // bytes of one staged activation row in LDS
    int H, W, Ho, Wo, stride; // geometry of a strided 1x1 layer (stride 1: M pixels, flat)
    uint32_t div_howo, div_wo;
};

// fp32 layer with the reduction of every output split over 8 lanes: see conv_wave_f32_kernel
struct WaveF32Args {
    const float *x;
    float *y;
    const float *residual;
    const float *bias;
    const int32_t *wg_ptr, *vg_f0;
    const uint32_t *kent;
    const float *w;
    int nvg, VB;
    int N, H, W, C, F, Ho, Wo, KH, KW, stride, pad, act;
};

// Host-side plan of one conv launch (tile shape, grid, LDS bytes).
struct ConvPlan {
    ConvGeom g;
    unsigned grid = 0;
    size_t lds_bytes = 0;
};

int build_device_format(npas_packed *p, const std::vector<uint8_t> &mask_full, const void *w_host);
int upload(npas_packed *p, void *hip_stream);
int plan_conv(const npas_packed *p, int N, int H, int W, int stride, int pad, ConvPlan *out);

int run_stack_impl(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *workspace_dev, size_t workspace_bytes,
                   void *hip_stream);

// launchers (kernels.hip)
int launch_conv_mfma(int dtype, int variant, const ConvMfmaArgs &a, unsigned grid, size_t lds_bytes, void *stream);
int launch_conv_valu(const ConvValuArgs &a, void *stream);
int launch_pointwise_ring(int dtype, const RingArgs &a, void *stream);
const char *route_name(const npas_packed *p, int N, int H, int W, int stride, int pad);
// Tile plan of the k x k streaming kernel (geometry fields of *a); false: use another kernel.
bool plan_spatial(const npas_packed *p, int N, int H, int W, int pad, int stride, SpatialRingArgs *a);
int launch_spatial_ring(int dtype, const SpatialRingArgs &a, void *stream);
int launch_spatial_resident(int dtype, const SpatialRingArgs &a, void *stream);
size_t spatial_resident_lds_bytes(int npb, int nst); // LDS of a launch with npb patch blocks and nst weight stages
int launch_conv_smallc(int dtype, const SmallCArgs &a, void *stream);
int launch_conv_smallm(int dtype, const SmallMArgs &a, void *stream);
int launch_fc_gather(int dtype, const FcGatherArgs &a, void *stream);
int launch_conv_wave_f32(const WaveF32Args &a, void *stream);
bool fpp_supported(int nt1, int nt2);
int launch_fused_pointwise_pair(int dtype, const void *x, void *y, const void *wblob, int M, int C1, int nt1, int F2,
                                int act1, int act2, uint32_t use0, uint32_t use1, void *stream);
size_t fused_ir_lds_bytes(int TH, int TW, int nslots, int stride);
// One launch of the fused 1x1 -> depthwise 3x3 -> 1x1 block (all pointers device memory).
struct IrLaunch {
    const void *x;
    void *y;
    const void *w1, *w3;       // operand images of the two 1x1 layers in slot order
    const uint32_t *wdw;       // depthwise weights in slot order
    const int *perm;           // intermediate channel of each slot (-1: padding)
    const float *b1, *b2, *b3; // biases in channel order, or null
    int N, H, W, C1, F3, nslots, TH, TW, stride;
    int act1, act2, act3, residual;
};
int launch_fused_inverted_residual(int dtype, const IrLaunch &l, void *stream);
int launch_depthwise3x3(int dt, const void *x, void *y, const void *w, const float *bias, const void *residual, int N, int H,
                        int W, int C, int stride, int act, void *stream);
int launch_empty(int count, void *stream);
int launch_maxpool(const void *x, void *y, int N, int H, int W, int C, int dt, void *stream);
int launch_avgpool(const void *x, void *y, int N, int H, int W, int C, int dt, void *stream);

} // namespace npas
