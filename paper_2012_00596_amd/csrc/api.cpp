// C-ABI run calls of libnpas: launch planning, single layers, glue layers and
// the stack runner.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <memory>

#include "npas_internal.h"

namespace npas {

static uint32_t magic_div(uint32_t d) { return d <= 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); }

static const size_t kLdsBudget = 64 * 1024;

// Chooses the output tile of one launch.  A workgroup owns TH x TW output pixels
// of one image (at most 128 = 8 MFMA column blocks) and stages the matching
// input patch; candidates are scored by how much of the MFMA columns and of the
// tile grid do useful work, then by halo overhead.
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
    g.pitch = (d.CC * 2 + 15) / 16 * 16 + 8;
    g.koff_cap = std::min(512, std::max(32, d.max_list));
    const size_t koff_bytes = (size_t)4 * g.koff_cap * 4;

    double best = -1e30;
    bool found = false;
    for (int TW = 1; TW <= std::min(g.Wo, 128); ++TW)
        for (int TH = 1; TH <= std::min(g.Ho, 128 / TW); ++TH) {
            int PH = pointwise ? TH : (TH - 1) * stride + p->KH;
            int PW = pointwise ? TW : (TW - 1) * stride + p->KW;
            size_t lds = ((size_t)PH * PW * g.pitch + 15) / 16 * 16 + koff_bytes;
            if (lds > kLdsBudget) continue;
            int used_cols = TH * TW > 64 ? 128 : 64; // kernel instances walk 4 or 8 column blocks
            double cover = (double)g.Ho * g.Wo /
                           ((double)((g.Ho + TH - 1) / TH) * ((g.Wo + TW - 1) / TW) * used_cols);
            double halo = (double)PH * PW / ((double)TH * TW);
            double score = cover - 0.05 * halo + 0.1 * (used_cols / 128.0);
            if (score > best) {
                best = score;
                found = true;
                g.TH = TH; g.TW = TW; g.PH = PH; g.PW = PW;
            }
        }
    if (!found) {
        set_error("no output tile fits in LDS (kernel %dx%d stride %d)", p->KH, p->KW, stride);
        return NPAS_E_SHAPE;
    }
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

static int check_run(const npas_packed *p, const void *x, void *y, int N, int H, int W, int stride, int pad)
{
    if (!p || !x || !y) {
        set_error("NULL argument (handle=%p x_dev=%p y_dev=%p)", (const void *)p, x, y);
        return NPAS_E_NULL;
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

int run_conv(const npas_packed *p, const ConvPlan *plan, const void *x, void *y, int N, int H, int W, int stride,
             int pad, const void *bias, const void *residual, int act, void *stream)
{
    if (act != NPAS_ACT_NONE && act != NPAS_ACT_RELU && act != NPAS_ACT_RELU6) {
        set_error("unknown activation %d", act);
        return NPAS_E_SHAPE;
    }
    if (p->fmt.variant == V_VALU_F32) {
        ConvValuArgs a;
        a.x = (const float *)x; a.y = (float *)y; a.residual = (const float *)residual; a.bias = (const float *)bias;
        a.vg_ptr = p->dev.vg_ptr; a.vg_f0 = p->dev.vg_f0; a.vkent = p->dev.vkent; a.vw = p->dev.vw;
        a.nvg = p->fmt.nvg; a.VB = p->fmt.VB;
        a.N = N; a.H = H; a.W = W; a.C = p->C; a.F = p->F;
        a.Ho = (H + 2 * pad - p->KH) / stride + 1; a.Wo = (W + 2 * pad - p->KW) / stride + 1;
        a.KH = p->KH; a.KW = p->KW; a.stride = stride; a.pad = pad; a.act = act;
        return launch_conv_valu(a, stream);
    }
    ConvPlan local;
    if (!plan) {
        int rc = plan_conv(p, N, H, W, stride, pad, &local);
        if (rc) return rc;
        plan = &local;
    }
    ConvMfmaArgs a;
    a.x = x; a.y = y; a.residual = residual; a.bias = (const float *)bias;
    a.tc_ptr = p->dev.tc_ptr; a.kent = p->dev.kent; a.wfrag = p->dev.wfrag;
    a.CC = p->fmt.CC; a.nchunks = p->fmt.nchunks; a.ntiles = p->fmt.ntiles;
    a.g = plan->g;
    a.g.act = act;
    return launch_conv_mfma(p->dtype, a, plan->grid, plan->lds_bytes, stream);
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
    };
    std::vector<Node> nodes;
    int H = 0, W = 0, C = 0, dtype = 0;
    unsigned flags = 0;
    // per-tensor placement for a given N is computed on the fly (sizes scale with N)
    std::vector<int> last_use; // last layer reading tensor t
};

namespace npas {

static size_t tensor_elems_per_image(const npas_stack *s, int t)
{
    if (t == 0) return (size_t)s->H * s->W * s->C;
    const npas_stack::Node &n = s->nodes[t - 1];
    return (size_t)n.Ho * n.Wo * n.F;
}

// Greedy first-fit placement of the intermediate tensors (1 .. n-1) into the
// workspace; a tensor's slot is free again after its last reader has run.
// Returns total bytes; offsets[t] for intermediates.
static size_t place_tensors(const npas_stack *s, int N, std::vector<size_t> *offsets)
{
    const int nt = (int)s->nodes.size() + 1;
    std::vector<size_t> off(nt, 0), sz(nt, 0);
    struct Live { size_t off, sz; int until; };
    std::vector<Live> live;
    size_t total = 0;
    const int esz = dtype_size(s->dtype);
    for (int t = 1; t < nt - 1; ++t) { // tensor t is written by layer t-1
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

extern "C" {

int npas_conv2d_sparse(const npas_packed *p, const void *x_dev, void *y_dev, int N, int H, int W, int stride,
                       int pad, const void *bias_dev, const void *residual_dev, npas_act act, void *hip_stream)
{
    int rc = check_run(p, x_dev, y_dev, N, H, W, stride, pad);
    if (rc) return rc;
    return run_conv(p, nullptr, x_dev, y_dev, N, H, W, stride, pad, bias_dev, residual_dev, act, hip_stream);
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
        if (pruned && !d.packed) {
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
        if (pruned && d.packed->dtype != s->dtype) {
            set_error("layer %d: storage type %d differs from the stack's %d", i, d.packed->dtype, s->dtype);
            return NPAS_E_DTYPE;
        }
        if (d.res >= 0) {
            const Dim r = dims[d.res];
            if (d.kind != NPAS_LAYER_CONV || r.H != nd.Ho || r.W != nd.Wo || r.C != nd.F) {
                set_error("layer %d: residual tensor %d has the wrong shape", i, d.res);
                return NPAS_E_SHAPE;
            }
            s->last_use[d.res] = i;
        }
        s->last_use[d.src] = i;
        dims[i + 1] = {nd.Ho, nd.Wo, nd.F};
        s->nodes.push_back(nd);
    }
    *out = s.release();
    return NPAS_OK;
}

size_t npas_stack_workspace_bytes(const npas_stack *s, int N)
{
    if (!s || N <= 0) return 0;
    return place_tensors(s, N, nullptr);
}

int npas_stack_num_launches(const npas_stack *s) { return s ? (int)s->nodes.size() : 0; }

int npas_run_stack(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *workspace_dev,
                   size_t workspace_bytes, void *hip_stream)
{
    if (!s || !x_dev || !y_dev) {
        set_error("NULL argument");
        return NPAS_E_NULL;
    }
    if (N <= 0) {
        set_error("bad batch %d", N);
        return NPAS_E_SHAPE;
    }
    std::vector<size_t> off;
    size_t need = place_tensors(s, N, &off);
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
        const void *x = tensor(n.d.src);
        void *y = tensor(i + 1);
        int rc = NPAS_OK;
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

void npas_stack_free(npas_stack *s) { delete s; }

} // extern "C"
