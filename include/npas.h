/*
 * libnpas — inference through layers pruned with NPAS's fine-grained structured
 * schemes on one AMD MI355X (gfx950).
 *
 *   block-punched pruning (CONV, any kernel size)   paper section 3, Fig. 1 (f)
 *   block-based pruning (FC)                         paper section 3, Fig. 1 (g)
 *   pattern-based pruning + kernel removal (3x3)     paper section 2.1, Fig. 1 (e)
 *
 * Pruning sets weights to zero; a pruned layer computes the masked-dense
 * result.  `pack` turns a dense weight tensor plus a 0/1 mask into a compact
 * form that lists, per group of filters, only the surviving (channel, kh, kw)
 * positions; the run calls execute that list as a gathered sub-GEMM.
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is either HOST memory (suffix _host) or DEVICE
 *     memory on the current HIP device (suffix _dev).  The caller owns all of
 *     them; the library owns only what lives inside the opaque handles.
 *   - Weights  W[F][C][KH][KW]  (filter, channel, kernel row, kernel column),
 *     row-major, in the layer's storage type.  Masks are uint8, same shape,
 *     1 = weight kept, 0 = pruned; weight values under a 0 are ignored.
 *   - Activations are NHWC, contiguous, in the same storage type as the packed
 *     weights.  16-bit layers (bf16 / fp16) accumulate in fp32 on the matrix cores;
 *     fp32 layers accumulate in fp64 (products of two fp32 values are exact there, so
 *     the stored result is the correctly rounded one).  Outputs are rounded to the
 *     storage type (round to nearest even).  bias is fp32 [F] and may be NULL.
 *   - Convolution is cross-correlation with zero padding:
 *       Y[n,y,x,f] = act(bias[f] + sum W[f,c,kh,kw] X[n, y*s+kh-p, x*s+kw-p, c] + residual[n,y,x,f])
 *       Ho = (H + 2p - KH)/s + 1.
 *   - All device work is enqueued on the caller's stream (`hip_stream` is a
 *     hipStream_t passed as void*, NULL = default stream).  Run calls neither
 *     allocate nor synchronise.  Pack calls allocate device memory for the handle,
 *     enqueue the upload on `hip_stream` and wait for it (the source is the
 *     library's own host buffer), so the handle is ready for any stream on return;
 *     on a machine without a GPU they still build the host-side compact form (so it
 *     can be exported), and run calls on such a handle fail with NPAS_E_HIP.
 *   - Every function returns 0 (NPAS_OK) or a negative npas_status;
 *     npas_last_error() gives a thread-local message for the last failure.
 *   - Activations must be finite: a stored zero weight (padding of a partial
 *     group or of a position shared with a neighbouring group) times an infinite
 *     activation would give NaN where the definition gives a finite value.
 */
#ifndef NPAS_H
#define NPAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct npas_packed npas_packed; /* one packed layer */
typedef struct npas_stack npas_stack;   /* a wired list of layers */

typedef enum { NPAS_F32 = 0, NPAS_BF16 = 1, NPAS_F16 = 2 } npas_dtype;
/* ReLU6 = min(max(v, 0), 6); hard-swish (what Phase 1 of the framework puts in place of swish,
 * section 5.1) = v * min(max(v + 3, 0), 6) / 6.  Applied after bias and residual, before rounding. */
typedef enum { NPAS_ACT_NONE = 0, NPAS_ACT_RELU = 1, NPAS_ACT_RELU6 = 2, NPAS_ACT_HARDSWISH = 3 } npas_act;
typedef enum { NPAS_SCHEME_BLOCK_PUNCHED = 0, NPAS_SCHEME_FC_BLOCK = 1, NPAS_SCHEME_PATTERN = 2,
               NPAS_SCHEME_DEPTHWISE = 3 } npas_scheme;

typedef enum {
    NPAS_OK = 0,
    NPAS_E_NULL = -1,                   /* a required pointer is NULL */
    NPAS_E_SHAPE = -2,                  /* a dimension is non-positive, inconsistent or too large */
    NPAS_E_MASK_NOT_BLOCK_UNIFORM = -3, /* mask violates the block-punched / block-based rule */
    NPAS_E_MASK_NOT_IN_LIBRARY = -4,    /* a 3x3 kernel is neither a library pattern nor removed */
    NPAS_E_DTYPE = -5,                  /* unknown storage type */
    NPAS_E_WORKSPACE = -6,              /* workspace too small or misaligned */
    NPAS_E_HIP = -7,                    /* HIP runtime error, or handle has no device copy */
    NPAS_E_MASK_VALUE = -8              /* mask holds a value other than 0 or 1 */
} npas_status;

const char *npas_last_error(void);

/* Testing aid.  The library reads two environment switches once, when it is loaded: NPAS_FORCE_VARIANT
 * (gather | slab | noring | nosmallc | spatial | nospatial2 | smallm | resident | noresident | nofcgather | valu:
 * overrides the format / kernel choice, nothing else) and NPAS_NO_BALANCE (pointwise tiles of full height).
 * This call replaces them for the process (force_variant NULL or "" = none); it must not race with pack / run calls. */
void npas_debug_set_switches(const char *force_variant, int no_balance);
/* Measurement aid: enqueues `count` launches of an empty kernel (one wave) on the stream, so that a report can
 * state the launch-to-launch floor of the machine next to the kernels' times. */
int npas_debug_launch_empty(int count, void *hip_stream);

/* ---- packing ------------------------------------------------------------- */

/* Block-punched pruning (section 3): the tensor is cut into blocks of Bf
 * consecutive filters x Bc consecutive channels (x all KH x KW taps; edge blocks
 * may be partial).  A punched (channel, kh, kw) position must be punched in every
 * filter of its block; a mask that breaks this is rejected, never repaired.
 * Bf = Bc = 1 is unstructured pruning, Bf = F and Bc = C coarse-grained
 * (section 3, "Compiler Optimizations").  On success *out owns host and device
 * copies of the compact form; release with npas_free. */
int npas_pack_block_punched(const void *w_host, const uint8_t *mask_host, int F, int C, int KH, int KW,
                            int Bf, int Bc, npas_dtype dt, void *hip_stream, npas_packed **out);

/* Block-based pruning of an FC weight matrix W[OUT][IN] (section 3): blocks of
 * Br rows x Bcol columns; inside a block whole columns and/or whole rows are
 * pruned (mask = rowkeep AND colkeep per block), anything else is rejected.
 * The handle behaves like a 1x1 convolution with F = OUT, C = IN, Bf = Br. */
int npas_pack_fc_block(const void *w_host, const uint8_t *mask_host, int OUT, int IN, int Br, int Bcol,
                       npas_dtype dt, void *hip_stream, npas_packed **out);

/* Pattern-based pruning with kernel removal (section 2.1), 3x3 only: every
 * kernel (f, c) of W[F][C][3][3] must equal one of the n_pat library patterns
 * (library_host: uint8 [n_pat][9], 0/1, tap order kh*3+kw, n_pat <= 254) or be
 * all zero (removed). */
int npas_pack_pattern(const void *w_host, const uint8_t *mask_host, int F, int C,
                      const uint8_t *library_host, int n_pat, npas_dtype dt, void *hip_stream,
                      npas_packed **out);

/* Depthwise 3x3 weights W[C][3][3]: the "3x3 DW" member of the layer cascades in the search
 * space (section 5.1.1), one 3x3 kernel per channel, not pruned.  The handle reports scheme
 * NPAS_SCHEME_DEPTHWISE with F = C; npas_packed_export returns the weights in w_compact
 * ([C][9], storage type); it runs through npas_depthwise3x3 or a DEPTHWISE3X3 stack layer. */
int npas_pack_depthwise3x3(const void *w_host, int C, npas_dtype dt, void *hip_stream, npas_packed **out);

/* info[0..15] = { scheme, dtype, F, C, KH, KW, Bf, Bc, G (filter groups),
 *                 K_total (length of k_pos), n_pat, device_ready, kernel variant,
 *                 device-format bytes, canonical compact-weight bytes, reserved }. */
int npas_packed_info(const npas_packed *p, int64_t info[16]);

/* The compact storage of a pruned layer (section 3, "Compiler Optimizations": only the weights a
 * block keeps are stored, with the positions its filters share), in one canonical order so that two
 * packers can be compared bit for bit.  Copied to caller's HOST buffers (any may be NULL):
 *   grp_ptr  int32 [G+1]        prefix sums of the per-group list lengths
 *   k_pos    int32 [K_total]    per group, ascending: (kh*KW + kw)*C + c of every
 *                               position kept by any filter of the group
 *   w_compact storage type [K_total][Bf]   weight of filter g*Bf+j at that position
 *                               (+0 where that filter's mask is 0 or past F)
 *   pattern scheme only:
 *   pat_id   uint8 [F][C]       library index (smallest match), 255 = removed
 *   w4       storage type [F][C][4]  kept weights in ascending tap order, +0 if removed
 * For the pattern scheme grp_ptr/k_pos/w_compact describe the same layer with
 * Bf = 1 (one list per filter). */
int npas_packed_export(const npas_packed *p, int32_t *grp_ptr, int32_t *k_pos, void *w_compact,
                       uint8_t *pat_id, void *w4);

void npas_free(npas_packed *p);

/* ---- running one layer ---------------------------------------------------- */

/* Inference through one pruned CONV layer (section 3, block-punched pruning, Fig. 1 (f); section 2.1,
 * pattern-based pruning, Fig. 1 (e)): the masked-dense convolution of the header comment, computed
 * from the packed form.  x_dev [N][H][W][C] -> y_dev [N][Ho][Wo][F], a packed layer of any scheme.  residual_dev (nullable) has y's shape and type and
 * is added before the activation.  Errors: NULL handle/x/y, non-positive sizes,
 * an empty output, or more than 2^31-1 elements in x or y -> NPAS_E_NULL /
 * NPAS_E_SHAPE; launch failure -> NPAS_E_HIP. */
int npas_conv2d_sparse(const npas_packed *p, const void *x_dev, void *y_dev, int N, int H, int W,
                       int stride, int pad, const void *bias_dev, const void *residual_dev,
                       npas_act act, void *hip_stream);

/* Name of the kernel npas_conv2d_sparse / npas_fc_sparse launch for this layer and geometry
 * ("conv_valu_f32", "conv_wave_f32", "conv_gather_mfma", "conv_slab_mfma", "pointwise_ring",
 * "spatial_ring", "spatial_resident", "conv_smallc_mfma", "conv_smallm_mfma", "fc_gather_mfma");
 * a static string, NULL for a NULL handle.  For reports and tests:
 * the choice depends on the packed format and on how well the problem fills the chip. */
const char *npas_conv2d_kernel_name(const npas_packed *p, int N, int H, int W, int stride, int pad);

/* Inference through one pruned FC layer (section 3, block-based pruning, Fig. 1 (g)):
 *   y[b,o] = act(bias[o] + sum over the columns i the block of row o keeps of W[o,i] x[b,i]).
 * x_dev [B][IN] -> y_dev [B][OUT]; the handle comes from npas_pack_fc_block (or any 1x1 packed layer). */
int npas_fc_sparse(const npas_packed *p, const void *x_dev, void *y_dev, int B, const void *bias_dev,
                   npas_act act, void *hip_stream);

/* Depthwise 3x3 convolution, padding 1, stride >= 1: x_dev [N][H][W][C] -> y_dev
 * [N][(H-1)/stride+1][(W-1)/stride+1][C],
 *   y[n,oy,ox,c] = act(bias[c] + sum_{kh,kw} W[c,kh,kw] x[n, oy*stride+kh-1, ox*stride+kw-1, c] + residual),
 * out-of-range input = 0, fp32 accumulation.  bias_dev (fp32) and residual_dev (y's shape and
 * type) are nullable.  Errors as npas_conv2d_sparse; a handle of another scheme -> NPAS_E_SHAPE. */
int npas_depthwise3x3(const npas_packed *p, const void *x_dev, void *y_dev, int N, int H, int W, int stride,
                      const void *bias_dev, const void *residual_dev, npas_act act, void *hip_stream);

/* Glue layers a residual stack needs around the pruned ones (not pruned
 * themselves): 3x3 stride-2 max-pool with padding 1 (padding never wins), and
 * global average pool [N][H][W][C] -> [N][C] (fp32 mean, rounded on store). */
int npas_maxpool3x3s2(const void *x_dev, void *y_dev, int N, int H, int W, int C, npas_dtype dt,
                      void *hip_stream);
int npas_global_avgpool(const void *x_dev, void *y_dev, int N, int H, int W, int C, npas_dtype dt,
                        void *hip_stream);

/* ---- running a stack ------------------------------------------------------ */

typedef enum { NPAS_LAYER_CONV = 0, NPAS_LAYER_FC = 1, NPAS_LAYER_MAXPOOL3X3S2 = 2,
               NPAS_LAYER_GLOBAL_AVGPOOL = 3, NPAS_LAYER_DEPTHWISE3X3 = 4 } npas_layer_kind;

/* A network is a sequence of such layers (section 5.1: per-layer filter type, scheme and rate); running
 * several as one call is where layer fusion (section 3, "Compiler Optimizations") can happen.
 * Tensor 0 is the stack input; layer i writes tensor i+1; the last layer's
 * tensor is the stack output.  `src` and `res` name earlier tensors (res = -1:
 * no residual).  `packed` must outlive the stack. */
typedef struct {
    int kind;                  /* npas_layer_kind */
    const npas_packed *packed; /* CONV / FC / DEPTHWISE3X3; NULL otherwise */
    int stride, pad;           /* CONV; DEPTHWISE3X3: stride (pad is 1) */
    int act;                   /* npas_act, CONV / FC / DEPTHWISE3X3 */
    int src;
    int res;
    const void *bias_dev;      /* nullable */
} npas_layer_desc;

enum {
    NPAS_STACK_FUSE_POINTWISE = 1,         /* allow a 1x1 -> act -> 1x1 pair to run as one kernel */
    NPAS_STACK_FUSE_INVERTED_RESIDUAL = 2, /* allow 1x1 -> depthwise 3x3 (stride 1 or 2) -> 1x1, each with or without bias, (+ block input at stride 1) to run as one kernel */
    NPAS_STACK_FUSE_CONV_MAXPOOL = 4       /* allow a conv on fewer than 8 channels (an image stem) and the max pool after it to run as one kernel */
};

/* Builds a stack for inputs of H x W x C (C is taken from the first layer).
 * Checks wiring, shapes and types (NPAS_E_SHAPE / NPAS_E_DTYPE). */
int npas_stack_create(const npas_layer_desc *layers, int n_layers, int H, int W, unsigned flags,
                      npas_stack **out);
/* Bytes of device workspace npas_run_stack needs for batch N (intermediate
 * tensors, 256-byte aligned, reused once dead). */
size_t npas_stack_workspace_bytes(const npas_stack *s, int N);
/* Runs the stack on the caller's stream: x_dev [N][H][W][C] -> y_dev (shape of
 * the last tensor).  workspace_dev must be 256-byte aligned and at least
 * npas_stack_workspace_bytes(s, N) long (NPAS_E_WORKSPACE otherwise). */
int npas_run_stack(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *workspace_dev,
                   size_t workspace_bytes, void *hip_stream);
/* npas_run_stack for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The intermediate tensors live in a device
 * array inside the library (NPAS_STATIC_WORKSPACE_BYTES on every GPU the process uses, held until it ends);
 * the call allocates nothing on host or device paths of HIP and launches the same kernels as npas_run_stack.
 * A stack that needs more workspace at batch N (npas_stack_workspace_bytes) is refused with
 * NPAS_E_WORKSPACE.  All calls on one GPU share the array: calls whose work overlaps in time on one GPU
 * (different streams, or threads) race; calls on one stream are safe.  Nothing in the array needs clearing. */
#define NPAS_STATIC_WORKSPACE_BYTES (32u << 20)
int npas_run_stack_static(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *hip_stream);
/* Number of kernels one npas_run_stack call launches (after fusion). */
int npas_stack_num_launches(const npas_stack *s);
/* For tests and reports: the launches one npas_run_stack call makes for batch N, in order, and where their
 * tensors live.  Row r of rows_host (int64 [max_rows][NPAS_DESCRIBE_COLS]) =
 *   { first layer of the launch, last layer it absorbs, input tensor, residual tensor (-1: none), output tensor,
 *     workspace offset of the input, of the residual, of the output (-1: the tensor is x_dev, -2: y_dev, -3: none),
 *     bytes of the input, of the residual, of the output }.
 * Returns the number of launches (rows beyond max_rows are not written), or a negative npas_status. */
#define NPAS_DESCRIBE_COLS 11
int npas_stack_describe(const npas_stack *s, int N, int64_t *rows_host, int max_rows);
void npas_stack_free(npas_stack *s);

#ifdef __cplusplus
}
#endif
#endif /* NPAS_H */
