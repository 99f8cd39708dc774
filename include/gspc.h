/*
 * gspc.h - C ABI of the MI355X (gfx950) grouped-convolution library.
 *
 * The library computes the forward grouped 2-D convolution G(g) of
 * arXiv 2006.09791 ("Optimizing Grouped Convolutions on Edge Devices"):
 * NCHW tensors in row-major order, g groups, filter oc reading only the
 * Cin/g input channels of its group (Section II, Fig. 2; shapes as in
 * Section III-B: input N x Cin x H x W, kernels Cout x Cin/g x KH x KW,
 * output N x Cout x Hout x Wout).  The paper's four GSPC stages map onto
 * this boundary as follows:
 *   stage 1 (kernel reshape, done ahead of time)  -> gspc_pack_weights
 *   stage 2 (input reshape)  -> fused into the convolution kernels' LDS
 *                               staging; gspc_pack_input_bf16 is the only
 *                               stand-alone input pass (a dtype cast)
 *   stage 3 (convolution)    -> gspc_conv2d_grouped
 *   stage 4 (output reshape) -> fused away: kernels store NCHW directly
 * and gspc_run_layer_chain runs whole grouped networks (Section IV-A).
 *
 * Conventions
 *   - Every pointer marked "dev" is device memory owned by the caller; the
 *     library never allocates or frees device memory and never synchronises
 *     the device unless stated.  Work is enqueued on the stream last given to
 *     gspc_set_stream by the calling thread (default: the null stream).
 *   - Square stride, symmetric zero padding, dilation 1, no bias.
 *     Hout = floor((H + 2*pad - KH) / stride) + 1, Wout likewise.
 *   - Cin and Cout must be divisible by groups (Section III-B).
 *   - All entry points returning int return GSPC_OK (0) or a negative error
 *     code.  Argument errors are detected on the host before any GPU work is
 *     issued, so no partial result is written.  gspc_last_error() describes
 *     the calling thread's most recent failure.
 *   - Input and output buffers must not overlap.
 */
#ifndef GSPC_H
#define GSPC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GSPC_OK = 0,
    GSPC_ERR_NULL = -1,     /* a required pointer is NULL */
    GSPC_ERR_DIM = -2,      /* non-positive dimension, negative pad, Hout or Wout <= 0 */
    GSPC_ERR_GROUPS = -3,   /* groups <= 0, or Cin or Cout not divisible by groups */
    GSPC_ERR_DTYPE = -4,    /* unknown element type */
    GSPC_ERR_MISMATCH = -5, /* call arguments disagree with the packed-weight handle */
    GSPC_ERR_SPACE = -6,    /* a caller-provided buffer is too small */
    GSPC_ERR_HIP = -7,      /* the HIP runtime reported a failure (launch, no device) */
    GSPC_ERR_ARG = -8       /* any other invalid argument (bad op code, buffer index, ...) */
};

/* Element type of the input tensor and of the packed weights.  The output is
 * always fp32 and accumulation is always fp32. */
enum { GSPC_F32 = 0, GSPC_BF16 = 1 };

/* Kernel families (for gspc_force_path / gspc_last_path). */
enum { GSPC_PATH_AUTO = -1, GSPC_PATH_DIRECT = 0, GSPC_PATH_MFMA = 1 };

/* Host-side descriptor of one layer's packed weights.  It records the layer's
 * (Cin, Cout, KH, KW, groups, dtype), the layout chosen and the address of the
 * caller-owned device bytes; it owns no device memory. */
typedef struct gspc_packed gspc_packed_t;

int gspc_version(void);

/* Selects the HIP stream (a hipStream_t passed as void*) used by subsequent
 * calls from this thread.  NULL selects the null stream. */
int gspc_set_stream(void *hip_stream);

/* Text of the calling thread's most recent error ("" if none). */
const char *gspc_last_error(void);

/* Output size of a convolution / pooling window.  GSPC_ERR_DIM if it is <= 0. */
int gspc_output_dims(int H, int W, int KH, int KW, int stride, int pad,
                     int *Hout, int *Wout);

/* MAC count of one layer, Eq. 2 of the paper:
 * N*Cin*Cout*KH*KW*Hout*Wout / groups.  0 on invalid arguments. */
uint64_t gspc_layer_macs(int N, int Cin, int Cout, int KH, int KW, int Hout,
                         int Wout, int groups);

/* ---- stage 1: kernel reshape ------------------------------------------- */

/* Bytes of device memory that gspc_pack_weights needs for this layer
 * (0 on invalid arguments). */
size_t gspc_packed_weight_bytes(int Cin, int Cout, int KH, int KW, int groups,
                                int dtype);

/* Reorders the kernels W [Cout][Cin/g][KH][KW] (dev, fp32) into the
 * group-blocked, tile-padded operand layouts the convolution kernels read
 * (the counterpart of the paper's 7-D W' of Section III-B, with the tile
 * sizes fixed by the matrix-core tile instead of T_O / T_I).  Padding lanes
 * are zero.  With dtype GSPC_BF16 the values are rounded to bf16
 * (nearest-even) on the way.  packed_dev (dev, packed_bytes >=
 * gspc_packed_weight_bytes(...), 256-byte aligned) is caller-owned and must
 * outlive the handle; *out receives a host descriptor to be released with
 * gspc_packed_free.  Meant to run once per layer, ahead of time. */
int gspc_pack_weights(const void *weight_dev, int Cin, int Cout, int KH, int KW,
                      int groups, int dtype, void *packed_dev,
                      size_t packed_bytes, gspc_packed_t **out);

/* Inverse of the reorder: writes W [Cout][Cin/g][KH][KW] (dev, fp32) back from
 * a packed buffer (values are the bf16-rounded ones for GSPC_BF16 handles).
 * which = GSPC_PATH_DIRECT or GSPC_PATH_MFMA selects the section to read;
 * GSPC_ERR_ARG if the handle holds no such section. */
int gspc_unpack_weights(const gspc_packed_t *packed, int which, void *weight_dev);

/* Releases the host descriptor only (NULL is ignored). */
void gspc_packed_free(gspc_packed_t *packed);

/* Reports the handle's fields; any output pointer may be NULL.
 * *has_mfma is 1 when a matrix-core operand section was packed. */
int gspc_packed_info(const gspc_packed_t *packed, int *Cin, int *Cout, int *KH,
                     int *KW, int *groups, int *dtype, int *has_mfma);

/* ---- input cast (only stand-alone input pass) --------------------------- */

/* fp32 -> bf16 (nearest-even) over count elements; in_dev fp32, out_dev
 * 2-byte elements.  Used to prepare bf16 activations for GSPC_BF16 layers. */
int gspc_pack_input_bf16(const void *in_dev, size_t count, void *out_dev);

/* ---- stages 2-4 fused: the convolution ---------------------------------- */

/* output[n][oc][oh][ow] = sum over c < Cin/g, kh < KH, kw < KW of
 *   Xz[n][j*Cin/g + c][oh*stride - pad + kh][ow*stride - pad + kw] * W[oc][c][kh][kw]
 * with j = oc / (Cout/g) and Xz the input extended by zeros (convolution stage
 * of Algorithm 1, no kernel flip).
 *   input  : dev, [N][Cin][H][W], fp32 or bf16 as recorded in packed_weight
 *   output : dev, fp32 [N][Cout][Hout][Wout], fully overwritten
 * Both pointers must be 16-byte aligned (GSPC_ERR_ARG otherwise): the kernels
 * move 16 bytes per lane wherever the row width allows.
 * (Cin, Cout, KH, KW, groups) must equal those of the handle
 * (GSPC_ERR_MISMATCH otherwise).  Asynchronous on the selected stream. */
int gspc_conv2d_grouped(const void *input, const gspc_packed_t *packed_weight,
                        int N, int Cin, int H, int W, int Cout, int KH, int KW,
                        int stride, int pad, int groups, void *output);

/* Testing / tuning aid: force the kernel family used by subsequent
 * convolutions of this thread (GSPC_PATH_AUTO restores the dispatcher).  A
 * forced family that cannot run a given layer yields GSPC_ERR_ARG. */
int gspc_force_path(int path);

/* Family used by this thread's most recent convolution, and its kernel's name. */
int gspc_last_path(void);
const char *gspc_last_kernel(void);

/* ---- layer chains -------------------------------------------------------- */

enum { GSPC_OP_CONV = 0, GSPC_OP_MAXPOOL = 1, GSPC_OP_ADD = 2, GSPC_OP_RELU = 3 };
enum { GSPC_FLAG_RELU = 1 }; /* clamp the result of a CONV / ADD at zero */

/* One step of a network.  src, src2 and dst index the caller's buffer table.
 *   CONV    : dst = conv(src) [+ src2 if src2 >= 0] [then ReLU]; w required
 *   MAXPOOL : dst = KH x KW max pooling of src (window clipped at the border)
 *   ADD     : dst = src + src2 [then ReLU], N*Cin*H*W elements
 *   RELU    : dst = max(src, 0), N*Cin*H*W elements (dst may equal src)
 * For ADD / RELU / MAXPOOL the tensors are fp32 [N][Cin][H][W]. */
typedef struct gspc_layer {
    int op;
    int src, src2, dst;
    int N, Cin, H, W, Cout, KH, KW, stride, pad, groups;
    int flags;
    const gspc_packed_t *w;
} gspc_layer_t;

/* Layer chains without per-layer timing are, by default, recorded into a HIP
 * graph on first use (keyed by the layer list, the buffer addresses and the
 * stream) and replayed on later calls; this needs a stream other than the null
 * stream and is skipped while the caller is itself capturing the stream.  The
 * recorded graphs belong to the calling thread; gspc_set_graph_mode(0) turns
 * the feature off and releases them, gspc_set_graph_mode(1) turns it back on. */
int gspc_set_graph_mode(int on);

/* Depth fusion of layer chains (Section II, Fig. 2: a grouped convolution only
 * mixes the channels of one group; Section III-A: groups are independent).  By default gspc_run_layer_chain evaluates a
 * run of consecutive fp32 CONV steps that share N, C, H, W and groups >= 2,
 * with 3x3 kernels, stride 1, pad 1, Cin = Cout and at most 32 channels per
 * group, in one kernel per run: one workgroup per (image, group) keeps the
 * activations of the run in on-chip memory.  Every buffer ends up with exactly
 * the contents the step-by-step execution leaves in it (the last value
 * written to it), up to floating-point summation order.  gspc_set_chain_fusion(0)
 * turns the feature off for the calling thread, (1) back on.  Runs with
 * per-layer timing are never fused. */
int gspc_set_chain_fusion(int on);

/* Winograd F(2x2, 3x3) evaluation (the grouped Winograd convolution that Section VI
 * of the paper leaves as future work).  fp32 3x3, stride-1, pad-1 layers with at
 * least 12 filters and a multiple of 4 (at least 8) channels per group can be
 * evaluated through the minimal-filtering identity
 * Y = A^T [sum_c (G g G^T) .* (B^T d B)] A: 16 instead of 36 multiplications per
 * channel and 2x2 outputs.  The result differs from the direct sum by rounding only
 * (fp32 throughout; about 1e-6 of sum |x||w| per output), but is not bit-identical
 * to it; since the input transform forms differences of inputs, an infinite input
 * can give NaN where the direct sum gives an infinity.  on < 0 (the default): used for such a layer when the launch is large enough
 * to fill the GPU, where it is the faster method; on = 0: never (every layer is the
 * direct sum); on > 0: for every such layer.  Per calling thread.  The environment
 * variable GSPC_WINOGRAD=0|1 sets the initial mode of every thread. */
int gspc_set_winograd(int on);

/* Runs the steps in order on the selected stream.  act_bufs[i] (dev) holds
 * act_bytes[i] bytes; every step is validated against those sizes before
 * anything is launched (GSPC_ERR_SPACE / GSPC_ERR_ARG); the buffers must be
 * 16-byte aligned (GSPC_ERR_ARG).  A CONV whose handle
 * is GSPC_BF16 reads a bf16 src; every dst is fp32.  If per_layer_ms is not
 * NULL it receives n_layers elapsed times measured with HIP events, and the
 * call then waits for the stream to drain; otherwise it is asynchronous. */
int gspc_run_layer_chain(const gspc_layer_t *layers, int n_layers,
                         void *const *act_bufs, const size_t *act_bytes,
                         int n_bufs, float *per_layer_ms);

#ifdef __cplusplus
}
#endif
#endif /* GSPC_H */
