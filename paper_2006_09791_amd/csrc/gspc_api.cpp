// Host side of libgspc: argument validation, kernel-family dispatch and the
// layer-chain runner.  All arithmetic happens in the HIP kernels.
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <unordered_map>
#include <vector>

#include "gspc_internal.h"

namespace {

thread_local hipStream_t t_stream = nullptr;
thread_local char t_error[512] = "";
thread_local int t_force_path = GSPC_PATH_AUTO;
thread_local int t_last_path = GSPC_PATH_AUTO;
thread_local const char *t_last_kernel = "";
thread_local int t_graph_mode = 1;
thread_local int t_fusion = 1;
thread_local int t_winograd = -2;   // -2: not yet read from the environment; -1 automatic, 0 off, 1 on

// Recorded layer chains, per thread, keyed by everything a replay depends on.
struct ChainGraph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};
thread_local std::unordered_map<uint64_t, ChainGraph> t_graphs;

void clear_graphs() {
    for (auto &kv : t_graphs) {
        (void)hipGraphExecDestroy(kv.second.exec);
        (void)hipGraphDestroy(kv.second.graph);
    }
    t_graphs.clear();
}

uint64_t fnv(uint64_t h, const void *data, size_t n) {
    const unsigned char *b = static_cast<const unsigned char *>(data);
    for (size_t i = 0; i < n; ++i) h = (h ^ b[i]) * 1099511628211ull;
    return h;
}

uint64_t chain_key(const gspc_layer_t *layers, int n_layers, void *const *bufs, int n_bufs,
                   hipStream_t stream, int force_path, int fusion) {
    uint64_t h = 1469598103934665603ull;
    for (int i = 0; i < n_layers; ++i) {
        const gspc_layer_t &L = layers[i];
        const int f[15] = {L.op, L.src, L.src2, L.dst, L.N, L.Cin, L.H, L.W, L.Cout, L.KH, L.KW,
                           L.stride, L.pad, L.groups, L.flags};
        h = fnv(h, f, sizeof(f));
        if (L.op == GSPC_OP_CONV && L.w) {
            h = fnv(h, &L.w->dev, sizeof(L.w->dev));
            h = fnv(h, &L.w->dtype, sizeof(L.w->dtype));
        }
    }
    h = fnv(h, bufs, sizeof(void *) * n_bufs);
    h = fnv(h, &stream, sizeof(stream));
    h = fnv(h, &force_path, sizeof(force_path));
    h = fnv(h, &fusion, sizeof(fusion));
    return h;
}

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_error, sizeof(t_error), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char *what) {
    return fail(GSPC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int out_dim(int in, int k, int stride, int pad) {
    long span = (long)in + 2L * pad - k;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

// Shared validation of a layer's shape arguments.
int check_shape(int Cin, int Cout, int KH, int KW, int groups) {
    if (Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0)
        return fail(GSPC_ERR_DIM, "non-positive dimension (Cin=%d Cout=%d KH=%d KW=%d)",
                    Cin, Cout, KH, KW);
    if (groups <= 0 || Cin % groups || Cout % groups)
        return fail(GSPC_ERR_GROUPS, "Cin=%d and Cout=%d must be divisible by groups=%d",
                    Cin, Cout, groups);
    return GSPC_OK;
}

bool valid_handle(const gspc_packed_t *h) {
    return h && h->magic == gspc::kPackedMagic && h->version == gspc::kVersion;
}

// Validates a convolution call and fills the kernel parameters.
int prepare_conv(const void *input, const gspc_packed_t *pw, int N, int Cin, int H,
                 int W, int Cout, int KH, int KW, int stride, int pad, int groups,
                 void *output, gspc::ConvParams *p) {
    if (!input || !pw || !output) return fail(GSPC_ERR_NULL, "null pointer argument");
    if ((reinterpret_cast<uintptr_t>(input) | reinterpret_cast<uintptr_t>(output)) & 15)
        return fail(GSPC_ERR_ARG, "input and output must be 16-byte aligned");
    if (!valid_handle(pw)) return fail(GSPC_ERR_MISMATCH, "not a packed-weight handle of this library version");
    if (N <= 0 || H <= 0 || W <= 0 || stride <= 0 || pad < 0)
        return fail(GSPC_ERR_DIM, "non-positive dimension (N=%d H=%d W=%d stride=%d pad=%d)",
                    N, H, W, stride, pad);
    int rc = check_shape(Cin, Cout, KH, KW, groups);
    if (rc) return rc;
    if (pw->Cin != Cin || pw->Cout != Cout || pw->KH != KH || pw->KW != KW ||
        pw->groups != groups)
        return fail(GSPC_ERR_MISMATCH,
                    "handle packed for (Cin=%d Cout=%d KH=%d KW=%d g=%d), called with "
                    "(Cin=%d Cout=%d KH=%d KW=%d g=%d)",
                    pw->Cin, pw->Cout, pw->KH, pw->KW, pw->groups, Cin, Cout, KH, KW, groups);
    const int Hout = out_dim(H, KH, stride, pad), Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0)
        return fail(GSPC_ERR_DIM, "kernel %dx%d does not fit the padded %dx%d input", KH, KW,
                    H + 2 * pad, W + 2 * pad);
    const double in_elems = (double)N * Cin * H * W, out_elems = (double)N * Cout * Hout * Wout;
    if (in_elems >= 2147483648.0 || out_elems >= 2147483648.0)
        return fail(GSPC_ERR_DIM, "tensor with 2^31 or more elements is not supported");
    p->x = input;
    p->wd = reinterpret_cast<const float *>(pw->dev);
    p->wm = pw->geom.mfma_bytes
                ? reinterpret_cast<const float *>(static_cast<const char *>(pw->dev) +
                                                  pw->geom.mfma_offset)
                : nullptr;
    p->wb = pw->geom.bf16_bytes ? static_cast<const char *>(pw->dev) + pw->geom.bf16_offset : nullptr;
    p->wx = pw->geom.wino_bytes
                ? reinterpret_cast<const float *>(static_cast<const char *>(pw->dev) + pw->geom.wino_offset)
                : nullptr;
    p->wr = pw->geom.row_bytes ? static_cast<const char *>(pw->dev) + pw->geom.row_offset : nullptr;
    p->y = static_cast<float *>(output);
    p->res = nullptr;
    p->N = N; p->Cin = Cin; p->H = H; p->W = W; p->Cout = Cout; p->KH = KH; p->KW = KW;
    p->H0 = H; p->W0 = W;
    p->stride = stride; p->pad = pad; p->groups = groups;
    p->CPG = Cin / groups; p->KPG = Cout / groups; p->Hout = Hout; p->Wout = Wout;
    p->KPGd = pw->geom.KPGd;
    p->relu = 0;
    p->in_bf16 = pw->dtype == GSPC_BF16;
    // A 1x1 convolution with stride 1 and no padding acts on each plane as on flat
    // memory: when the row length is not a multiple of 4 (14x14, 7x7 planes) but the
    // plane is, hand the kernels the same bytes as H' x W' with W' % 4 == 0, which
    // opens their 16-byte staging paths.  W' is the multiple-of-4 divisor of H*W that
    // fills the staging's power-of-two lane groups best (ties: the longer row).
    if (KH == 1 && KW == 1 && stride == 1 && pad == 0 && W % 4 != 0 && (H * W) % 4 == 0 && H * W <= 16384) {
        const int hw = H * W;
        int best_w = 0;
        double best_fill = 0.0;
        for (int w = 4; w <= hw && w <= 256; w += 4) {
            if (hw % w) continue;
            int lanes = 1;
            while (lanes < w / 4) lanes *= 2;
            const double fill = (double)(w / 4) / lanes;
            if (fill >= best_fill) {
                best_fill = fill;
                best_w = w;
            }
        }
        if (best_w) {
            p->W = p->Wout = best_w;
            p->H = p->Hout = hw / best_w;
        }
    } else if (KH == 1 && KW == 1 && stride == 1 && pad == 0 && H > 1 && (H * W) % 4 != 0 && H * W <= 256) {
        // Planes whose size is not a multiple of 4 (7x7, 5x5 ...): one row of H*W elements.  The plain
        // 16x16x4 kernel then stages blocks of four channels as single aligned rows.
        p->W = p->Wout = H * W;
        p->H = p->Hout = 1;
    }
    return GSPC_OK;
}

// Picks the kernel family and launches.
int dispatch_conv(const gspc::ConvParams &p, const gspc_packed_t *pw) {
    // Groups too small for a matrix-core tile: the layer as block-diagonal groups of at least four
    // channels and filters (zero weights between the original groups, Section II / Fig. 2), which the
    // 4x4x1 kernel takes; a layer with 2 channels per group then runs exactly as the one with half
    // as many groups does.
    if (pw->geom.md[0].m && t_force_path != GSPC_PATH_DIRECT && !p.in_bf16) {
        const gspc::PackGeom::MergedDirect &d = pw->geom.md[0];
        gspc::ConvParams q = p;
        q.groups = d.groups;
        q.CPG = d.CPG;
        q.KPG = d.KPG;
        q.KPGd = d.KPGd;
        q.wd = reinterpret_cast<const float *>(static_cast<const char *>(pw->dev) + d.offset);
        q.wm = nullptr;
        q.wb = nullptr;
        q.wx = nullptr;
        q.wr = nullptr;
        const gspc::PackGeom gm = gspc::merged_geom(pw->geom, 0, p.KH, p.KW);
        if (gspc::mfma_supported(q, gm)) {
            const char *name = "";
            const hipError_t e = gspc::launch_mfma(q, gm, t_stream, &name);
            if (e != hipSuccess) return hip_fail(e, "convolution launch");
            t_last_path = GSPC_PATH_MFMA;
            t_last_kernel = name;
            return GSPC_OK;
        }
    }
    const bool can_mfma = gspc::mfma_supported(p, pw->geom);
    int path = t_force_path;
    if (path == GSPC_PATH_AUTO) path = can_mfma ? GSPC_PATH_MFMA : GSPC_PATH_DIRECT;
    if (path == GSPC_PATH_MFMA && !can_mfma)
        return fail(GSPC_ERR_ARG, "matrix-core path forced but not available for this layer");
    const char *name = "";
    hipError_t e = path == GSPC_PATH_MFMA ? gspc::launch_mfma(p, pw->geom, t_stream, &name)
                                          : gspc::launch_direct(p, t_stream, &name);
    if (e != hipSuccess) return hip_fail(e, "convolution launch");
    t_last_path = path;
    t_last_kernel = name;
    return GSPC_OK;
}

}  // namespace

namespace gspc {

int winograd_mode() {
    static const char *env = std::getenv("GSPC_WINOGRAD");   // process-wide default: 0 | 1 (else automatic)
    if (t_winograd == -2) t_winograd = env ? (std::atoi(env) > 0 ? 1 : 0) : -1;
    return t_winograd;
}

PackGeom make_pack_geom(int Cin, int Cout, int KH, int KW, int groups, int dtype) {
    PackGeom g{};
    g.CPG = Cin / groups;
    g.KPG = Cout / groups;
    g.Kred = g.CPG * KH * KW;
    g.KPGd = round_up(g.KPG, 4);
    g.direct_bytes = (size_t)groups * g.Kred * g.KPGd * sizeof(float);
    if (g.KPG % 16 == 0) g.variant = kMfma16;
    else if (g.KPG % 4 == 0) g.variant = kMfma4;
    else g.variant = kMfmaNone;
    // The 16x16x4 operand section: filter tiles of 16, the last one zero-padded.  Below five
    // filters per group a tile would be more than two thirds padding: those layers stay on
    // the direct kernels.
    if (g.variant == kMfma16 || g.KPG >= 5) {
        g.ksub = 4;
        g.CPGp = round_up(g.CPG, g.ksub);
        g.ksteps = g.CPGp / g.ksub * KH * KW;
        g.mtiles = (g.KPG + 15) / 16;
        g.mfma_bytes = (size_t)groups * g.mtiles * g.ksteps * 64 * sizeof(float);
    }
    g.mfma_offset = (g.direct_bytes + 255) / 256 * 256;
    g.bf16_offset = (g.mfma_offset + g.mfma_bytes + 255) / 256 * 256;
    if (dtype == GSPC_BF16 && KH == 3 && KW == 3) {
        // 16x16x32 section: merge groups until a group has a multiple of 8 channels and of 4 filters
        // and at least 16 channels (block-diagonal weights: a half-empty filter tile and a reduction
        // of 72 padded to 96 cost more than the idle multiplications; 256 -> 256 on 14x14 at batch
        // 256, g = 32: 25.8 -> 20.5 us).  `GSPC_MERGE_B` (measurement aid) sets another width.
        static const char *menv = std::getenv("GSPC_MERGE_B");
        const int want_c = menv ? std::atoi(menv) : 16;
        int m = 1;
        while (m < 8 && groups % (2 * m) == 0 && ((g.CPG * m) % 8 || (g.KPG * m) % 4 || g.CPG * m < want_c)) m *= 2;
        if ((g.CPG * m) % 8 == 0 && (g.KPG * m) % 4 == 0) {
            g.mb = m;
            g.gb = groups / m;
            g.CPGb = g.CPG * m;
            g.KPGb = g.KPG * m;
            g.ckb = g.CPGb % 32 == 0 ? 32 : g.CPGb % 16 == 0 ? 16 : 8;
            g.nchunks_b = g.CPGb / g.ckb;
            g.ks_b = (9 * g.ckb / 8 + 3) / 4;
            g.mtiles_b = (g.KPGb + 15) / 16;   // filter tiles, the last one zero-padded
            g.bf16_bytes = (size_t)g.gb * g.nchunks_b * g.ks_b * g.mtiles_b * 1024;
        }
    }
    g.total_bytes = g.bf16_bytes ? g.bf16_offset + g.bf16_bytes : g.mfma_offset + g.mfma_bytes;
    if (dtype == GSPC_BF16 && KH == 3 && KW == 3) {
        // row-product section: merged groups of 8 channels (16 where a group has 16 of its own)
        int m = 1;
        while (m < 8 && groups % (2 * m) == 0 && g.CPG * m < 8) m *= 2;
        const int c = g.CPG * m, k = g.KPG * m;
        if ((c == 8 || c == 16) && k % 4 == 0 && k <= 64) {
            g.mt = m;
            g.gt = groups / m;
            g.CPGt = c;
            g.KPGt = k;
            g.row_offset = (g.total_bytes + 255) / 256 * 256;
            g.row_bytes = (size_t)g.gt * (k / 4) * 3 * (c / 4) * 1024;
            g.total_bytes = g.row_offset + g.row_bytes;
        }
    }
    if (dtype == GSPC_F32 && (Cin == 32 || Cin == 64 || Cin == 128)) {
        int m = 0;
        if (KH == 3 && KW == 3 && Cin == Cout && groups < Cin) {
            m = 1;
            while ((g.KPG * m) % 16 && groups % (2 * m) == 0) m *= 2;
            if ((g.KPG * m) % 16) m = 0;
        } else if (KH == 1 && KW == 1 && groups == 1 && Cout % 16 == 0) {
            m = 1;
        }
        if (m) {
            g.qk_m = m;
            g.qk_groups = groups / m;
            g.qk_CPG = g.CPG * m;
            g.qk_KPG = g.KPG * m;
            g.qk_offset = (g.total_bytes + 255) / 256 * 256;
            g.qk_bytes = (size_t)g.qk_groups * (g.qk_CPG / 4 * KH * KW / 4) * (g.qk_KPG / 16) * 1024;
            g.total_bytes = g.qk_offset + g.qk_bytes;
        }
    }
    if (KH == 3 && KW == 3 && g.CPG * g.KPG > 1) {
        const int lo = g.CPG < g.KPG ? g.CPG : g.KPG;
        for (int which = 0; which < 2; ++which) {
            const int target = which == 0 ? 4 : 8;
            int m = 1;
            while (lo * m < target && m < 8 && groups % (2 * m) == 0) m *= 2;
            if (m == 1 || lo * m < target || g.CPG * m > 32 || g.KPG * m > 32) continue;
            if (which == 1 && g.md[0].m == m) continue;   // the same view
            PackGeom::MergedDirect &d = g.md[which];
            d.m = m;
            d.groups = groups / m;
            d.CPG = g.CPG * m;
            d.KPG = g.KPG * m;
            d.KPGd = round_up(d.KPG, 4);
            d.offset = (g.total_bytes + 255) / 256 * 256;
            d.bytes = (size_t)d.groups * d.CPG * 9 * d.KPGd * sizeof(float);
            g.total_bytes = d.offset + d.bytes;
        }
    }
    // (the Winograd section stays the last one)
    if (dtype == GSPC_F32 && KH == 3 && KW == 3 && g.KPG >= 12 && g.CPG % 4 == 0 && g.CPG >= 8) {
        g.wino_offset = (g.total_bytes + 255) / 256 * 256;
        g.wino_bytes = (size_t)groups * (g.CPG / 4) * ((g.KPG + 15) / 16) * 4096;
        g.total_bytes = g.wino_offset + g.wino_bytes;
    }
    return g;
}

PackGeom merged_geom(const PackGeom &g, int which, int KH, int KW) {
    const PackGeom::MergedDirect &d = g.md[which];
    PackGeom v{};
    v.CPG = d.CPG;
    v.KPG = d.KPG;
    v.Kred = d.CPG * KH * KW;
    v.KPGd = d.KPGd;
    v.variant = d.KPG % 16 == 0 ? kMfma16 : d.KPG % 4 == 0 ? kMfma4 : kMfmaNone;
    v.direct_bytes = d.bytes;
    return v;
}

}  // namespace gspc

extern "C" {

int gspc_version(void) { return gspc::kVersion; }

int gspc_set_stream(void *hip_stream) {
    t_stream = static_cast<hipStream_t>(hip_stream);
    return GSPC_OK;
}

const char *gspc_last_error(void) { return t_error; }

int gspc_output_dims(int H, int W, int KH, int KW, int stride, int pad, int *Hout,
                     int *Wout) {
    if (!Hout || !Wout) return fail(GSPC_ERR_NULL, "null output pointer");
    if (H <= 0 || W <= 0 || KH <= 0 || KW <= 0 || stride <= 0 || pad < 0)
        return fail(GSPC_ERR_DIM, "non-positive dimension");
    const int ho = out_dim(H, KH, stride, pad), wo = out_dim(W, KW, stride, pad);
    if (ho <= 0 || wo <= 0) return fail(GSPC_ERR_DIM, "window does not fit the padded input");
    *Hout = ho;
    *Wout = wo;
    return GSPC_OK;
}

uint64_t gspc_layer_macs(int N, int Cin, int Cout, int KH, int KW, int Hout, int Wout,
                         int groups) {
    if (N <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0 || Hout <= 0 || Wout <= 0 ||
        groups <= 0)
        return 0;
    return (uint64_t)N * Cin * Cout * KH * KW * Hout * Wout / (uint64_t)groups;
}

size_t gspc_packed_weight_bytes(int Cin, int Cout, int KH, int KW, int groups, int dtype) {
    if (check_shape(Cin, Cout, KH, KW, groups)) return 0;
    if (dtype != GSPC_F32 && dtype != GSPC_BF16) {
        fail(GSPC_ERR_DTYPE, "unknown dtype %d", dtype);
        return 0;
    }
    return gspc::make_pack_geom(Cin, Cout, KH, KW, groups, dtype).total_bytes;
}

int gspc_pack_weights(const void *weight_dev, int Cin, int Cout, int KH, int KW, int groups,
                      int dtype, void *packed_dev, size_t packed_bytes, gspc_packed_t **out) {
    if (!weight_dev || !packed_dev || !out) return fail(GSPC_ERR_NULL, "null pointer argument");
    int rc = check_shape(Cin, Cout, KH, KW, groups);
    if (rc) return rc;
    if (dtype != GSPC_F32 && dtype != GSPC_BF16) return fail(GSPC_ERR_DTYPE, "unknown dtype %d", dtype);
    if ((double)Cout * (Cin / groups) * KH * KW >= 2147483648.0)
        return fail(GSPC_ERR_DIM, "weight tensor with 2^31 or more elements is not supported");
    const gspc::PackGeom g = gspc::make_pack_geom(Cin, Cout, KH, KW, groups, dtype);
    if (packed_bytes < g.total_bytes)
        return fail(GSPC_ERR_SPACE, "packed buffer holds %zu bytes, %zu needed", packed_bytes,
                    g.total_bytes);
    if (reinterpret_cast<uintptr_t>(packed_dev) % 256)
        return fail(GSPC_ERR_ARG, "packed buffer must be 256-byte aligned");
    gspc_packed_t *h = new (std::nothrow) gspc_packed_t;
    if (!h) return fail(GSPC_ERR_SPACE, "out of host memory");
    h->magic = gspc::kPackedMagic;
    h->version = gspc::kVersion;
    h->Cin = Cin; h->Cout = Cout; h->KH = KH; h->KW = KW; h->groups = groups; h->dtype = dtype;
    h->geom = g;
    h->dev = packed_dev;
    h->bytes = g.total_bytes;
    hipError_t e = gspc::launch_pack_weights(static_cast<const float *>(weight_dev), h, t_stream);
    if (e != hipSuccess) {
        delete h;
        return hip_fail(e, "weight pack launch");
    }
    *out = h;
    return GSPC_OK;
}

int gspc_unpack_weights(const gspc_packed_t *packed, int which, void *weight_dev) {
    if (!packed || !weight_dev) return fail(GSPC_ERR_NULL, "null pointer argument");
    if (!valid_handle(packed)) return fail(GSPC_ERR_MISMATCH, "not a packed-weight handle");
    if (which != GSPC_PATH_DIRECT && which != GSPC_PATH_MFMA)
        return fail(GSPC_ERR_ARG, "which must be GSPC_PATH_DIRECT or GSPC_PATH_MFMA");
    if (which == GSPC_PATH_MFMA && packed->geom.mfma_bytes == 0)
        return fail(GSPC_ERR_ARG, "handle holds no matrix-core section");
    hipError_t e = gspc::launch_unpack_weights(packed, which, static_cast<float *>(weight_dev), t_stream);
    if (e != hipSuccess) return hip_fail(e, "weight unpack launch");
    return GSPC_OK;
}

void gspc_packed_free(gspc_packed_t *packed) {
    if (!packed) return;
    packed->magic = 0;
    delete packed;
}

int gspc_packed_info(const gspc_packed_t *packed, int *Cin, int *Cout, int *KH, int *KW,
                     int *groups, int *dtype, int *has_mfma) {
    if (!packed) return fail(GSPC_ERR_NULL, "null handle");
    if (!valid_handle(packed)) return fail(GSPC_ERR_MISMATCH, "not a packed-weight handle");
    if (Cin) *Cin = packed->Cin;
    if (Cout) *Cout = packed->Cout;
    if (KH) *KH = packed->KH;
    if (KW) *KW = packed->KW;
    if (groups) *groups = packed->groups;
    if (dtype) *dtype = packed->dtype;
    if (has_mfma) *has_mfma = packed->geom.mfma_bytes != 0;
    return GSPC_OK;
}

int gspc_pack_input_bf16(const void *in_dev, size_t count, void *out_dev) {
    if (!in_dev || !out_dev) return fail(GSPC_ERR_NULL, "null pointer argument");
    if (count == 0) return GSPC_OK;
    hipError_t e = gspc::launch_cast_bf16(static_cast<const float *>(in_dev), count,
                                          static_cast<uint16_t *>(out_dev), t_stream);
    if (e != hipSuccess) return hip_fail(e, "bf16 cast launch");
    return GSPC_OK;
}

int gspc_conv2d_grouped(const void *input, const gspc_packed_t *packed_weight, int N, int Cin,
                        int H, int W, int Cout, int KH, int KW, int stride, int pad, int groups,
                        void *output) {
    gspc::ConvParams p;
    int rc = prepare_conv(input, packed_weight, N, Cin, H, W, Cout, KH, KW, stride, pad, groups,
                          output, &p);
    if (rc) return rc;
    return dispatch_conv(p, packed_weight);
}

int gspc_force_path(int path) {
    if (path != GSPC_PATH_AUTO && path != GSPC_PATH_DIRECT && path != GSPC_PATH_MFMA)
        return fail(GSPC_ERR_ARG, "unknown path %d", path);
    t_force_path = path;
    return GSPC_OK;
}

int gspc_set_graph_mode(int on) {
    t_graph_mode = on ? 1 : 0;
    if (!on) clear_graphs();
    return GSPC_OK;
}

int gspc_set_chain_fusion(int on) {
    t_fusion = on ? 1 : 0;
    return GSPC_OK;
}

int gspc_set_winograd(int on) {
    t_winograd = on < 0 ? -1 : on ? 1 : 0;
    return GSPC_OK;
}

int gspc_last_path(void) { return t_last_path; }
const char *gspc_last_kernel(void) { return t_last_kernel; }

int gspc_run_layer_chain(const gspc_layer_t *layers, int n_layers, void *const *act_bufs,
                         const size_t *act_bytes, int n_bufs, float *per_layer_ms) {
    if (!layers || !act_bufs || !act_bytes) return fail(GSPC_ERR_NULL, "null pointer argument");
    if (n_layers <= 0 || n_bufs <= 0) return fail(GSPC_ERR_ARG, "empty chain or buffer table");
    for (int b = 0; b < n_bufs; ++b)
        if (!act_bufs[b] && act_bytes[b]) return fail(GSPC_ERR_NULL, "activation buffer %d is null", b);
    for (int b = 0; b < n_bufs; ++b)
        if (reinterpret_cast<uintptr_t>(act_bufs[b]) & 15)
            return fail(GSPC_ERR_ARG, "activation buffer %d is not 16-byte aligned", b);

    // Pass 1: validate every step before anything is launched.
    std::vector<gspc::ConvParams> params(n_layers);
    for (int i = 0; i < n_layers; ++i) {
        const gspc_layer_t &L = layers[i];
        auto buf_ok = [&](int idx) { return idx >= 0 && idx < n_bufs; };
        if (!buf_ok(L.src) || !buf_ok(L.dst))
            return fail(GSPC_ERR_ARG, "layer %d: buffer index out of range", i);
        if (L.N <= 0 || L.Cin <= 0 || L.H <= 0 || L.W <= 0)
            return fail(GSPC_ERR_DIM, "layer %d: non-positive dimension", i);
        const double in_elems = (double)L.N * L.Cin * L.H * L.W;
        if (in_elems >= 2147483648.0) return fail(GSPC_ERR_DIM, "layer %d: tensor too large", i);
        switch (L.op) {
        case GSPC_OP_CONV: {
            if (!L.w) return fail(GSPC_ERR_NULL, "layer %d: conv without weights", i);
            if (L.dst == L.src || L.dst == L.src2)
                return fail(GSPC_ERR_ARG, "layer %d: conv output aliases an input", i);
            int rc = prepare_conv(act_bufs[L.src], L.w, L.N, L.Cin, L.H, L.W, L.Cout, L.KH, L.KW,
                                  L.stride, L.pad, L.groups, act_bufs[L.dst], &params[i]);
            if (rc) return rc;
            gspc::ConvParams &p = params[i];
            const size_t in_b = (size_t)in_elems * (p.in_bf16 ? 2 : 4);
            const size_t out_b = (size_t)L.N * L.Cout * p.Hout * p.Wout * 4;
            if (act_bytes[L.src] < in_b || act_bytes[L.dst] < out_b)
                return fail(GSPC_ERR_SPACE, "layer %d: activation buffer too small", i);
            if (L.src2 >= 0) {
                if (!buf_ok(L.src2)) return fail(GSPC_ERR_ARG, "layer %d: residual index out of range", i);
                if (act_bytes[L.src2] < out_b)
                    return fail(GSPC_ERR_SPACE, "layer %d: residual buffer too small", i);
                p.res = static_cast<const float *>(act_bufs[L.src2]);
            }
            p.relu = (L.flags & GSPC_FLAG_RELU) ? 1 : 0;
            break;
        }
        case GSPC_OP_MAXPOOL: {
            if (L.KH <= 0 || L.KH != L.KW || L.stride <= 0 || L.pad < 0 || 2 * L.pad > L.KH)
                return fail(GSPC_ERR_DIM, "layer %d: bad pooling window", i);
            const int ho = out_dim(L.H, L.KH, L.stride, L.pad), wo = out_dim(L.W, L.KW, L.stride, L.pad);
            if (ho <= 0 || wo <= 0) return fail(GSPC_ERR_DIM, "layer %d: pooling window does not fit", i);
            if (L.dst == L.src) return fail(GSPC_ERR_ARG, "layer %d: pooling in place", i);
            if (act_bytes[L.src] < (size_t)in_elems * 4 ||
                act_bytes[L.dst] < (size_t)L.N * L.Cin * ho * wo * 4)
                return fail(GSPC_ERR_SPACE, "layer %d: activation buffer too small", i);
            break;
        }
        case GSPC_OP_ADD:
            if (!buf_ok(L.src2)) return fail(GSPC_ERR_ARG, "layer %d: second operand index out of range", i);
            if (act_bytes[L.src2] < (size_t)in_elems * 4)
                return fail(GSPC_ERR_SPACE, "layer %d: activation buffer too small", i);
            // fallthrough
        case GSPC_OP_RELU:
            if (act_bytes[L.src] < (size_t)in_elems * 4 || act_bytes[L.dst] < (size_t)in_elems * 4)
                return fail(GSPC_ERR_SPACE, "layer %d: activation buffer too small", i);
            break;
        default:
            return fail(GSPC_ERR_ARG, "layer %d: unknown op %d", i, L.op);
        }
    }

    // Pass 2: launch.  Without per-layer timing, and on a capturable stream,
    // the launches are recorded once into a HIP graph and replayed afterwards:
    // at batch 1 the kernels are shorter than the host's launch cost.
    auto launch_step = [&](int i) -> int {
        const gspc_layer_t &L = layers[i];
        const size_t elems = (size_t)L.N * L.Cin * L.H * L.W;
        hipError_t e = hipSuccess;
        switch (L.op) {
        case GSPC_OP_CONV:
            return dispatch_conv(params[i], L.w);
        case GSPC_OP_MAXPOOL:
            e = gspc::launch_maxpool(static_cast<const float *>(act_bufs[L.src]),
                                     static_cast<float *>(act_bufs[L.dst]), L.N, L.Cin, L.H, L.W,
                                     L.KH, L.stride, L.pad, out_dim(L.H, L.KH, L.stride, L.pad),
                                     out_dim(L.W, L.KW, L.stride, L.pad), t_stream);
            break;
        case GSPC_OP_ADD:
            e = gspc::launch_add(static_cast<const float *>(act_bufs[L.src]),
                                 static_cast<const float *>(act_bufs[L.src2]),
                                 static_cast<float *>(act_bufs[L.dst]), elems,
                                 (L.flags & GSPC_FLAG_RELU) ? 1 : 0, t_stream);
            break;
        case GSPC_OP_RELU:
            e = gspc::launch_relu(static_cast<const float *>(act_bufs[L.src]),
                                  static_cast<float *>(act_bufs[L.dst]), elems, t_stream);
            break;
        }
        return e == hipSuccess ? GSPC_OK : hip_fail(e, "chain op launch");
    };

    if (!per_layer_ms) {
        // Steps of the untimed path: single layers, or fused runs of grouped layers.
        struct Step {
            int first, count;
            gspc::FusedPlan *plan;
            gspc::DwPwPlan *pair;
            gspc::GpwPlan *gpair;
        };
        std::vector<Step> steps;
        std::vector<std::unique_ptr<gspc::FusedPlan>> plans;
        std::vector<std::unique_ptr<gspc::DwPwPlan>> pairs;
        std::vector<std::unique_ptr<gspc::GpwPlan>> gpairs;
        for (int i = 0; i < n_layers;) {
            int covered = 0;
            if (t_fusion && t_force_path == GSPC_PATH_AUTO) {
                auto pl = std::make_unique<gspc::FusedPlan>();
                covered = gspc::plan_fused_run(layers, i, n_layers - i, act_bufs, pl.get());
                if (covered > 0) {
                    steps.push_back({i, covered, pl.get(), nullptr, nullptr});
                    plans.push_back(std::move(pl));
                } else {
                    auto pr = std::make_unique<gspc::DwPwPlan>();
                    covered = gspc::plan_dwpw(layers, i, n_layers - i, act_bufs, pr.get());
                    if (covered > 0) {
                        steps.push_back({i, covered, nullptr, pr.get(), nullptr});
                        pairs.push_back(std::move(pr));
                    } else {
                        auto gp = std::make_unique<gspc::GpwPlan>();
                        covered = gspc::plan_gpw(layers, i, n_layers - i, act_bufs, gp.get());
                        if (covered > 0) {
                            steps.push_back({i, covered, nullptr, nullptr, gp.get()});
                            gpairs.push_back(std::move(gp));
                        }
                    }
                }
            }
            if (covered == 0) {
                steps.push_back({i, 1, nullptr, nullptr, nullptr});
                covered = 1;
            }
            i += covered;
        }
        auto run_steps = [&]() -> int {
            for (const Step &st : steps) {
                if (st.plan) {
                    const hipError_t e = gspc::launch_fused_run(*st.plan, t_stream, &t_last_kernel);
                    if (e != hipSuccess) return hip_fail(e, "fused run launch");
                    t_last_path = GSPC_PATH_DIRECT;
                } else if (st.pair) {
                    const hipError_t e = gspc::launch_dwpw(*st.pair, t_stream, &t_last_kernel);
                    if (e != hipSuccess) return hip_fail(e, "fused pair launch");
                    t_last_path = GSPC_PATH_MFMA;
                } else if (st.gpair) {
                    const hipError_t e = gspc::launch_gpw(*st.gpair, t_stream, &t_last_kernel);
                    if (e != hipSuccess) return hip_fail(e, "fused pair launch");
                    t_last_path = GSPC_PATH_MFMA;
                } else {
                    const int rc2 = launch_step(st.first);
                    if (rc2 != GSPC_OK) return rc2;
                }
            }
            return GSPC_OK;
        };
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        const bool try_graph = t_graph_mode && t_stream != nullptr && n_layers > 1 &&
                               hipStreamIsCapturing(t_stream, &cap) == hipSuccess &&
                               cap == hipStreamCaptureStatusNone;
        if (try_graph) {
            const uint64_t key = chain_key(layers, n_layers, act_bufs, n_bufs, t_stream, t_force_path, t_fusion + 2 * (gspc::winograd_mode() + 1) + 8 * (gspc::gpw_enabled() ? 1 : 0));
            auto it = t_graphs.find(key);
            if (it == t_graphs.end()) {
                hipGraph_t graph = nullptr;
                hipGraphExec_t exec = nullptr;
                if (hipStreamBeginCapture(t_stream, hipStreamCaptureModeThreadLocal) == hipSuccess) {
                    const int rc2 = run_steps();
                    const hipError_t ee = hipStreamEndCapture(t_stream, &graph);
                    if (rc2 != GSPC_OK) {
                        if (graph) (void)hipGraphDestroy(graph);
                        return rc2;
                    }
                    if (ee == hipSuccess && graph &&
                        hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess) {
                        if (t_graphs.size() >= 64) clear_graphs();
                        it = t_graphs.emplace(key, ChainGraph{graph, exec}).first;
                    } else {
                        if (graph) (void)hipGraphDestroy(graph);
                        (void)hipGetLastError();
                    }
                } else {
                    (void)hipGetLastError();
                }
            }
            if (it != t_graphs.end()) {
                const hipError_t e = hipGraphLaunch(it->second.exec, t_stream);
                if (e != hipSuccess) return hip_fail(e, "hipGraphLaunch");
                return GSPC_OK;
            }
        }
        return run_steps();
    }

    std::vector<hipEvent_t> ev(n_layers + 1);
    for (auto &e : ev) {
        hipError_t er = hipEventCreate(&e);
        if (er != hipSuccess) return hip_fail(er, "hipEventCreate");
    }
    (void)hipEventRecord(ev[0], t_stream);
    int rc = GSPC_OK;
    for (int i = 0; i < n_layers && rc == GSPC_OK; ++i) {
        rc = launch_step(i);
        (void)hipEventRecord(ev[i + 1], t_stream);
    }
    {
        hipError_t e = hipStreamSynchronize(t_stream);
        if (e != hipSuccess && rc == GSPC_OK) rc = hip_fail(e, "hipStreamSynchronize");
        for (int i = 0; i < n_layers; ++i) {
            float ms = 0.f;
            if (rc == GSPC_OK) (void)hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
            per_layer_ms[i] = ms;
        }
        for (auto &e2 : ev) (void)hipEventDestroy(e2);
    }
    return rc;
}

}  // extern "C"
