// Stage 1 of GSPC (kernel reshape, Section III-B of arXiv 2006.09791) for the
// GPU layouts, its inverse, and the fp32 -> bf16 input cast.
#include "gspc_internal.h"

namespace gspc {

struct PackArgs {
    int groups, CPG, KPG, KH, KW, Kred, KPGd;
    int variant, ksub, ksteps, mtiles;
    int to_bf16;
};

__device__ __forceinline__ float round_bf16(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return v;  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

// total covers the section plus the alignment gap behind it, which is zeroed.
__global__ void pack_direct_kernel(const float *__restrict__ w, float *__restrict__ out,
                                   PackArgs a, size_t section, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    if (d >= section) {
        out[d] = 0.f;
        return;
    }
    const int o = (int)(d % a.KPGd);
    const size_t r = d / a.KPGd;
    const int k = (int)(r % a.Kred);
    const int j = (int)(r / a.Kred);
    float v = 0.f;
    if (o < a.KPG) {
        v = w[((size_t)j * a.KPG + o) * a.Kred + k];
        if (a.to_bf16) v = round_bf16(v);
    }
    out[d] = v;
}

__global__ void pack_mfma_kernel(const float *__restrict__ w, float *__restrict__ out,
                                 PackArgs a, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int lane = (int)(d % 64);
    size_t r = d / 64;
    const int mt = (int)(r % a.mtiles);
    r /= a.mtiles;
    const int ks = (int)(r % a.ksteps);
    const int j = (int)(r / a.ksteps);
    const int taps = a.KH * a.KW;
    const int cblk = ks / taps, tap = ks % taps;
    const int oc_in = lane % 16;
    const int sub = lane / 16;
    const int c = cblk * a.ksub + sub;
    float v = 0.f;
    if (c < a.CPG && mt * 16 + oc_in < a.KPG) {
        const int oc = j * a.KPG + mt * 16 + oc_in;
        v = w[(size_t)oc * a.Kred + (size_t)c * taps + tap];
        if (a.to_bf16) v = round_bf16(v);
    }
    out[d] = v;
}

// Winograd section: U = G g G^T of every 3x3 filter slice (G of F(2x2, 3x3): rows (1, 0, 0),
// (1/2, 1/2, 1/2), (1/2, -1/2, 1/2), (0, 0, 1)), one thread per element.
__global__ void pack_wino_kernel(const float *__restrict__ w, float *__restrict__ out, PackArgs a, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int e = (int)(d % 4);
    size_t r = d / 4;
    const int lane = (int)(r % 64);
    r /= 64;
    const int quad = (int)(r % 4);
    r /= 4;
    const int mtiles = (a.KPG + 15) / 16, cblks = a.CPG / 4;
    const int mt = (int)(r % mtiles);
    r /= mtiles;
    const int cb = (int)(r % cblks);
    const int j = (int)(r / cblks);
    const int xi = quad, nu = e;   // position 4*quad + e = 4*xi + nu
    if (mt * 16 + lane % 16 >= a.KPG) {   // padding filter of the last tile
        out[d] = 0.f;
        return;
    }
    const int oc = j * a.KPG + mt * 16 + lane % 16, c = cb * 4 + lane / 16;
    const float *g = w + (size_t)oc * a.Kred + (size_t)c * 9;
    const float G[4][3] = {{1.f, 0.f, 0.f}, {0.5f, 0.5f, 0.5f}, {0.5f, -0.5f, 0.5f}, {0.f, 0.f, 1.f}};
    float u = 0.f;
    for (int p = 0; p < 3; ++p) {
        float row = 0.f;   // (g G^T)[p][nu]
        for (int q = 0; q < 3; ++q) row += g[p * 3 + q] * G[nu][q];
        u += G[xi][p] * row;
    }
    out[d] = u;
}

// Weight of filter fo and channel cm of a merged group (m consecutive groups seen as one
// block-diagonal group): zero unless both belong to the same original group.
__device__ __forceinline__ float merged_weight(const float *__restrict__ w, const PackArgs &a, int m, int jm, int fo,
                                               int cm, int tap) {
    if (fo >= a.KPG * m || cm >= a.CPG * m || fo / a.KPG != cm / a.CPG) return 0.f;
    const int oc = jm * a.KPG * m + fo;
    return w[(size_t)oc * a.Kred + (size_t)(cm % a.CPG) * 9 + tap];
}

// Merged direct section [groups/m][m*CPG*9][KPGd2] (3x3 layers): the direct section of the layer
// seen as groups / m block-diagonal groups.
__global__ void pack_direct_merged_kernel(const float *__restrict__ w, float *__restrict__ out, PackArgs a, int m,
                                          int KPGd2, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int o = (int)(d % KPGd2);
    const size_t r = d / KPGd2;
    const int kred2 = a.CPG * m * 9;
    const int k = (int)(r % kred2);
    const int j = (int)(r / kred2);
    float v = merged_weight(w, a, m, j, o, k / 9, k % 9);
    if (a.to_bf16) v = round_bf16(v);
    out[d] = v;
}

// Quad-k section [groups/m][k-steps/4][m*KPG/16][64 lanes][4], taps = KH*KW (9 or 1).
__global__ void pack_quadk_kernel(const float *__restrict__ w, float *__restrict__ out, PackArgs a, int m, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int taps = a.KH * a.KW;
    const int e = (int)(d % 4);
    size_t r = d / 4;
    const int lane = (int)(r % 64);
    r /= 64;
    const int mtiles = a.KPG * m / 16, quads = a.CPG * m / 4 * taps / 4;
    const int mt = (int)(r % mtiles);
    r /= mtiles;
    const int quad = (int)(r % quads);
    const int j = (int)(r / quads);
    const int ks = 4 * quad + e, cm = (ks / taps) * 4 + lane / 16, tap = ks % taps, fo = mt * 16 + lane % 16;
    float v = 0.f;
    if (fo / a.KPG == cm / a.CPG)   // same original group
        v = w[(size_t)(j * a.KPG * m + fo) * a.Kred + (size_t)(cm % a.CPG) * taps + tap];
    out[d] = v;
}

// bf16 matrix-core section, one thread per 2-byte element; m = groups merged per section group.
__global__ void pack_bf16_kernel(const float *__restrict__ w, uint16_t *__restrict__ out, PackArgs a,
                                 int ckb, int ks_b, int nchunks, int m, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int e = (int)(d % 8);
    size_t r = d / 8;
    const int lane = (int)(r % 64);
    r /= 64;
    const int mtiles = (a.KPG * m + 15) / 16;
    const int mt = (int)(r % mtiles);
    r /= mtiles;
    const int ks = (int)(r % ks_b);
    r /= ks_b;
    const int chunk = (int)(r % nchunks);
    const int j = (int)(r / nchunks);
    const int u8 = ckb / 8, u = 4 * ks + lane / 16;
    uint16_t v = 0;
    if (u < 9 * u8) {
        const int tap = u / u8, cb8 = u % u8;
        v = (uint16_t)(__float_as_uint(round_bf16(merged_weight(w, a, m, j, mt * 16 + lane % 16,
                                                                 chunk * ckb + cb8 * 8 + e, tap))) >> 16);
    }
    out[d] = v;
}

// bf16 row-product section: banded operands [merged group][filter quad][kh][channel quad][lane][8].
__global__ void pack_row_kernel(const float *__restrict__ w, uint16_t *__restrict__ out, PackArgs a, int m,
                                size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int e = (int)(d % 8);
    size_t r = d / 8;
    const int lane = (int)(r % 64);
    r /= 64;
    const int cqs = a.CPG * m / 4, fqs = a.KPG * m / 4;
    const int cq = (int)(r % cqs);
    r /= cqs;
    const int kh = (int)(r % 3);
    r /= 3;
    const int fq = (int)(r % fqs);
    const int j = (int)(r / fqs);
    // product row (lane % 16) = (filter of the quad, output column of the window); reduction slot
    // (lane / 16, e) = (channel of the quad, input column of the window); the window starts two
    // columns left of its first output column
    const int f = (lane % 16) / 4, ow = (lane % 16) % 4, kw = e - ow - 1;
    uint16_t v = 0;
    if (kw >= 0 && kw < 3)
        v = (uint16_t)(__float_as_uint(round_bf16(merged_weight(w, a, m, j, fq * 4 + f, cq * 4 + lane / 16, kh * 3 + kw))) >> 16);
    out[d] = v;
}

__global__ void unpack_kernel(const float *__restrict__ sec, float *__restrict__ w, PackArgs a,
                              int from_mfma, size_t total) {
    size_t d = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= total) return;
    const int k = (int)(d % a.Kred);
    const int oc = (int)(d / a.Kred);
    const int j = oc / a.KPG, o = oc % a.KPG;
    if (!from_mfma) {
        w[d] = sec[((size_t)j * a.Kred + k) * a.KPGd + o];
        return;
    }
    const int taps = a.KH * a.KW;
    const int c = k / taps, tap = k % taps;
    const int mt = o / 16, oc_in = o % 16;
    const int cblk = c / a.ksub, sub = c % a.ksub;
    const int lane = sub * 16 + oc_in;
    const int ks = cblk * taps + tap;
    w[d] = sec[(((size_t)j * a.ksteps + ks) * a.mtiles + mt) * 64 + lane];
}

__global__ void cast_bf16_kernel(const float *__restrict__ in, uint16_t *__restrict__ out,
                                 size_t count) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += step) out[i] = (uint16_t)(__float_as_uint(round_bf16(in[i])) >> 16);
}

static PackArgs make_args(const gspc_packed *h) {
    PackArgs a;
    a.groups = h->groups; a.CPG = h->geom.CPG; a.KPG = h->geom.KPG; a.KH = h->KH; a.KW = h->KW;
    a.Kred = h->geom.Kred; a.KPGd = h->geom.KPGd;
    a.variant = h->geom.variant; a.ksub = h->geom.ksub; a.ksteps = h->geom.ksteps;
    a.mtiles = h->geom.mtiles;
    a.to_bf16 = h->dtype == GSPC_BF16;
    return a;
}

static unsigned blocks_for(size_t total, int threads) {
    return (unsigned)((total + threads - 1) / threads);
}

hipError_t launch_pack_weights(const float *w, const gspc_packed *h, hipStream_t s) {
    const PackArgs a = make_args(h);
    float *dsec = static_cast<float *>(h->dev);
    const size_t nd = h->geom.direct_bytes / sizeof(float);
    const size_t nd_gap = h->geom.mfma_offset / sizeof(float);
    hipLaunchKernelGGL(pack_direct_kernel, dim3(blocks_for(nd_gap, 256)), dim3(256), 0, s, w, dsec, a,
                       nd, nd_gap);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (h->geom.bf16_bytes) {
        uint16_t *bsec = reinterpret_cast<uint16_t *>(static_cast<char *>(h->dev) + h->geom.bf16_offset);
        const size_t nb = h->geom.bf16_bytes / 2;
        hipLaunchKernelGGL(pack_bf16_kernel, dim3(blocks_for(nb, 256)), dim3(256), 0, s, w, bsec, a,
                           h->geom.ckb, h->geom.ks_b, h->geom.nchunks_b, h->geom.mb, nb);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (h->geom.row_bytes) {
        uint16_t *rsec = reinterpret_cast<uint16_t *>(static_cast<char *>(h->dev) + h->geom.row_offset);
        const size_t nr = h->geom.row_bytes / 2;
        hipLaunchKernelGGL(pack_row_kernel, dim3(blocks_for(nr, 256)), dim3(256), 0, s, w, rsec, a, h->geom.mt, nr);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (h->geom.wino_bytes) {
        float *xsec = reinterpret_cast<float *>(static_cast<char *>(h->dev) + h->geom.wino_offset);
        const size_t nx = h->geom.wino_bytes / sizeof(float);
        hipLaunchKernelGGL(pack_wino_kernel, dim3(blocks_for(nx, 256)), dim3(256), 0, s, w, xsec, a, nx);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (h->geom.qk_bytes) {
        float *qsec = reinterpret_cast<float *>(static_cast<char *>(h->dev) + h->geom.qk_offset);
        const size_t nq = h->geom.qk_bytes / sizeof(float);
        hipLaunchKernelGGL(pack_quadk_kernel, dim3(blocks_for(nq, 256)), dim3(256), 0, s, w, qsec, a, h->geom.qk_m, nq);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int which = 0; which < 2; ++which) {
        const PackGeom::MergedDirect &md = h->geom.md[which];
        if (!md.m) continue;
        float *dsec2 = reinterpret_cast<float *>(static_cast<char *>(h->dev) + md.offset);
        const size_t n2 = md.bytes / sizeof(float);
        hipLaunchKernelGGL(pack_direct_merged_kernel, dim3(blocks_for(n2, 256)), dim3(256), 0, s, w, dsec2, a, md.m,
                           md.KPGd, n2);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (h->geom.mfma_bytes) {
        float *msec = reinterpret_cast<float *>(static_cast<char *>(h->dev) + h->geom.mfma_offset);
        const size_t nm = h->geom.mfma_bytes / sizeof(float);
        hipLaunchKernelGGL(pack_mfma_kernel, dim3(blocks_for(nm, 256)), dim3(256), 0, s, w, msec, a, nm);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_unpack_weights(const gspc_packed *h, int which, float *w, hipStream_t s) {
    const PackArgs a = make_args(h);
    const size_t total = (size_t)h->Cout * h->geom.Kred;
    const int from_mfma = which == GSPC_PATH_MFMA;
    const float *sec = from_mfma
                           ? reinterpret_cast<const float *>(static_cast<const char *>(h->dev) +
                                                             h->geom.mfma_offset)
                           : static_cast<const float *>(h->dev);
    hipLaunchKernelGGL(unpack_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, sec, w, a,
                       from_mfma, total);
    return hipGetLastError();
}

hipError_t launch_cast_bf16(const float *in, size_t count, uint16_t *out, hipStream_t s) {
    size_t blocks = (count + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, out, count);
    return hipGetLastError();
}

}  // namespace gspc
