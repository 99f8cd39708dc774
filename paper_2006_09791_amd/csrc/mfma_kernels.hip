// Per-group implicit-GEMM grouped convolution on the gfx950 matrix cores.
//
// For one group the convolution stage of Algorithm 1 (arXiv 2006.09791) is the
// contraction  Y[oc][pixel] = sum_k W[oc][k] * X[k][pixel],  k = (c, kh, kw),
// pixel = (n, oh, ow).  Filters sit on the M edge of the MFMA tile, output
// pixels on the N edge, and the im2col matrix X[k][pixel] is never built: a
// zero-haloed input tile is staged in LDS (the paper's input reshape, fused)
// and every lane reads its own (pixel, k) element from it.  Results go
// straight to NCHW (the paper's output reshape, fused away).
#include "gspc_internal.h"

namespace gspc {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int VAR> struct Mma;

// v_mfma_f32_32x32x2_f32: A lane l = (row l%32, k l/32), B lane l = (k l/32, col l%32),
// D reg r of lane l = (row 8*(r/4) + 4*(l/32) + r%4, col l%32).
template <> struct Mma<32> {
    static constexpr int KSUB = 2, PT = 32, NACC = 16;
    typedef f32x16 acc_t;
    __device__ static __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int row(int r, int lane) { return 8 * (r / 4) + 4 * (lane / 32) + r % 4; }
    __device__ static __forceinline__ int ksub(int lane) { return lane / 32; }
};

// v_mfma_f32_16x16x4_f32: A lane l = (row l%16, k l/16), B lane l = (k l/16, col l%16),
// D reg r of lane l = (row 4*(l/16) + r, col l%16).
template <> struct Mma<16> {
    static constexpr int KSUB = 4, PT = 16, NACC = 4;
    typedef f32x4 acc_t;
    __device__ static __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int row(int r, int lane) { return 4 * (lane / 16) + r; }
    __device__ static __forceinline__ int ksub(int lane) { return lane / 16; }
};

// v_mfma_f32_4x4x1_16b_f32: sixteen independent 4x4 outer products.  Block
// l/4 of lane l; A lane = row l%4, B lane = col l%4, D reg r = (row r, col l%4).
// The packed A operand repeats the same four filters in every block, so the
// sixteen blocks act as 64 pixel columns.
template <> struct Mma<4> {
    static constexpr int KSUB = 1, PT = 64, NACC = 4;
    typedef f32x4 acc_t;
    __device__ static __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int row(int r, int /*lane*/) { return r; }
    __device__ static __forceinline__ int ksub(int /*lane*/) { return 0; }
};

// Block tiling chosen on the host.
struct MfmaTile {
    int NB, TH;            // images and output rows per block
    int IHt, LW, IMG, PLANE;  // staged rows, LDS row pitch, floats per image, per channel
    int CK;                // input channels staged per chunk (multiple of KSUB, divides CPGp)
    int CPGp;
    int row_blocks, img_blocks, oc_blocks;
    int in_floats;         // CK * PLANE
    int ksteps, mtiles;    // of the packed section
};

__device__ __forceinline__ float ld_in(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_in(const uint16_t *p, size_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);
}

// Block = WM x WP waves; each wave owns MI x NI MFMA tiles, i.e. VAR*MI filters
// by PT*NI pixels.  Pixels of a block = NB images x TH output rows x Wout.
template <int VAR, int MI, int NI, int WM, int WP, int KH, int KW, int S, typename TIN>
__global__ __launch_bounds__(64 * WM * WP) void conv_mfma(ConvParams p, MfmaTile t) {
    typedef Mma<VAR> M;
    constexpr int KSUB = M::KSUB, PT = M::PT, NACC = M::NACC;
    constexpr int NT = 64 * WM * WP;
    constexpr int TAPS = KH * KW;
    extern __shared__ float smem[];
    float *xs = smem;                 // [CK][PLANE]
    float *ws = smem + t.in_floats;   // [MI*WM][CK/KSUB*TAPS][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WP, wp = wave % WP;
    const int rb = blockIdx.x % t.row_blocks, ib = blockIdx.x / t.row_blocks;
    const int ob = blockIdx.y % t.oc_blocks, j = blockIdx.y / t.oc_blocks;
    const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;

    int base[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        int q = (wp * NI + ni) * PT + lane % PT;
        if (q >= tot) q = 0;
        const int img = q / ppi, rem = q % ppi;
        const int r = rem / p.Wout, col = rem % p.Wout;
        base[ni] = M::ksub(lane) * t.PLANE + img * t.IMG + r * S * t.LW + col * S;
    }

    typename M::acc_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < NACC; ++r) acc[mi][ni][r] = 0.f;

    // Halo columns are never written by the staging loop below: clear once.
    for (int i = tid; i < t.in_floats; i += NT) xs[i] = 0.f;

    const int kchunk = t.CK / KSUB * TAPS;  // k-steps per chunk
    const TIN *xin = static_cast<const TIN *>(p.x);
    const int stage_elems = t.CK * t.NB * t.IHt * p.W;

    for (int c0 = 0; c0 < t.CPGp; c0 += t.CK) {
        __syncthreads();
        for (int e = tid; e < stage_elems; e += NT) {
            const int col = e % p.W;
            int q = e / p.W;
            const int r = q % t.IHt;
            q /= t.IHt;
            const int img = q % t.NB, c = q / t.NB;
            const int ih = ih0 + r, n = n0 + img, cc = c0 + c;
            float v = 0.f;
            if (cc < p.CPG && n < p.N && ih >= 0 && ih < p.H)
                v = ld_in(xin, (((size_t)n * p.Cin + (size_t)j * p.CPG + cc) * p.H + ih) * p.W + col);
            xs[c * t.PLANE + img * t.IMG + r * t.LW + col + p.pad] = v;
        }
        {
            const int per_tile = kchunk * 64;
            const int cb = c0 / KSUB * TAPS;
            for (int e = tid; e < MI * WM * per_tile; e += NT) {
                const int mt = e / per_tile, off = e % per_tile;
                const size_t src =
                    (((size_t)j * t.mtiles + (size_t)ob * (MI * WM) + mt) * t.ksteps + cb) * 64 + off;
                ws[e] = p.wm[src];
            }
        }
        __syncthreads();

        for (int cb = 0; cb < t.CK / KSUB; ++cb) {
            const float *xrow = xs + cb * KSUB * t.PLANE;
            const float *wrow = ws + cb * TAPS * 64 + lane;
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
#pragma unroll
                for (int kw = 0; kw < KW; ++kw) {
                    float a[MI], b[NI];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        a[mi] = wrow[((wm * MI + mi) * kchunk + kh * KW + kw) * 64];
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) b[ni] = xrow[base[ni] + kh * t.LW + kw];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = M::run(a[mi], b[ni], acc[mi][ni]);
                }
            }
        }
    }

    // Epilogue: optional residual and ReLU, NCHW store.
    const size_t HWo = (size_t)p.Hout * p.Wout;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * PT + lane % PT;
        const int img = q / ppi, rem = q % ppi;
        const int oh = oh0 + rem / p.Wout, ow = rem % p.Wout, n = n0 + img;
        if (q >= tot || n >= p.N || oh >= p.Hout) continue;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int r = 0; r < NACC; ++r) {
                const int oc = j * p.KPG + (ob * (MI * WM) + wm * MI + mi) * VAR + M::row(r, lane);
                const size_t idx = ((size_t)n * p.Cout + oc) * HWo + (size_t)oh * p.Wout + ow;
                float v = acc[mi][ni][r];
                if (p.res) v += p.res[idx];
                if (p.relu) v = fmaxf(v, 0.f);
                p.y[idx] = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: tile planning and instance selection.
// ---------------------------------------------------------------------------
namespace {

constexpr int kLdsBudget = 40 * 1024;

struct Cfg {
    int VAR, MI, NI, WM, WP;
};

// Instantiated block shapes, per variant, widest filter tile first.
const Cfg kCfgs[] = {
    {32, 2, 2, 2, 2},  // 128 filters x 128 pixels
    {32, 2, 2, 1, 4},  //  64 filters x 256 pixels
    {32, 1, 2, 1, 4},  //  32 filters x 256 pixels
    {16, 1, 4, 1, 4},  //  16 filters x 256 pixels
    {4, 2, 1, 1, 4},   //   8 filters x 256 pixels
    {4, 1, 1, 1, 4},   //   4 filters x 256 pixels
};

bool shape_instantiated(int KH, int KW, int S) {
    return (KH == 3 && KW == 3 && (S == 1 || S == 2)) || (KH == 1 && KW == 1 && (S == 1 || S == 2)) ||
           (KH == 7 && KW == 7 && S == 2);
}

bool plan(const ConvParams &p, const PackGeom &g, Cfg *cfg_out, MfmaTile *t_out) {
    if (g.variant == kMfmaNone || !p.wm) return false;
    if (!shape_instantiated(p.KH, p.KW, p.stride)) return false;
    for (const Cfg &c : kCfgs) {
        if (c.VAR != g.variant) continue;
        const int MB = c.VAR * c.MI * c.WM;
        if (g.KPG % MB) continue;
        const int PT = c.VAR == 4 ? 64 : c.VAR;
        const int PB = PT * c.NI * c.WP;
        if (p.Wout > PB) continue;
        MfmaTile t{};
        const int HWo = p.Hout * p.Wout;
        if (HWo <= PB) {
            t.TH = p.Hout;
            t.NB = PB / HWo;
            if (t.NB > p.N) t.NB = p.N;
        } else {
            t.NB = 1;
            const int thmax = PB / p.Wout;
            const int rbk = (p.Hout + thmax - 1) / thmax;
            t.TH = (p.Hout + rbk - 1) / rbk;
        }
        t.IHt = (t.TH - 1) * p.stride + p.KH;
        t.LW = p.W + 2 * p.pad;
        t.IMG = t.IHt * t.LW;
        t.PLANE = t.NB * t.IMG;
        t.CPGp = g.CPGp;
        t.ksteps = g.ksteps;
        t.mtiles = g.mtiles;
        t.row_blocks = (p.Hout + t.TH - 1) / t.TH;
        t.img_blocks = (p.N + t.NB - 1) / t.NB;
        t.oc_blocks = g.KPG / MB;
        // Largest chunk (in k-blocks of ksub channels) that divides CPGp/ksub and fits the budget.
        const int cblks = g.CPGp / g.ksub;
        int best = 0;
        for (int d = 1; d <= cblks; ++d) {
            if (cblks % d) continue;
            const size_t bytes = ((size_t)d * g.ksub * t.PLANE +
                                  (size_t)c.MI * c.WM * d * p.KH * p.KW * 64) * sizeof(float);
            if (bytes <= (size_t)kLdsBudget) best = d;
        }
        if (!best) continue;
        t.CK = best * g.ksub;
        t.in_floats = t.CK * t.PLANE;
        if ((long)t.row_blocks * t.img_blocks > 2147483647L || p.groups * t.oc_blocks > 65535) continue;
        *cfg_out = c;
        *t_out = t;
        return true;
    }
    return false;
}

template <int VAR, int MI, int NI, int WM, int WP, int KH, int KW, int S, typename TIN>
hipError_t launch_inst(const ConvParams &p, const MfmaTile &t, hipStream_t s) {
    const size_t lds = ((size_t)t.in_floats + (size_t)MI * WM * (t.CK / Mma<VAR>::KSUB) * KH * KW * 64) *
                       sizeof(float);
    dim3 grid(t.row_blocks * t.img_blocks, p.groups * t.oc_blocks);
    hipLaunchKernelGGL((conv_mfma<VAR, MI, NI, WM, WP, KH, KW, S, TIN>), grid, dim3(64 * WM * WP), lds, s,
                       p, t);
    return hipGetLastError();
}

template <int VAR, int MI, int NI, int WM, int WP, typename TIN>
hipError_t launch_shape(const ConvParams &p, const MfmaTile &t, hipStream_t s) {
    if (p.KH == 3 && p.stride == 1) return launch_inst<VAR, MI, NI, WM, WP, 3, 3, 1, TIN>(p, t, s);
    if (p.KH == 3 && p.stride == 2) return launch_inst<VAR, MI, NI, WM, WP, 3, 3, 2, TIN>(p, t, s);
    if (p.KH == 1 && p.stride == 1) return launch_inst<VAR, MI, NI, WM, WP, 1, 1, 1, TIN>(p, t, s);
    if (p.KH == 1 && p.stride == 2) return launch_inst<VAR, MI, NI, WM, WP, 1, 1, 2, TIN>(p, t, s);
    if (p.KH == 7 && p.stride == 2) return launch_inst<VAR, MI, NI, WM, WP, 7, 7, 2, TIN>(p, t, s);
    return hipErrorNotSupported;
}

template <typename TIN>
hipError_t launch_cfg(const Cfg &c, const ConvParams &p, const MfmaTile &t, hipStream_t s,
                      const char **name) {
#define GSPC_CFG(V, MI_, NI_, WM_, WP_, NAME)                                      \
    if (c.VAR == V && c.MI == MI_ && c.NI == NI_ && c.WM == WM_ && c.WP == WP_) { \
        *name = NAME;                                                              \
        return launch_shape<V, MI_, NI_, WM_, WP_, TIN>(p, t, s);                  \
    }
    GSPC_CFG(32, 2, 2, 2, 2, "conv_mfma<32x32x2,128x128>")
    GSPC_CFG(32, 2, 2, 1, 4, "conv_mfma<32x32x2,64x256>")
    GSPC_CFG(32, 1, 2, 1, 4, "conv_mfma<32x32x2,32x256>")
    GSPC_CFG(16, 1, 4, 1, 4, "conv_mfma<16x16x4,16x256>")
    GSPC_CFG(4, 2, 1, 1, 4, "conv_mfma<4x4x1,8x256>")
    GSPC_CFG(4, 1, 1, 1, 4, "conv_mfma<4x4x1,4x256>")
#undef GSPC_CFG
    return hipErrorNotSupported;
}

}  // namespace

bool mfma_supported(const ConvParams &p, const PackGeom &g) {
    Cfg c;
    MfmaTile t;
    return plan(p, g, &c, &t);
}

hipError_t launch_mfma(const ConvParams &p, const PackGeom &g, hipStream_t s, const char **name) {
    Cfg c;
    MfmaTile t;
    if (!plan(p, g, &c, &t)) return hipErrorNotSupported;
    return p.in_bf16 ? launch_cfg<uint16_t>(c, p, t, s, name) : launch_cfg<float>(c, p, t, s, name);
}

}  // namespace gspc
