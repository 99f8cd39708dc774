// Direct (sliding-window) grouped convolution kernels: the convolution stage of
// Algorithm 1 of arXiv 2006.09791 with the input and output reshapes fused
// away.  These cover every shape; the matrix-core kernels take over where the
// per-group contraction is wide.
#include <cstdlib>
#include <cstring>
#include <unordered_map>

#include "conv_common.h"

namespace gspc {

__device__ __forceinline__ float load_in(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_in(const uint16_t *p, size_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);
}

__device__ __forceinline__ float epilogue(float v, const float *res, size_t idx, int relu) {
    if (res) v += res[idx];
    return relu ? fmaxf(v, 0.f) : v;
}

// One thread = one output pixel x OCT consecutive filters of one group.
// Weights come from the direct section [g][Kred][KPGd]; the OCT values of a
// tap are adjacent and their address is uniform over the block.
template <int OCT, typename TIN>
__global__ __launch_bounds__(256) void conv_direct_generic(ConvParams p) {
    const int HWo = p.Hout * p.Wout;
    const int pix = blockIdx.x * blockDim.x + threadIdx.x;
    const int tiles = p.KPGd / OCT;
    const int j = blockIdx.y / tiles;
    const int oc0 = (blockIdx.y % tiles) * OCT;
    const int n = blockIdx.z;
    if (pix >= HWo) return;
    const int oh = pix / p.Wout, ow = pix % p.Wout;
    const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
    const size_t plane = (size_t)p.H * p.W;
    const TIN *xg = static_cast<const TIN *>(p.x) + ((size_t)n * p.Cin + (size_t)j * p.CPG) * plane;
    const float *wg = p.wd + (size_t)j * p.CPG * p.KH * p.KW * p.KPGd + oc0;

    float acc[OCT];
#pragma unroll
    for (int o = 0; o < OCT; ++o) acc[o] = 0.f;

    for (int c = 0; c < p.CPG; ++c) {
        for (int kh = 0; kh < p.KH; ++kh) {
            const int ih = ih0 + kh;
            const bool row_ok = ih >= 0 && ih < p.H;
            for (int kw = 0; kw < p.KW; ++kw) {
                const int iw = iw0 + kw;
                float xv = 0.f;
                if (row_ok && iw >= 0 && iw < p.W) xv = load_in(xg, c * plane + (size_t)ih * p.W + iw);
                const float *wk = wg + (size_t)((c * p.KH + kh) * p.KW + kw) * p.KPGd;
#pragma unroll
                for (int o = 0; o < OCT; ++o) acc[o] = fmaf(xv, wk[o], acc[o]);
            }
        }
    }
#pragma unroll
    for (int o = 0; o < OCT; ++o) {
        if (oc0 + o < p.KPG) {
            const size_t idx = (((size_t)n * p.Cout + (size_t)j * p.KPG + oc0 + o) * p.Hout + oh) * p.Wout + ow;
            p.y[idx] = epilogue(acc[o], p.res, idx, p.relu);
        }
    }
}

template <int OCT, typename TIN>
static hipError_t launch_generic(const ConvParams &p, hipStream_t s) {
    const int HWo = p.Hout * p.Wout;
    dim3 grid((HWo + 255) / 256, p.groups * (p.KPGd / OCT), p.N);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorNotSupported;
    hipLaunchKernelGGL((conv_direct_generic<OCT, TIN>), grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Register-tiled 3x3 kernel for groups with very few channels (large g) and
// depthwise layers (g = C): the HBM-bound end of the sweep.
//
// One thread owns a strip of 4 output columns x R output rows of one
// (image, group) and all KPG filters of the group.  Each input row segment is
// read once from global memory as an aligned 16-byte load; the single extra
// column needed on each side comes from the neighbouring lanes with wavefront
// shuffles (zero at the image border), so nothing is staged through LDS and no
// element is fetched twice within a wave.  The group's filter bank sits in
// registers.  Requires pad = 1, Wout a multiple of 4 and, for stride 2, W = 2*Wout.
// ---------------------------------------------------------------------------
struct TileS {
    int SPR, RG;            // strip slots per output row (see SPRv), row groups per plane
    int SPRv;               // strips that exist; SPR is rounded up to a divisor of 64 so that a row's
                            // strips never straddle a wavefront (the surplus lanes idle)
    int total;              // threads with work
    int shfl;               // strips of a row never straddle a wave: neighbours by shuffle
    unsigned m_spr, m_rg, m_g;
    unsigned x_bytes, w_bytes, y_bytes;
};

template <int CPG, int KPG, int S, int R, typename TIN>
__global__ __launch_bounds__(256) void conv_direct_small(ConvParams p, TileS t) {
    constexpr int ES = (int)sizeof(TIN);
    constexpr int IR = S == 1 ? R + 2 : 2 * R + 1;   // input rows per strip
    constexpr int NV = S;                            // 16-byte loads per input row
    const unsigned gt = blockIdx.x * 256 + threadIdx.x;
    const unsigned g0 = gt < (unsigned)t.total ? gt : 0;
    const unsigned srow = fast_div(g0, t.m_spr), colv = g0 - srow * t.SPR;
    const bool live = gt < (unsigned)t.total && colv < (unsigned)t.SPRv;
    const unsigned plane = fast_div(srow, t.m_rg), rg = srow - plane * t.RG;
    const unsigned n = fast_div(plane, t.m_g), j = plane - n * p.groups;
    const int oh0 = rg * R, ih0 = oh0 * S - 1;
    const int lane = threadIdx.x & 63;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);

    // filter bank: w[k][o], k = (c, kh, kw); the direct section pads KPG to 4
    f32x4 w[CPG * 9];
#pragma unroll
    for (int k = 0; k < CPG * 9; ++k)
        w[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                             rw, (j * (CPG * 9) + k) * (p.KPGd * 4), 0, 0));

    float acc[KPG][R][4];
#pragma unroll
    for (int o = 0; o < KPG; ++o)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int x = 0; x < 4; ++x) acc[o][r][x] = 0.f;

    const bool has_left = colv > 0, has_right = colv + 1 < (unsigned)t.SPRv;
#pragma unroll
    for (int c = 0; c < CPG; ++c) {
        const unsigned cbase = ((n * p.Cin + j * CPG + c) * p.H) * p.W;
#pragma unroll
        for (int i = 0; i < IR; ++i) {
            const int ih = ih0 + i;
            const bool row_ok = live && ih >= 0 && ih < p.H;
            // xv[0] = column 4*S*colv - 1, xv[1..4*S] = the strip, xv[4*S+1] = next column
            float xv[4 * NV + 2];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const unsigned off = row_ok ? (cbase + ih * p.W + (colv * NV + v) * 4) * ES : kOob;
                const f32x4 q = buf_load_in<TIN>(rx, off, 0, 1);
                xv[1 + 4 * v] = q.x; xv[2 + 4 * v] = q.y; xv[3 + 4 * v] = q.z; xv[4 + 4 * v] = q.w;
            }
            if (t.shfl) {
                const float l = __shfl_up(xv[4 * NV], 1), r = __shfl_down(xv[1], 1);
                xv[0] = has_left ? l : 0.f;
                xv[4 * NV + 1] = has_right ? r : 0.f;
            } else {
                const unsigned lo = (row_ok && has_left) ? (cbase + ih * p.W + colv * NV * 4 - 1) * ES : kOob;
                const unsigned ro = (row_ok && has_right) ? (cbase + ih * p.W + (colv + 1) * NV * 4) * ES : kOob;
                xv[0] = buf_load_in<TIN>(rx, lo, 0, 0).x;
                xv[4 * NV + 1] = S == 1 ? buf_load_in<TIN>(rx, ro, 0, 0).x : 0.f;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int kh = i - r * S;
                if (kh < 0 || kh > 2) continue;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const f32x4 wk = w[(c * 3 + kh) * 3 + kw];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const float xin = xv[x * S + kw];
                        acc[0][r][x] = fmaf(xin, wk.x, acc[0][r][x]);
                        if (KPG > 1) acc[KPG > 1 ? 1 : 0][r][x] = fmaf(xin, wk.y, acc[KPG > 1 ? 1 : 0][r][x]);
                        if (KPG > 2) acc[KPG > 2 ? 2 : 0][r][x] = fmaf(xin, wk.z, acc[KPG > 2 ? 2 : 0][r][x]);
                        if (KPG > 3) acc[KPG > 3 ? 3 : 0][r][x] = fmaf(xin, wk.w, acc[KPG > 3 ? 3 : 0][r][x]);
                    }
                }
            }
        }
    }
    (void)lane;

    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, p.res ? t.y_bytes : 0u);
#pragma unroll
    for (int o = 0; o < KPG; ++o) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int oh = oh0 + r;
            const unsigned off = (live && oh < p.Hout)
                                     ? (((n * p.Cout + j * KPG + o) * p.Hout + oh) * p.Wout + colv * 4) * 4
                                     : kOob;
            f32x4 v = f32x4{acc[o][r][0], acc[o][r][1], acc[o][r][2], acc[o][r][3]};
            if (p.res) v += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, off, 0, 0));
            if (p.relu) v = f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), ry, off, 0, 0);
        }
    }
}

// ---------------------------------------------------------------------------
// Flat 3x3 kernel for the shapes the strip kernel cannot take (planes whose
// width is not a multiple of 4, e.g. 14x14 and 7x7 depthwise layers): one thread
// per output pixel of one (image, group), all KPG <= 4 filters of the group,
// planes treated as flat memory so that neighbouring lanes read neighbouring
// addresses even when a row is only 7 elements long.
// ---------------------------------------------------------------------------
struct TileF {
    unsigned total;
    float r_hwo;             // 1 / (Hout*Wout), for the one division whose numerator is large
    unsigned m_wout, m_g;
    unsigned x_bytes, w_bytes, y_bytes;
};

template <int KPG, typename TIN>
__global__ __launch_bounds__(256) void conv_direct_flat(ConvParams p, TileF t) {
    constexpr int ES = (int)sizeof(TIN);
    const unsigned gt = blockIdx.x * 256 + threadIdx.x;
    const bool live = gt < t.total;
    const unsigned g0 = live ? gt : 0;
    const unsigned HWo = p.Hout * p.Wout;
    // g0 / HWo by reciprocal estimate and correction (g0 may be close to 2^32)
    unsigned plane = (unsigned)(__uint2float_rz(g0) * t.r_hwo);
    int rem = (int)(g0 - plane * HWo);
    while (rem < 0) { --plane; rem += (int)HWo; }
    while (rem >= (int)HWo) { ++plane; rem -= (int)HWo; }
    const unsigned pix = (unsigned)rem;
    const unsigned oh = fast_div(pix, t.m_wout), ow = pix - oh * p.Wout;
    const unsigned n = fast_div(plane, t.m_g), j = plane - n * p.groups;
    const int ih0 = (int)(oh * p.stride) - p.pad, iw0 = (int)(ow * p.stride) - p.pad;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < p.CPG; ++c) {
        const unsigned cbase = ((n * p.Cin + j * p.CPG + c) * p.H) * p.W;
        const unsigned wbase = ((j * p.CPG + c) * 9) * (p.KPGd * 4);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int ih = ih0 + kh, iw = iw0 + kw;
                const bool ok = live && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                const float xv = buf_load_in<TIN>(rx, ok ? (cbase + ih * p.W + iw) * ES : kOob, 0, 0).x;
                const f32x4 wk = __builtin_bit_cast(
                    f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, wbase + (kh * 3 + kw) * (p.KPGd * 4), 0, 0));
                acc += xv * wk;
            }
        }
    }
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, p.res ? t.y_bytes : 0u);
#pragma unroll
    for (int o = 0; o < KPG; ++o) {
        const unsigned off = live ? ((n * p.Cout + j * KPG + o) * HWo + pix) * 4 : kOob;
        float v = acc[o];
        if (p.res) v += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, off, 0, 0));
        if (p.relu) v = fmaxf(v, 0.f);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), ry, off, 0, 0);
    }
}

namespace {

bool plan_flat(const ConvParams &p, TileF *out) {
    if (p.KH != 3 || p.KW != 3 || p.KPG > 4 || p.CPG > 8) return false;
    const double total = (double)p.N * p.groups * p.Hout * p.Wout;
    const double xb = (double)p.N * p.Cin * p.H * p.W * (p.in_bf16 ? 2 : 4);
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    const double wb = (double)p.groups * p.CPG * 9 * p.KPGd * 4;
    if (total >= 4.0e9 || xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    const double hwo = (double)p.Hout * p.Wout;
    // fast_div exactness: numerator * divisor < 2^32 at each step
    if (hwo >= 1.0e6 || hwo * p.Wout >= 4.29e9 || (total / hwo) * p.groups >= 4.29e9) return false;
    TileF t{};
    t.total = (unsigned)total;
    t.r_hwo = 1.0f / (float)(p.Hout * p.Wout);
    t.m_wout = div_magic(p.Wout);
    t.m_g = div_magic(p.groups);
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    *out = t;
    return true;
}

template <typename TIN>
hipError_t launch_flat(const ConvParams &p, const TileF &t, hipStream_t s) {
    dim3 grid((t.total + 255) / 256);
    switch (p.KPG) {
    case 1: hipLaunchKernelGGL((conv_direct_flat<1, TIN>), grid, dim3(256), 0, s, p, t); break;
    case 2: hipLaunchKernelGGL((conv_direct_flat<2, TIN>), grid, dim3(256), 0, s, p, t); break;
    case 3: hipLaunchKernelGGL((conv_direct_flat<3, TIN>), grid, dim3(256), 0, s, p, t); break;
    default: hipLaunchKernelGGL((conv_direct_flat<4, TIN>), grid, dim3(256), 0, s, p, t); break;
    }
    return hipGetLastError();
}

}  // namespace

namespace {

bool plan_small(const ConvParams &p, TileS *out) {
    if (p.KH != 3 || p.KW != 3 || p.pad != 1 || (p.stride != 1 && p.stride != 2)) return false;
    if (p.Wout % 4 || (p.stride == 2 && p.W != 2 * p.Wout) || p.W % 4) return false;
    const bool inst = (p.CPG == 1 && (p.KPG == 1 || p.KPG == 2)) || (p.CPG == 2 && p.KPG == 2) ||
                      (p.CPG == 4 && p.KPG == 2) || (p.CPG == 2 && p.KPG == 1);
    if (!inst) return false;
    const int R = p.stride == 1 ? 4 : 2;
    TileS t{};
    t.SPRv = p.Wout / 4;
    t.SPR = t.SPRv;
    if (t.SPR <= 64 && 64 % t.SPR) {   // e.g. 14 strips of a 56-wide row take 16 lanes
        t.SPR = 1;
        while (t.SPR < t.SPRv) t.SPR *= 2;
    }
    t.RG = (p.Hout + R - 1) / R;
    const double total = (double)p.N * p.groups * t.RG * t.SPR;
    const double xb = (double)p.N * p.Cin * p.H * p.W * (p.in_bf16 ? 2 : 4);
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    const double wb = (double)p.groups * p.CPG * 9 * p.KPGd * 4;
    if (total >= 2.0e9 || xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    // fast_div exactness: numerator * divisor < 2^32 at each step
    if (total * t.SPR >= 4.0e9 || (total / t.SPR) * t.RG >= 4.0e9 || (double)p.N * p.groups * p.groups >= 4.0e9)
        return false;
    t.total = (int)total;
    t.shfl = t.SPR <= 64 && (64 % t.SPR) == 0;
    t.m_spr = div_magic(t.SPR);
    t.m_rg = div_magic(t.RG);
    t.m_g = div_magic(p.groups);
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    *out = t;
    return true;
}

template <int CPG, int KPG, typename TIN>
hipError_t launch_small_cfg(const ConvParams &p, const TileS &t, hipStream_t s) {
    dim3 grid((t.total + 255) / 256);
    if (p.stride == 1) hipLaunchKernelGGL((conv_direct_small<CPG, KPG, 1, 4, TIN>), grid, dim3(256), 0, s, p, t);
    else hipLaunchKernelGGL((conv_direct_small<CPG, KPG, 2, 2, TIN>), grid, dim3(256), 0, s, p, t);
    return hipGetLastError();
}

template <typename TIN>
hipError_t launch_small(const ConvParams &p, const TileS &t, hipStream_t s) {
    if (p.CPG == 1 && p.KPG == 1) return launch_small_cfg<1, 1, TIN>(p, t, s);
    if (p.CPG == 1 && p.KPG == 2) return launch_small_cfg<1, 2, TIN>(p, t, s);
    if (p.CPG == 2 && p.KPG == 1) return launch_small_cfg<2, 1, TIN>(p, t, s);
    if (p.CPG == 2 && p.KPG == 2) return launch_small_cfg<2, 2, TIN>(p, t, s);
    if (p.CPG == 4 && p.KPG == 2) return launch_small_cfg<4, 2, TIN>(p, t, s);
    return hipErrorNotSupported;
}

}  // namespace

hipError_t launch_direct(const ConvParams &p, hipStream_t s, const char **name) {
    static const bool no_small = std::getenv("GSPC_NO_SMALL") != nullptr;   // tuning aid
    // depthwise planes small enough to sit whole in LDS (up to about 40x40)
    DwPlan dw;
    if (plan_dw_planes(p, &dw)) return launch_dw_planes(p, dw, s, name);
    TileS ts;
    if (!no_small && plan_small(p, &ts)) {
        *name = intern_name("conv_direct_small<" + std::to_string(p.CPG) + "," + std::to_string(p.KPG) + "," +
                            std::to_string(p.stride) + "," + std::to_string(p.stride == 1 ? 4 : 2) +
                            (p.in_bf16 ? ",bf16>" : ",f32>"));
        return p.in_bf16 ? launch_small<uint16_t>(p, ts, s) : launch_small<float>(p, ts, s);
    }
    TileF tf;
    if (plan_flat(p, &tf)) {
        *name = intern_name("conv_direct_flat<" + std::to_string(p.KPG) + (p.in_bf16 ? ",bf16>" : ",f32>"));
        return p.in_bf16 ? launch_flat<uint16_t>(p, tf, s) : launch_flat<float>(p, tf, s);
    }
    const bool oct8 = p.KPGd % 8 == 0;
    if (p.in_bf16) {
        *name = oct8 ? "conv_direct_generic<8,bf16>" : "conv_direct_generic<4,bf16>";
        return oct8 ? launch_generic<8, uint16_t>(p, s) : launch_generic<4, uint16_t>(p, s);
    }
    *name = oct8 ? "conv_direct_generic<8,f32>" : "conv_direct_generic<4,f32>";
    return oct8 ? launch_generic<8, float>(p, s) : launch_generic<4, float>(p, s);
}

}  // namespace gspc
