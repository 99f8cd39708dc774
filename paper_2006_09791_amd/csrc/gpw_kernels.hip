// Grouped 3x3 convolution fused with the pointwise 1x1 convolution that follows it: the
// building block of the paper's networks (every 3x3 convolution a -> b replaced by a grouped
// 3x3 a -> a and a pointwise a -> b, Sections II and IV-A of arXiv 2006.09791) as ONE kernel,
// so that the grouped result never makes the round trip through HBM and the pair costs one
// launch.  The depthwise end of the sweep has a kernel of its own (dwpw_kernels.hip).
//
// Both stages run on v_mfma_f32_16x16x4_f32 with filters on the M edge and 16 output pixels on
// the N edge.  A wave owns its 16 pixels through both stages and ALL channels:
//   stage A  D[c][px] = sum over the group's channels and the 9 taps (Algorithm 1's convolution
//            stage; groups of fewer than 16 filters are taken as block-diagonal groups of 16,
//            merged by the pack step); the B operand comes from a zero-haloed LDS tile of the
//            input that the block stages once, the A operand from a packed section in which one
//            16-byte load gives a lane its weights for four consecutive k-steps;
//   stage B  Y[k][px] = sum_c W2[k][c] * D[c][px]: the lane that holds D[16t + 4q + r][px] after
//            stage A (lane group q, register r of filter tile t) is not the lane the product wants
//            it in; a 4x4 exchange between registers and lane groups (v_permlane16/32_swap) turns
//            the accumulator tile t into the B operands of k-steps 4t .. 4t+3.  D never leaves
//            the registers, and after the one barrier behind the input tile no wave waits for
//            another.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "conv_common.h"

namespace gspc {

struct GpwParams {
    const float *x;    // input of the grouped layer [N][C][Hd][Wd]
    const float *wa;   // grouped layer, quad-k section [G'][KQ][MTA][64 lanes][4]
    const float *wb;   // pointwise layer, quad-k section [C/16][C2/16][64 lanes][4]
    float *d;          // grouped result [N][C][H][W], or nullptr when nothing reads it later
    float *y;          // pointwise result [N][C2][H][W]
    const float *res;  // optional residual of the pointwise layer
    int N, C, Hd, Wd, H, W, C2;
    int relu_a, relu_b;
};

struct TileG {
    int NB, TH, IHt;          // images, output rows per block; staged input rows
    int LW, IMG, PLANE, XO;   // LDS row pitch, floats per image / per channel, column of input column 0
    int row_blocks, tiles;
    int CPGa, KQ;             // channels per merged group, 16-channel chunks per merged group
    int pieces_log2;          // 16-byte pieces per staged row, rounded up to a power of two (log2)
    unsigned m_IHt, m_NB, m_ppi, m_W, m_rowb;
    unsigned x_bytes, d_bytes, y_bytes, wa_bytes, wb_bytes;
};
static_assert(sizeof(GpwParams) <= sizeof(((GpwPlan *)0)->params), "plan storage too small");
static_assert(sizeof(TileG) <= sizeof(((GpwPlan *)0)->tile), "plan storage too small");

__device__ __forceinline__ void gpw_transpose(f32x4 &a) {
    // register i, lane group r <- register r, lane group i (see the header)
    unsigned a0 = __float_as_uint(a.x), a1 = __float_as_uint(a.y), a2 = __float_as_uint(a.z), a3 = __float_as_uint(a.w);
    const auto p01 = __builtin_amdgcn_permlane16_swap(a0, a1, false, false);
    const auto p23 = __builtin_amdgcn_permlane16_swap(a2, a3, false, false);
    const auto q02 = __builtin_amdgcn_permlane32_swap(p01[0], p23[0], false, false);
    const auto q13 = __builtin_amdgcn_permlane32_swap(p01[1], p23[1], false, false);
    a = f32x4{__uint_as_float(q02[0]), __uint_as_float(q13[0]), __uint_as_float(q02[1]), __uint_as_float(q13[1])};
}

// CT = C / 16 filter tiles of the grouped layer, MTA of them per merged group, KT = C2 / 16
// filter tiles of the pointwise layer, S = stride of the grouped layer.
template <int CT, int MTA, int KT, int S>
__global__ __launch_bounds__(256, 2) void conv_gpw(GpwParams p, TileG t) {
    constexpr int NT = 256, GA = CT / MTA;
    extern __shared__ f32x4 smem4[];
    float *xs = reinterpret_cast<float *>(smem4);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned HWd = p.Hd * p.Wd, HW = p.H * p.W;
    const int ppi = t.TH * p.W, tot = t.NB * ppi;

    const unsigned tg = blockIdx.x;
    const unsigned ib = fast_div(tg, t.m_rowb);
    const int rb = tg - ib * t.row_blocks;
    const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - 1;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rwa = make_rsrc(p.wa, t.wa_bytes);
    const __amdgpu_buffer_rsrc_t rwb = make_rsrc(p.wb, t.wb_bytes);

    // ---- the block's input tile: every channel, NB images, IHt rows with a zero halo.  Eight
    // 16-byte pieces per thread are requested before the first of them is written to LDS, so that
    // their latencies overlap. -------------------------------------------------------------------
    {
        const int rows = p.C * t.NB * t.IHt, npiece = 1 << t.pieces_log2, wq = p.Wd / 4;
        const int total = rows << t.pieces_log2;
        for (int i0 = tid; i0 < total; i0 += 8 * NT) {
            f32x4 v[8];
            float *dst[8];
            int kind[8];   // 0: nothing, 1: a piece of a row, 2: the row's halo columns
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * NT;
                const int row = i >> t.pieces_log2, pc = i & (npiece - 1);
                const int cimg = fast_div(row, t.m_IHt), r = row - cimg * t.IHt;
                const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
                dst[k] = xs + c * t.PLANE + img * t.IMG + r * t.LW;
                kind[k] = i >= total ? 0 : pc < wq ? 1 : pc == wq ? 2 : 0;
                const int ih = ih0 + r;
                const bool ok = kind[k] == 1 && n0 + img < p.N && (unsigned)ih < (unsigned)p.Hd;
                const unsigned off = ((((unsigned)(n0 + img) * p.C + c) * p.Hd + ih) * p.Wd + pc * 4) * 4u;
                v[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? off : kOob, 0, 0));
                dst[k] += kind[k] == 1 ? t.XO + pc * 4 : 0;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (kind[k] == 1) {
                    *reinterpret_cast<f32x4 *>(dst[k]) = v[k];
                } else if (kind[k] == 2) {   // halo columns: never written by the copies
                    for (int x = 0; x < t.XO; ++x) dst[k][x] = 0.f;
                    for (int x = t.XO + p.Wd; x < t.LW; ++x) dst[k][x] = 0.f;
                }
            }
        }
    }

    // ---- this lane's pixel -----------------------------------------------------------------------
    const int q = wave * 16 + (lane & 15);
    const int qq = q < tot ? q : 0;
    const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
    const int r = fast_div(rem, t.m_W), col = rem - r * p.W;
    const bool live = q < tot && n0 + img < p.N && oh0 + r < p.H;
    // word offset of (channel lane/16, this pixel's window origin) in the tile
    const int xbase = (lane >> 4) * t.PLANE + img * t.IMG + r * S * t.LW + (t.XO - 1) + col * S;
    // byte offset of (image, filter 4*(lane/16), pixel) in an output tensor with `planes` channels
    auto out_off = [&](int planes) -> unsigned {
        return live ? ((((unsigned)(n0 + img) * planes + 4 * (lane >> 4)) * p.H + oh0 + r) * p.W + col) * 4u : kOob;
    };

    __syncthreads();

    // ---- stage A: grouped 3x3, all merged groups side by side (CT independent accumulator tiles) ---
    f32x4 D[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) D[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        const float *xg = xs + xbase;
        const int nquads = 9 * t.KQ;
        // operand quads of tile ct = ga * MTA + mt: section [ga][quad][mt][lane][4]
        f32x4 A[2][CT];
        const unsigned abase = (unsigned)lane * 16u;
        auto load_a = [&](int quad, f32x4(&dst)[CT]) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)   // past the last quad: out of range, zeros that are not used
                dst[ct] = __builtin_bit_cast(
                    f32x4, __builtin_amdgcn_raw_buffer_load_b128(rwa, quad < nquads ? abase : kOob,
                                                                 (((ct / MTA) * nquads + quad) * MTA + ct % MTA) * 1024, 0));
        };
        // one chunk of 16 channels of every group: 36 k-steps (4 channels at one tap each); P0: the
        // register set that holds the chunk's first quad (nine quads per chunk, so it alternates)
        auto chunk = [&](int kc, auto P0) {
            constexpr int par = decltype(P0)::value;
            const float *xc = xg + kc * 16 * t.PLANE;
#pragma unroll
            for (int qd = 0; qd < 9; ++qd) {
                load_a(kc * 9 + qd + 1, A[(par + qd + 1) & 1]);   // the next quad travels while this one multiplies
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ks = qd * 4 + e, cb = ks / 9, tap = ks % 9;
                    float bop[GA];
#pragma unroll
                    for (int ga = 0; ga < GA; ++ga)
                        bop[ga] = xc[(ga * t.CPGa + cb * 4) * t.PLANE + (tap / 3) * t.LW + tap % 3];
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
                        D[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(A[(par + qd) & 1][ct][e], bop[ct / MTA], D[ct], 0, 0, 0);
                }
            }
        };
        load_a(0, A[0]);
        for (int kc = 0; kc < t.KQ; kc += 2) {
            chunk(kc, std::integral_constant<int, 0>());
            if (kc + 1 < t.KQ) chunk(kc + 1, std::integral_constant<int, 1>());
        }
    }
    {
        const __amdgpu_buffer_rsrc_t rd = make_rsrc(p.d ? p.d : p.y, p.d ? t.d_bytes : 0u);
        const unsigned doff = p.d ? out_off(p.C) : kOob;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            if (p.relu_a) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) D[ct][rr] = fmaxf(D[ct][rr], 0.f);
            }
            if (p.d) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(D[ct][rr]), rd, doff, (ct * 16 + rr) * HW * 4, 0);
            }
            gpw_transpose(D[ct]);
        }
    }

    // ---- stage B: pointwise, D from registers ------------------------------------------------------
    f32x4 Y[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) Y[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        f32x4 A2[2][KT];
        const unsigned bbase = (unsigned)lane * 16u;
        auto load_b = [&](int kq, f32x4(&dst)[KT]) {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
                dst[kt] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                        rwb, kq < CT ? bbase : kOob, (kq * KT + kt) * 1024, 0));
        };
        load_b(0, A2[0]);
#pragma unroll
        for (int kq = 0; kq < CT; ++kq) {
            load_b(kq + 1, A2[(kq + 1) & 1]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
                    Y[kt] = __builtin_amdgcn_mfma_f32_16x16x4f32(A2[kq & 1][kt][e], D[kq][e], Y[kt], 0, 0, 0);
        }
    }

    // ---- epilogue: optional residual and ReLU, NCHW stores -----------------------------------------
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const unsigned yoff = out_off(p.C2);
    if (p.res) {
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int rr4 = 0; rr4 < 4; ++rr4)
                Y[kt][rr4] += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, yoff, (kt * 16 + rr4) * HW * 4, 0));
    }
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int rr4 = 0; rr4 < 4; ++rr4) {
            float v = Y[kt][rr4];
            if (p.relu_b) v = fmaxf(v, 0.f);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), ry, yoff, (kt * 16 + rr4) * HW * 4, 0);
        }
    (void)HWd;
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kLdsGpw = 64 * 1024;   // two blocks per compute unit

bool planG_tile(const GpwParams &p, int stride, const PackGeom &ga, TileG *out) {
    TileG t{};
    ConvParams q{};
    q.N = p.N;
    q.Hout = p.H;
    q.Wout = p.W;
    if (!split_pixels(q, 64, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * stride + 3;
    t.XO = 4;
    t.LW = round_up(t.XO + p.Wd + 1, 4);
    t.IMG = t.IHt * t.LW;
    // the four lane groups of a B-operand read are one channel apart: a pitch of 16 mod 32 floats
    // puts the two groups that are read in the same cycle on disjoint banks
    t.PLANE = round_up(t.NB * t.IMG, 32) + 16;
    if ((size_t)p.C * t.PLANE * sizeof(float) > kLdsGpw) return false;
    t.row_blocks = (p.H + t.TH - 1) / t.TH;
    const long tiles = (long)t.row_blocks * ((p.N + t.NB - 1) / t.NB);
    if (tiles > 2147483647L / 4) return false;
    t.tiles = (int)tiles;
    t.CPGa = ga.qk_CPG;
    t.KQ = ga.qk_CPG / 16;
    t.pieces_log2 = 0;
    while ((1 << t.pieces_log2) < p.Wd / 4 + 1) ++t.pieces_log2;
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.W);
    t.m_W = div_magic(p.W);
    t.m_rowb = div_magic(t.row_blocks);
    const double xb = (double)p.N * p.C * p.Hd * p.Wd * 4, db = (double)p.N * p.C * p.H * p.W * 4;
    const double yb = (double)p.N * p.C2 * p.H * p.W * 4;
    if (xb >= (double)kOob || db >= (double)kOob || yb >= (double)kOob) return false;
    if ((double)p.C * t.NB * t.IHt * t.IHt >= 4.0e9 || (double)tiles * t.row_blocks >= 4.0e9 || t.TH * p.W >= 65536 ||
        (double)p.C * t.NB * t.IHt * 64 >= 2.0e9)
        return false;
    t.x_bytes = (unsigned)xb;
    t.d_bytes = (unsigned)db;
    t.y_bytes = (unsigned)yb;
    *out = t;
    return true;
}

template <int CT, int MTA, int KT>
hipError_t launchG_s(const GpwParams &p, const TileG &t, int stride, hipStream_t s) {
    const size_t lds = (size_t)p.C * t.PLANE * sizeof(float);
    if (stride == 1) hipLaunchKernelGGL((conv_gpw<CT, MTA, KT, 1>), dim3(t.tiles), dim3(256), lds, s, p, t);
    else hipLaunchKernelGGL((conv_gpw<CT, MTA, KT, 2>), dim3(t.tiles), dim3(256), lds, s, p, t);
    return hipGetLastError();
}

template <int CT, int MTA>
hipError_t launchG_kt(int kt, const GpwParams &p, const TileG &t, int stride, hipStream_t s) {
    switch (kt) {
    case 2: return launchG_s<CT, MTA, 2>(p, t, stride, s);
    case 4: return launchG_s<CT, MTA, 4>(p, t, stride, s);
    case 8: return launchG_s<CT, MTA, 8>(p, t, stride, s);
    }
    return hipErrorNotSupported;
}

hipError_t launchG(int ct, int mta, int kt, const GpwParams &p, const TileG &t, int stride, hipStream_t s) {
    switch (ct * 16 + mta) {
    case 2 * 16 + 1: return launchG_kt<2, 1>(kt, p, t, stride, s);
    case 2 * 16 + 2: return launchG_kt<2, 2>(kt, p, t, stride, s);
    case 4 * 16 + 1: return launchG_kt<4, 1>(kt, p, t, stride, s);
    case 4 * 16 + 2: return launchG_kt<4, 2>(kt, p, t, stride, s);
    case 4 * 16 + 4: return launchG_kt<4, 4>(kt, p, t, stride, s);
    case 8 * 16 + 1: return launchG_kt<8, 1>(kt, p, t, stride, s);
    case 8 * 16 + 2: return launchG_kt<8, 2>(kt, p, t, stride, s);
    case 8 * 16 + 4: return launchG_kt<8, 4>(kt, p, t, stride, s);
    case 8 * 16 + 8: return launchG_kt<8, 8>(kt, p, t, stride, s);
    }
    return hipErrorNotSupported;
}

}  // namespace

bool gpw_enabled() {
    const char *on = std::getenv("GSPC_GPW");
    return on && on[0] == '1';
}

// layers[first], layers[first + 1]: grouped 3x3 (pad 1, stride 1 | 2, fp32, Cin = Cout of 32, 64 or
// 128 channels, not depthwise) whose result feeds an ungrouped 1x1 fp32 convolution with 32, 64 or
// 128 filters.  Returns 2 when the pair runs as one kernel: the feature is switched on (see below), both
// handles hold a quad-k section and the launch has at least one wave per SIMD (a wave carries every filter of its 16 pixels, so the
// parallelism is in the pixels; small launches stay two kernels, whose blocks split the filters).
// The grouped result is written to its buffer only if the rest of the chain can still see it.
int plan_gpw(const gspc_layer_t *layers, int first, int count, void *const *bufs, GpwPlan *out) {
    // Off unless GSPC_GPW=1 (read at every call, so a process can switch it): measured against the
    // pair as two kernels it does not pay yet.  Both of its stages are plain 16x16x4 products, while
    // the separate grouped layer runs Winograd F(2x2, 3x3) (g <= 4) or the 4x4x1 kernel on unmerged
    // groups (g >= 8) and so executes 2-4 times fewer multiplications; the launch and the round trip
    // this kernel saves are worth less than that (32 channels, 32x32, batch 64: 20.1 against 19.5 us
    // at g = 2, 19.7 against 17.7 us at g = 8; batch 256: 55 against 40-51 us).
    if (!gpw_enabled() || count < 2) return 0;
    const char *mw = std::getenv("GSPC_GPW_MIN_WAVES");
    const long min_waves = mw ? std::atol(mw) : 4L * kNumCU;
    const gspc_layer_t &A = layers[first], &B = layers[first + 1];
    if (A.op != GSPC_OP_CONV || B.op != GSPC_OP_CONV || !A.w || !B.w) return 0;
    if (A.w->dtype != GSPC_F32 || B.w->dtype != GSPC_F32) return 0;
    if (A.KH != 3 || A.KW != 3 || A.pad != 1 || (A.stride != 1 && A.stride != 2) || A.Cout != A.Cin || A.src2 >= 0 ||
        A.groups == A.Cin)
        return 0;
    const int H = (A.H + 2 - 3) / A.stride + 1, W = (A.W + 2 - 3) / A.stride + 1;
    if (B.KH != 1 || B.KW != 1 || B.pad != 0 || B.stride != 1 || B.groups != 1 || B.src != A.dst || B.N != A.N ||
        B.Cin != A.Cout || B.H != H || B.W != W)
        return 0;
    if (B.dst == A.dst || B.dst == A.src || B.src2 == A.dst) return 0;
    const PackGeom &ga = A.w->geom, &gb = B.w->geom;
    if (!ga.qk_bytes || !gb.qk_bytes || A.W % 4) return 0;
    const int ct = A.Cin / 16, mta = ga.qk_KPG / 16, kt = B.Cout / 16;
    if ((ct != 2 && ct != 4 && ct != 8) || ct % mta || (kt != 2 && kt != 4 && kt != 8))
        return 0;
    auto misaligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) != 0; };
    if (misaligned(bufs[A.src])) return 0;
    if ((long)A.N * H * W < 16 * min_waves) return 0;

    GpwParams p{};
    p.x = static_cast<const float *>(bufs[A.src]);
    p.wa = reinterpret_cast<const float *>(static_cast<const char *>(A.w->dev) + ga.qk_offset);
    p.wb = reinterpret_cast<const float *>(static_cast<const char *>(B.w->dev) + gb.qk_offset);
    p.y = static_cast<float *>(bufs[B.dst]);
    p.res = B.src2 >= 0 ? static_cast<const float *>(bufs[B.src2]) : nullptr;
    p.N = A.N; p.C = A.Cin; p.Hd = A.H; p.Wd = A.W; p.H = H; p.W = W; p.C2 = B.Cout;
    p.relu_a = (A.flags & GSPC_FLAG_RELU) ? 1 : 0;
    p.relu_b = (B.flags & GSPC_FLAG_RELU) ? 1 : 0;
    bool keep = true;   // is the grouped result visible after the pair?
    for (int m = first + 2; m < first + count; ++m) {
        const gspc_layer_t &L = layers[m];
        if (L.src == A.dst || L.src2 == A.dst) break;
        if (L.dst == A.dst) {
            keep = false;
            break;
        }
    }
    p.d = keep ? static_cast<float *>(bufs[A.dst]) : nullptr;
    TileG t;
    if (!planG_tile(p, A.stride, ga, &t)) return 0;
    if ((double)ga.qk_bytes >= (double)kOob || (double)gb.qk_bytes >= (double)kOob) return 0;
    t.wa_bytes = (unsigned)ga.qk_bytes;
    t.wb_bytes = (unsigned)gb.qk_bytes;
    out->ct = ct;
    out->mta = mta;
    out->kt = kt;
    out->stride = A.stride;
    std::memcpy(out->params, &p, sizeof(p));
    std::memcpy(out->tile, &t, sizeof(t));
    return 2;
}

hipError_t launch_gpw(const GpwPlan &plan, hipStream_t s, const char **name) {
    GpwParams p;
    TileG t;
    std::memcpy(&p, plan.params, sizeof(p));
    std::memcpy(&t, plan.tile, sizeof(t));
    *name = intern_name("conv_gpw<" + std::to_string(plan.ct) + "," + std::to_string(plan.mta) + "," +
                        std::to_string(plan.kt) + "," + std::to_string(plan.stride) + ">");
    return launchG(plan.ct, plan.mta, plan.kt, p, t, plan.stride, s);
}

}  // namespace gspc
