// Depthwise 3x3 convolution (g = Cin = Cout, the G(N) end of the paper's sweep,
// Section IV of arXiv 2006.09791) for small planes of any width.
//
// With one channel per group the input planes of consecutive (image, channel)
// pairs are consecutive in NCHW memory, and so are the output planes: a block
// takes PB whole planes as one contiguous piece, copies it with 16-byte loads
// into zero-haloed LDS tiles (the paper's input reshape, here a re-pitch from
// W to W+2 columns), and every thread then produces output elements that are
// consecutive across the wavefront, so the stores are contiguous as well.
// Nothing depends on W being a multiple of 4 or on the plane filling a
// wavefront (14x14 and 7x7 planes, odd strides of planes).  HBM-bound.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

struct TileD {
    int PB;                 // planes per block (4, 8, ..., 64)
    int LWp, PL;            // tile row pitch (W+2) and floats per plane tile ((H+2)*(W+2), rounded up to 4)
    int HW, HoWo;
    unsigned planes;        // N * C
    unsigned m_HW, m_W, m_HoWo, m_Wout, m_C;
    unsigned x_bytes, y_bytes, w_bytes;
};

template <int S>
__global__ __launch_bounds__(256) void conv_direct_dw(ConvParams p, TileD t) {
    extern __shared__ f32x4 smem4[];
    float *tile = reinterpret_cast<float *>(smem4);
    float *wl = tile + t.PB * t.PL;   // [plane][9]
    const int tid = threadIdx.x;
    const unsigned plane0 = blockIdx.x * t.PB;
    const int np = (int)(t.planes - plane0 < (unsigned)t.PB ? t.planes - plane0 : (unsigned)t.PB);

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);

    // ---- clear the tiles (the halo must be zero; the interior is overwritten) ----
    {
        const int n4 = t.PB * t.PL / 4;
        for (int i = tid; i < n4; i += 256) smem4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // ---- filters: direct section [g][9][KPGd], filter 0 of group c ------------
    for (int i = tid; i < np * 9; i += 256) {
        const unsigned pl = fast_div(i, 0x1c71c71du);   // i / 9, exact for i < 2^16
        const unsigned k = i - pl * 9;
        const unsigned pg = plane0 + pl;
        const unsigned c = pg - fast_div(pg, t.m_C) * p.Cin;
        wl[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, ((c * 9 + k) * p.KPGd) * 4, 0, 0));
    }
    __syncthreads();
    // ---- the block's planes: one contiguous piece of np*HW floats ---------------
    {
        const int total = np * t.HW;
        const unsigned gbase = plane0 * t.HW * 4;   // 16-byte aligned: PB is a multiple of 4
        for (int e4 = tid * 4; e4 < total; e4 += 1024) {
            // elements past the tensor's end read as zero (the range check covers the vector offset)
            // and are not written
            const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, gbase + e4 * 4, 0, 0));
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int e = e4 + k;
                if (e < total) {
                    const int pl = fast_div(e, t.m_HW), r = e - pl * t.HW;
                    const int h = fast_div(r, t.m_W), w = r - h * p.W;
                    tile[pl * t.PL + (h + 1) * t.LWp + (w + 1)] = v[k];
                }
            }
        }
    }
    __syncthreads();
    // ---- outputs: 256 / PB threads per plane (PB is a power of two), so that a thread keeps its
    // plane's nine weights in registers; the lanes of a plane produce consecutive elements ----
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    const int tpp = 256 / t.PB, pl = tid / tpp, sub = tid - pl * tpp;
    if (pl < np) {
        float w[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = wl[pl * 9 + k];
        const float *tp = tile + pl * t.PL;
        const unsigned obase = (plane0 + pl) * t.HoWo * 4;
        for (int o = sub; o < t.HoWo; o += tpp) {
            const int oh = fast_div(o, t.m_Wout), ow = o - oh * p.Wout;
            const float *ip = tp + oh * S * t.LWp + ow * S;
            float acc = 0.f;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) acc = fmaf(ip[kh * t.LWp + kw], w[kh * 3 + kw], acc);
            if (p.res) acc += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, obase + o * 4, 0, 0));
            if (p.relu) acc = fmaxf(acc, 0.f);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc), ry, obase + o * 4, 0, 0);
        }
    }
}

bool plan_dw_planes(const ConvParams &p, DwPlan *out) {
    static const bool off = std::getenv("GSPC_NO_DWPLANES") != nullptr;   // tuning aid
    if (off || p.CPG != 1 || p.KPG != 1 || p.in_bf16 || p.KH != 3 || p.KW != 3 || p.pad != 1 ||
        (p.stride != 1 && p.stride != 2))
        return false;
    TileD t{};
    t.LWp = p.W + 2;
    t.PL = round_up((p.H + 2) * t.LWp, 4);
    t.HW = p.H * p.W;
    t.HoWo = p.Hout * p.Wout;
    // as many planes as fit 32 KB of tiles, at most 64, a multiple of 4
    int pb = (32 * 1024 / 4) / t.PL;
    // measured: 8 planes per block for planes of 14x14 and more (32 threads per plane: 128-byte
    // store segments), 32 for smaller ones
    static const int pb_force = std::getenv("GSPC_DW_PB") ? std::atoi(std::getenv("GSPC_DW_PB")) : 0;   // tuning aid
    const int pb_cap = pb_force ? pb_force : (t.HW >= 128 ? 8 : 32);
    pb = pb > pb_cap ? pb_cap : pb;
    if (pb < 4) return false;
    {
        int q = 4;   // a power of two: the block's 256 threads divide evenly over the planes
        while (2 * q <= pb) q *= 2;
        pb = q;
    }
    const double planes = (double)p.N * p.Cin;
    // small batches: fewer planes per block rather than idle compute units
    const long spread = (long)(planes / (2 * kNumCU));
    while (pb > 4 && spread < pb) pb /= 2;
    t.PB = pb;
    const double xb = planes * t.HW * 4, yb = planes * t.HoWo * 4, wb = (double)p.groups * 9 * p.KPGd * 4;
    if (planes >= 2147483648.0 || xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    // fast_div exactness: numerator * divisor < 2^32 at each step
    if ((double)pb * t.HW * t.HW >= 4.29e9 || (double)pb * t.HoWo * t.HoWo >= 4.29e9 ||
        planes * p.Cin >= 4.29e9 || pb * 9 >= 65536)
        return false;
    t.planes = (unsigned)planes;
    t.m_HW = div_magic(t.HW);
    t.m_W = div_magic(p.W);
    t.m_HoWo = div_magic(t.HoWo);
    t.m_Wout = div_magic(p.Wout);
    t.m_C = div_magic(p.Cin);
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    static_assert(sizeof(TileD) <= sizeof(out->data), "plan storage too small");
    std::memcpy(out->data, &t, sizeof(t));
    return true;
}

hipError_t launch_dw_planes(const ConvParams &p, const DwPlan &plan, hipStream_t s, const char **name) {
    TileD t;
    std::memcpy(&t, plan.data, sizeof(t));
    const size_t lds = ((size_t)t.PB * t.PL + (size_t)t.PB * 9 + 4) * sizeof(float);
    const dim3 grid((t.planes + t.PB - 1) / t.PB);
    if (p.stride == 1) {
        *name = "conv_direct_dw<1,f32>";
        hipLaunchKernelGGL(conv_direct_dw<1>, grid, dim3(256), lds, s, p, t);
    } else {
        *name = "conv_direct_dw<2,f32>";
        hipLaunchKernelGGL(conv_direct_dw<2>, grid, dim3(256), lds, s, p, t);
    }
    return hipGetLastError();
}

}  // namespace gspc
