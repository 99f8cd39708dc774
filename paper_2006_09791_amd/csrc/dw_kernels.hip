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
//
// For the plane widths of the MobileNet / ResNet tails (WT = 28, 14, 7) a thread produces a whole
// output row: three tile rows pass through registers once, no index arithmetic per output, and
// the row leaves as 16-, 8- or 4-byte stores; other widths take one output per thread and step.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

struct TileD {
    int PB;                 // planes per block (4, 8, ..., 64)
    int LWp, PL;            // tile row pitch (W+2) and floats per plane tile ((H+2)*(W+2), rounded up to 4)
    int HW, HoWo;
    unsigned planes;        // N * C
    unsigned m_HW, m_W, m_HoWo, m_Wout, m_C, m_Hout;
    unsigned x_bytes, y_bytes, w_bytes;
};

constexpr int kDwSlots = 8;   // 16-byte loads per thread: 32 KB of tiles at most

template <int S, int WT>
__global__ __launch_bounds__(256) void conv_direct_dw(ConvParams p, TileD t) {
    extern __shared__ f32x4 smem4[];
    float *tile = reinterpret_cast<float *>(smem4);
    float *wl = tile + t.PB * t.PL;   // [plane][9]
    const int tid = threadIdx.x;
    const unsigned plane0 = blockIdx.x * t.PB;
    const int np = (int)(t.planes - plane0 < (unsigned)t.PB ? t.planes - plane0 : (unsigned)t.PB);

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);

    // ---- the block's planes: one contiguous piece of np*HW floats, requested first so that the
    // memory latency passes while the tiles are cleared.  Elements past the tensor's end read
    // as zero (the range check covers the vector offset) and are not used. ----
    const int total = np * t.HW;
    const unsigned gbase = plane0 * t.HW * 4;   // 16-byte aligned: PB is a multiple of 4
    f32x4 pin[kDwSlots];
#pragma unroll
    for (int k = 0; k < kDwSlots; ++k) {
        const int e4 = (tid + k * 256) * 4;
        pin[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, e4 < total ? gbase + e4 * 4 : kOob, 0, 0));
    }
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
#pragma unroll
    for (int k = 0; k < kDwSlots; ++k) {
        const int e4 = (tid + k * 256) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = e4 + i;
            if (e < total) {
                const int pl = fast_div(e, t.m_HW), r = e - pl * t.HW;
                const int h = fast_div(r, t.m_W), w = r - h * p.W;
                tile[pl * t.PL + (h + 1) * t.LWp + (w + 1)] = pin[k][i];
            }
        }
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    if constexpr (WT > 0) {
        // ---- a thread per output row of a plane ----
        constexpr int WO = (WT - 1) / S + 1, LW = WT + 2;
        const int rows = np * p.Hout;
        for (int row = tid; row < rows; row += 256) {
            const int pl = fast_div(row, t.m_Hout), oh = row - pl * p.Hout;
            float w[9];
#pragma unroll
            for (int k = 0; k < 9; ++k) w[k] = wl[pl * 9 + k];
            float acc[WO];
#pragma unroll
            for (int x = 0; x < WO; ++x) acc[x] = 0.f;
            const float *ip = tile + pl * t.PL + oh * S * LW;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                float xr[LW];
                if (LW % 2 == 0) {   // tile rows start on 8-byte boundaries when the pitch is even
#pragma unroll
                    for (int x = 0; x < LW; x += 2) {
                        const float2 v = *reinterpret_cast<const float2 *>(ip + kh * LW + x);
                        xr[x] = v.x;
                        xr[x + 1] = v.y;
                    }
                } else {
#pragma unroll
                    for (int x = 0; x < LW; ++x) xr[x] = ip[kh * LW + x];
                }
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                    for (int x = 0; x < WO; ++x) acc[x] = fmaf(xr[x * S + kw], w[kh * 3 + kw], acc[x]);
            }
            const unsigned ob = ((plane0 + pl) * t.HoWo + oh * WO) * 4;
            constexpr int VW = WO % 4 == 0 ? 4 : WO % 2 == 0 ? 2 : 1;   // the row start is VW*4-byte aligned
#pragma unroll
            for (int x = 0; x < WO; x += VW) {
                if (VW == 4) {
                    f32x4 v = f32x4{acc[x], acc[x + 1], acc[x + 2], acc[x + 3]};
                    if (p.res) v += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, ob + x * 4, 0, 0));
                    if (p.relu) v = f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), ry, ob + x * 4, 0, 0);
                } else if (VW == 2) {
                    float a0 = acc[x], a1 = acc[x + 1];
                    if (p.res) {
                        const u32x2 rv = __builtin_amdgcn_raw_buffer_load_b64(rr, ob + x * 4, 0, 0);
                        a0 += __uint_as_float(rv.x);
                        a1 += __uint_as_float(rv.y);
                    }
                    if (p.relu) {
                        a0 = fmaxf(a0, 0.f);
                        a1 = fmaxf(a1, 0.f);
                    }
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{__float_as_uint(a0), __float_as_uint(a1)}, ry, ob + x * 4, 0, 0);
                } else {
                    float a0 = acc[x];
                    if (p.res) a0 += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, ob + x * 4, 0, 0));
                    if (p.relu) a0 = fmaxf(a0, 0.f);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a0), ry, ob + x * 4, 0, 0);
                }
            }
        }
        return;
    }
    // ---- any width: 256 / PB threads per plane (PB is a power of two), so that a thread keeps its
    // plane's nine weights in registers; the lanes of a plane produce consecutive elements ----
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
    // measured: 8 planes per block for planes of 28x28 and more (32 threads per plane: 128-byte
    // store segments), 16 for 14x14, 32 for smaller ones
    static const int pb_force = std::getenv("GSPC_DW_PB") ? std::atoi(std::getenv("GSPC_DW_PB")) : 0;   // tuning aid
    const int pb_cap = pb_force ? pb_force : (t.HW >= 512 ? 8 : t.HW >= 128 ? 16 : 32);
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
    t.m_Hout = div_magic(p.Hout);
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    static_assert(sizeof(TileD) <= sizeof(out->data), "plan storage too small");
    std::memcpy(out->data, &t, sizeof(t));
    return true;
}

namespace {

template <int S, int WT>
hipError_t launch_dw_inst(const ConvParams &p, const TileD &t, hipStream_t s) {
    const size_t lds = ((size_t)t.PB * t.PL + (size_t)t.PB * 9 + 4) * sizeof(float);
    const dim3 grid((t.planes + t.PB - 1) / t.PB);
    hipLaunchKernelGGL((conv_direct_dw<S, WT>), grid, dim3(256), lds, s, p, t);
    return hipGetLastError();
}

// Measured at N = 256: a thread per output row pays for stride 2 at widths 28 and 7 (the row's
// few outputs leave in one or two stores); for stride 1 and for width 14 the per-plane split is
// as fast or faster.
inline int dw_row_width(const ConvParams &p) {
    static const bool generic = std::getenv("GSPC_DW_GENERIC") != nullptr;   // tuning aid
    return (!generic && p.stride == 2 && (p.W == 28 || p.W == 7)) ? p.W : 0;
}

}  // namespace

hipError_t launch_dw_planes(const ConvParams &p, const DwPlan &plan, hipStream_t s, const char **name) {
    TileD t;
    std::memcpy(&t, plan.data, sizeof(t));
    const int wt = dw_row_width(p);
    *name = intern_name("conv_direct_dw<" + std::to_string(p.stride) + "," + std::to_string(wt) + ",f32>");
    if (wt == 28) return launch_dw_inst<2, 28>(p, t, s);
    if (wt == 7) return launch_dw_inst<2, 7>(p, t, s);
    return p.stride == 1 ? launch_dw_inst<1, 0>(p, t, s) : launch_dw_inst<2, 0>(p, t, s);
}

}  // namespace gspc
