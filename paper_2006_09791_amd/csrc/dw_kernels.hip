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
//
// Launches that fill the chip on 56x56, 28x28, 14x14 and 7x7 planes take conv_dw_wave instead
// (further down): whole planes per wavefront, no block-level barrier, every global and almost
// every LDS access 16 bytes wide; on 112x112 planes conv_dw_band does the same with a band of 16
// rows per wavefront.  The block form above keeps the small launches (it shrinks its tiles to
// spread over the chip) and the other plane sizes.
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


// ---- whole planes per wavefront -------------------------------------------------------------
// For the square planes of the network tails (28x28, 14x14, 7x7) a wavefront takes G consecutive
// planes by itself: their floats are one contiguous, 16-byte aligned piece of the input and their
// outputs one contiguous piece of the output.  The piece is copied flat into a wave-private LDS
// region (16-byte loads and LDS writes, no re-pitch and no halo: the left and right padding
// columns are dropped from the unrolled sums at compile time, the top and bottom padding rows are
// selected to zero per lane), a lane reads the (R-1)*S + 3 input rows of its R output rows as one
// contiguous window into registers, multiplies them out, writes the R*Wout results back into the
// region at their flat output position (the region is reused: every lane has its window in
// registers by then), and the wave reads the results back 16 bytes per lane in flat order for
// coalesced stores (residual and ReLU applied there).  LDS operations of one wavefront execute in
// order, so no barrier is needed anywhere; memory clobbers keep the compiler from reordering the
// phases.  Per lane and R*Wout outputs this takes a few dozen wide LDS operations where the
// per-output form above takes nine 4-byte reads per output.
template <int S, int H, int W, int R, int CP = -1>
struct DwWaveGeom {
    static constexpr int Hout = (H - 1) / S + 1, Wout = (W - 1) / S + 1;
    static constexpr int HW = H * W, HoWo = Hout * Wout;
    static constexpr int LP = (Hout + R - 1) / R;           // lanes per plane (the last one may own fewer rows)
    static constexpr bool RAG = Hout % R != 0;
    static constexpr int pick_g() {
        for (int g = 64 / LP; g >= 1; --g)
            if ((g * HW) % 4 == 0 && (g * HoWo) % 4 == 0) return g;
        return 0;
    }
    static constexpr int G = pick_g();                      // planes per wavefront
    static constexpr int IN = G * HW, OUT = G * HoWo;       // floats per wavefront
    static constexpr int NSI = (IN / 4 + 63) / 64, NSO = (OUT / 4 + 63) / 64;
    static constexpr int NR = (R - 1) * S + 3;              // input rows of a lane's window
    static constexpr int FRONT = (W + 3) / 4 * 4;           // the first plane's row -1
    static constexpr int over = (LP * R - 1) * S + 2 - H;   // rows the last window reaches past its plane
    static constexpr int BACK = (over > 0 ? over : 0) * W;
    static constexpr int REGION = (FRONT + IN + BACK + 3) / 4 * 4;   // floats per wavefront
    static constexpr int VR = W % 4 == 0 ? 4 : W % 2 == 0 ? 2 : 1;   // window reads
    static constexpr int ao = RAG ? Wout : R * Wout;        // floats written at one aligned position
    static constexpr int VO = (ao % 4 == 0 && HoWo % 4 == 0) ? 4 : (ao % 2 == 0 && HoWo % 2 == 0) ? 2 : 1;
    // the nine weights of the wave's planes: fetched lane by lane (9 loads), or, when the wave has few planes,
    // as one flat list of G*9 values through LDS (NWS loads)
    static constexpr int NWS = (G * 9 + 63) / 64;
    static constexpr bool COOP = CP < 0 ? NWS <= 4 : CP != 0;
    static constexpr int WTS = COOP ? (G * 9 + 3) / 4 * 4 : 0;
    static constexpr int WAVE_FLOATS = REGION + WTS;
    static_assert(G > 0 && OUT <= IN, "unsupported shape");
};

struct TileW {
    unsigned chunks, planes, m_C;
    unsigned x_bytes, y_bytes, w_bytes;
};

template <int S, int H, int W, int R, int CP>
__global__ __launch_bounds__(256) void conv_dw_wave(ConvParams p, TileW t) {
    using Q = DwWaveGeom<S, H, W, R, CP>;
    extern __shared__ f32x4 smem4[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned chunk = blockIdx.x * 4 + wv;
    if (chunk >= t.chunks) return;   // wave-uniform; the kernel has no barriers
    float *reg = reinterpret_cast<float *>(smem4) + wv * Q::WAVE_FLOATS;
    float *data = reg + Q::FRONT;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);

    // ---- the wave's planes, requested first ----
    const unsigned gbase = chunk * (unsigned)(Q::IN * 4);
    f32x4 pin[Q::NSI];
#pragma unroll
    for (int j = 0; j < Q::NSI; ++j) {
        const int q = lane + 64 * j;
        pin[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, q * 4 < Q::IN ? gbase + q * 16 : kOob, 0, 0));
    }
    // ---- the lane's plane, rows and weights ----
    const bool active = lane < Q::G * Q::LP;
    const int la = active ? lane : 0;
    const int pl = Q::LP == 1 ? la : la / Q::LP;
    const int oh0 = Q::LP == 1 ? 0 : (la - pl * Q::LP) * R;
    float w[9];
    if constexpr (Q::COOP) {
        float *wts = reg + Q::REGION;
#pragma unroll
        for (int j = 0; j < Q::NWS; ++j) {
            const int i = lane + 64 * j;
            if (i < Q::G * 9) {
                const int wp = i / 9, k = i - wp * 9;
                unsigned pg = chunk * Q::G + wp;
                pg = pg < t.planes ? pg : t.planes - 1;
                const unsigned c = pg - fast_div(pg, t.m_C) * p.Cin;
                wts[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, ((c * 9 + k) * p.KPGd) * 4, 0, 0));
            }
        }
    } else {
        unsigned pg = chunk * Q::G + pl;
        pg = pg < t.planes ? pg : t.planes - 1;
        const unsigned c = pg - fast_div(pg, t.m_C) * p.Cin;
#pragma unroll
        for (int k = 0; k < 9; ++k)
            w[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, ((c * 9 + k) * p.KPGd) * 4, 0, 0));
    }
#pragma unroll
    for (int j = 0; j < Q::NSI; ++j) {
        const int q = lane + 64 * j;
        if (q * 4 < Q::IN) *reinterpret_cast<f32x4 *>(data + q * 4) = pin[j];
    }
    asm volatile("" ::: "memory");
    if constexpr (Q::COOP) {
        const float *wts = reg + Q::REGION;
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = wts[pl * 9 + k];
    }
    // ---- window: rows oh0*S - 1 .. oh0*S - 1 + NR - 1 of the plane ----
    float xr[Q::NR][W];
    {
        const int ih0 = oh0 * S - 1;
        const float *wp = data + pl * Q::HW + ih0 * W;
#pragma unroll
        for (int i = 0; i < Q::NR; ++i) {
            const bool valid = (unsigned)(ih0 + i) < (unsigned)H;
#pragma unroll
            for (int x = 0; x < W; x += Q::VR) {
                if constexpr (Q::VR == 4) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(wp + i * W + x);
                    xr[i][x] = valid ? v.x : 0.f;
                    xr[i][x + 1] = valid ? v.y : 0.f;
                    xr[i][x + 2] = valid ? v.z : 0.f;
                    xr[i][x + 3] = valid ? v.w : 0.f;
                } else if constexpr (Q::VR == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(wp + i * W + x);
                    xr[i][x] = valid ? v.x : 0.f;
                    xr[i][x + 1] = valid ? v.y : 0.f;
                } else {
                    const float v = wp[i * W + x];
                    xr[i][x] = valid ? v : 0.f;
                }
            }
        }
    }
    asm volatile("" ::: "memory");
    // ---- R rows of Wout outputs, written to their flat position in the region ----
    {
        float *op = data + pl * Q::HoWo + oh0 * Q::Wout;
        float acc[R * Q::Wout];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int ow = 0; ow < Q::Wout; ++ow) {
                float a = 0.f;
#pragma unroll
                for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        const int col = ow * S - 1 + kw;
                        if (col >= 0 && col < W) a = fmaf(xr[r * S + kh][col], w[kh * 3 + kw], a);
                    }
                acc[r * Q::Wout + ow] = a;
            }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            // without ragged rows the lane's R rows are written as one run
            if (active && (!Q::RAG || oh0 + r < Q::Hout)) {
#pragma unroll
                for (int x = 0; x < Q::Wout; x += (Q::RAG ? Q::VO : 1)) {
                    const int e = r * Q::Wout + x;
                    if (!Q::RAG && e % Q::VO != 0) continue;
                    if constexpr (Q::VO == 4) *reinterpret_cast<f32x4 *>(op + e) = f32x4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
                    else if constexpr (Q::VO == 2) *reinterpret_cast<float2 *>(op + e) = float2{acc[e], acc[e + 1]};
                    else op[e] = acc[e];
                }
            }
        }
    }
    asm volatile("" ::: "memory");
    // ---- flat read-back, residual, ReLU, 16-byte stores ----
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    const unsigned obase = chunk * (unsigned)(Q::OUT * 4);
#pragma unroll
    for (int j = 0; j < Q::NSO; ++j) {
        const int q = lane + 64 * j;
        if (q * 4 < Q::OUT) {
            f32x4 v = *reinterpret_cast<const f32x4 *>(data + q * 4);
            if (p.res) v += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, obase + q * 16, 0, 0));
            if (p.relu) v = f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), ry, obase + q * 16, 0, 0);
        }
    }
}

constexpr int kDwKind = 23, kDwInst = 22;   // plan slots: 1 = whole planes per wavefront, and its instance

// Instances of conv_dw_wave: (stride, plane edge, output rows per lane, weights through LDS), each the fastest of
// the forms measured at N = 256 (one row per lane except on 7x7 planes at stride 2; the 56x56 stride-2 layer
// is faster on the strip kernel and has no instance).
template <int I> struct DwWaveInst;
#define GSPC_DW_WAVE_INST(I, S_, E_, R_, CP_) \
    template <> struct DwWaveInst<I> { using Q = DwWaveGeom<S_, E_, E_, R_, CP_>; static constexpr int S = S_, E = E_, R = R_, CP = CP_; }
GSPC_DW_WAVE_INST(0, 1, 28, 1, 0);
GSPC_DW_WAVE_INST(1, 2, 28, 1, 0);
GSPC_DW_WAVE_INST(2, 1, 14, 1, 0);
GSPC_DW_WAVE_INST(3, 2, 14, 1, 0);
GSPC_DW_WAVE_INST(4, 1, 7, 1, 1);
GSPC_DW_WAVE_INST(5, 2, 7, 2, 0);
GSPC_DW_WAVE_INST(6, 1, 56, 1, 0);
constexpr int kDwWaveInsts = 7;

template <int I>
bool plan_dw_wave_inst(const ConvParams &p, DwPlan *out) {
    using T = DwWaveInst<I>;
    using Q = typename T::Q;
    if (p.stride != T::S || p.H != T::E || p.W != T::E) return false;
    const double planes = (double)p.N * p.Cin;
    const double chunks = (planes + Q::G - 1) / Q::G;
    // small launches stay on the block form, which shrinks its tiles to spread over the chip
    static const bool force = std::getenv("GSPC_DW_WAVE") != nullptr;   // tuning aid
    if (!force && chunks < 4.0 * 2 * kNumCU) return false;
    const double xb = planes * Q::HW * 4, yb = planes * Q::HoWo * 4, wb = (double)p.groups * 9 * p.KPGd * 4;
    const double slack = 4.0 * Q::IN * 4 + 65536;   // offsets past the tensor's end must not wrap
    if (planes >= 2147483648.0 || xb + slack >= (double)kOob || yb + slack >= (double)kOob || wb >= (double)kOob ||
        planes * p.Cin >= 4.29e9)
        return false;
    TileW t{};
    t.planes = (unsigned)planes;
    t.chunks = (unsigned)((t.planes + Q::G - 1) / Q::G);
    t.m_C = div_magic(p.Cin);
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    static_assert(sizeof(TileW) <= sizeof(int) * kDwInst, "plan storage too small");
    std::memcpy(out->data, &t, sizeof(t));
    out->data[kDwKind] = 1;
    out->data[kDwInst] = I;
    return true;
}

template <int I = 0>
bool plan_dw_wave(const ConvParams &p, DwPlan *out) {
    static const bool off = std::getenv("GSPC_NO_DWWAVE") != nullptr;   // tuning aid
    if (off) return false;
    if constexpr (I < kDwWaveInsts) return plan_dw_wave_inst<I>(p, out) || plan_dw_wave<I + 1>(p, out);
    else return false;
}

template <int I = 0>
hipError_t launch_dw_wave(int inst, const ConvParams &p, const TileW &t, hipStream_t s, const char **name) {
    if constexpr (I < kDwWaveInsts) {
        if (inst != I) return launch_dw_wave<I + 1>(inst, p, t, s, name);
        using T = DwWaveInst<I>;
        using Q = typename T::Q;
        *name = intern_name("conv_dw_wave<" + std::to_string(T::S) + "," + std::to_string(T::E) + "," + std::to_string(T::E) +
                            "," + std::to_string(T::R) + "," + std::to_string(T::CP) + ">");
        const size_t lds = (size_t)4 * Q::WAVE_FLOATS * sizeof(float);
        hipLaunchKernelGGL((conv_dw_wave<T::S, T::E, T::E, T::R, T::CP>), dim3((t.chunks + 3) / 4), dim3(256), lds, s, p, t);
        return hipGetLastError();
    } else {
        return hipErrorNotSupported;
    }
}

// ---- bands of rows per wavefront (planes too large for the form above) ---------------------------
// The same scheme for one band of BR output rows of one plane per wavefront: the (BR-1)*S + 3 input rows the
// band needs are contiguous in memory and are copied flat (the rows above the first and below the last band are
// other planes' rows, or lie outside the tensor and arrive as zeros: either way they are selected to zero).  A lane
// owns CW = Wout / NQ consecutive outputs of one row; its 3-row window is read with aligned 8- or 16-byte LDS reads
// that start VR floats to the left of its first column, the columns left of the plane and right of it are selected
// to zero.  The plane's nine weights are uniform over the wavefront and sit in scalar registers.
template <int S, int H, int W, int BR, int NQ>
struct DwBandGeom {
    static constexpr int Hout = (H - 1) / S + 1, Wout = (W - 1) / S + 1;
    static constexpr int NBD = Hout / BR;                    // bands per plane
    static constexpr int CW = Wout / NQ;                     // outputs per lane
    static constexpr int NRB = (BR - 1) * S + 3;             // input rows per band
    static constexpr int IN = NRB * W, OUT = BR * Wout;      // floats per band
    static constexpr int NSI = (IN / 4 + 63) / 64, NSO = (OUT / 4 + 63) / 64;
    static constexpr int VR = (CW * S) % 4 == 0 ? 4 : 2;     // alignment (floats) of a lane's first column
    static constexpr int WIN = (CW - 1) * S + 3;             // window columns
    static constexpr int XW = (VR - 1 + WIN + VR - 1) / VR * VR;   // floats read per window row
    static constexpr int REGION = (VR + IN + XW + 3) / 4 * 4;
    static constexpr int VO = CW % 4 == 0 ? 4 : CW % 2 == 0 ? 2 : 1;
    static_assert(Hout % BR == 0 && Wout % NQ == 0 && BR * NQ <= 64 && W % 4 == 0 && OUT % 4 == 0 &&
                      (Hout * Wout) % 4 == 0 && (CW * S) % 2 == 0 && VR >= 2,
                  "unsupported band shape");
};

template <int S, int H, int W, int BR, int NQ>
__global__ __launch_bounds__(256) void conv_dw_band(ConvParams p, TileW t) {
    using Q = DwBandGeom<S, H, W, BR, NQ>;
    extern __shared__ f32x4 smem4[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned chunk = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wv);
    if (chunk >= t.chunks) return;   // wave-uniform; the kernel has no barriers
    float *data = reinterpret_cast<float *>(smem4) + wv * Q::REGION + Q::VR;
    const unsigned plane = chunk / Q::NBD, band = chunk - plane * Q::NBD;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);

    // ---- the band's input rows, requested first (the row above the first band of the first plane has a
    // "negative" offset, which wraps to out of range and reads as zero) ----
    const int ihb = (int)band * (BR * S) - 1;   // first input row of the band
    const unsigned gbase = (plane * (unsigned)(H * W) + (unsigned)(ihb * W)) * 4u;
    f32x4 pin[Q::NSI];
#pragma unroll
    for (int j = 0; j < Q::NSI; ++j) {
        const int q = lane + 64 * j;
        pin[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, q * 4 < Q::IN ? gbase + q * 16 : kOob, 0, 0));
    }
    // ---- weights: uniform over the wave ----
    float w[9];
    {
        const unsigned c = plane - fast_div(plane, t.m_C) * p.Cin;
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = p.wd[(c * 9 + k) * p.KPGd];
    }
    const bool active = lane < BR * NQ;
    const int la = active ? lane : 0;
    const int r = la / NQ, qs = la - r * NQ;
#pragma unroll
    for (int j = 0; j < Q::NSI; ++j) {
        const int q = lane + 64 * j;
        if (q * 4 < Q::IN) *reinterpret_cast<f32x4 *>(data + q * 4) = pin[j];
    }
    asm volatile("" ::: "memory");
    // ---- window: 3 rows x XW floats from column qs*CW*S - VR ----
    float acc[Q::CW];
#pragma unroll
    for (int x = 0; x < Q::CW; ++x) acc[x] = 0.f;
    {
        const float *wp = data + (r * S) * W + qs * (Q::CW * S) - Q::VR;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const bool rvalid = (unsigned)(ihb + r * S + kh) < (unsigned)H;
            float xr[Q::XW];
#pragma unroll
            for (int x = 0; x < Q::XW; x += Q::VR) {
                if constexpr (Q::VR == 4) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(wp + kh * W + x);
                    xr[x] = v.x;
                    xr[x + 1] = v.y;
                    xr[x + 2] = v.z;
                    xr[x + 3] = v.w;
                } else {
                    const float2 v = *reinterpret_cast<const float2 *>(wp + kh * W + x);
                    xr[x] = v.x;
                    xr[x + 1] = v.y;
                }
            }
            // window column j is xr[j + VR - 1]; column 0 lies left of the plane for the first segment, the last one
            // right of it for the last segment of a stride-1 row
#pragma unroll
            for (int j = 0; j < Q::WIN; ++j) {
                bool ok = rvalid;
                if (j == 0) ok = ok && qs != 0;
                if (S == 1 && j == Q::WIN - 1) ok = ok && qs != NQ - 1;
                xr[j + Q::VR - 1] = ok ? xr[j + Q::VR - 1] : 0.f;
            }
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int x = 0; x < Q::CW; ++x) acc[x] = fmaf(xr[x * S + kw + Q::VR - 1], w[kh * 3 + kw], acc[x]);
        }
    }
    asm volatile("" ::: "memory");
    // ---- results to their flat position in the region (every lane has read its window) ----
    if (active) {
        float *op = data + r * Q::Wout + qs * Q::CW;
#pragma unroll
        for (int e = 0; e < Q::CW; e += Q::VO) {
            if constexpr (Q::VO == 4) *reinterpret_cast<f32x4 *>(op + e) = f32x4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
            else if constexpr (Q::VO == 2) *reinterpret_cast<float2 *>(op + e) = float2{acc[e], acc[e + 1]};
            else op[e] = acc[e];
        }
    }
    asm volatile("" ::: "memory");
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    const unsigned obase = (plane * (unsigned)(Q::Hout * Q::Wout) + band * (unsigned)Q::OUT) * 4u;
#pragma unroll
    for (int j = 0; j < Q::NSO; ++j) {
        const int q = lane + 64 * j;
        if (q * 4 < Q::OUT) {
            f32x4 v = *reinterpret_cast<const f32x4 *>(data + q * 4);
            if (p.res) v += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, obase + q * 16, 0, 0));
            if (p.relu) v = f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), ry, obase + q * 16, 0, 0);
        }
    }
}

template <int I> struct DwBandInst;
#define GSPC_DW_BAND_INST(I, S_, E_, BR_, NQ_) \
    template <> struct DwBandInst<I> { using Q = DwBandGeom<S_, E_, E_, BR_, NQ_>; static constexpr int S = S_, E = E_, BR = BR_, NQ = NQ_; }
// One instance, the only shape where the form measured faster than the strip kernel at N = 256: 112x112 stride 1
// (168 -> 144 and 316 -> 291 us for 32 and 64 channels).  Within 2 % either way: 112x112 stride 2 in bands of 14 rows;
// slower: 56x56 in bands of 14 rows (stride 1: 173 against 150 us for whole planes; stride 2: 107 against 100 us for
// the strip kernel), lanes of 14 instead of 28 outputs on 112x112 (169 us).
GSPC_DW_BAND_INST(0, 1, 112, 16, 4);
constexpr int kDwBandInsts = 1;

template <int I = 0>
bool plan_dw_band(const ConvParams &p, DwPlan *out) {
    if constexpr (I < kDwBandInsts) {
        using T = DwBandInst<I>;
        using Q = typename T::Q;
        const bool shape = p.stride == T::S && p.H == T::E && p.W == T::E;
        const double planes = (double)p.N * p.Cin, chunks = planes * Q::NBD;
        const double xb = planes * (T::E * T::E) * 4, yb = planes * (Q::Hout * Q::Wout) * 4, wb = (double)p.groups * 9 * p.KPGd * 4;
        const double slack = 4.0 * Q::IN * 4 + 65536;
        if (!shape || chunks < 4.0 * 2 * kNumCU || chunks >= 4.0e9 || xb + slack >= (double)kOob || yb + slack >= (double)kOob ||
            wb >= (double)kOob || planes * p.Cin >= 4.29e9)
            return plan_dw_band<I + 1>(p, out);
        TileW t{};
        t.planes = (unsigned)planes;
        t.chunks = (unsigned)chunks;
        t.m_C = div_magic(p.Cin);
        t.x_bytes = (unsigned)xb;
        t.y_bytes = (unsigned)yb;
        t.w_bytes = (unsigned)wb;
        std::memcpy(out->data, &t, sizeof(t));
        out->data[kDwKind] = 2;
        out->data[kDwInst] = I;
        return true;
    } else {
        return false;
    }
}

template <int I = 0>
hipError_t launch_dw_band(int inst, const ConvParams &p, const TileW &t, hipStream_t s, const char **name) {
    if constexpr (I < kDwBandInsts) {
        if (inst != I) return launch_dw_band<I + 1>(inst, p, t, s, name);
        using T = DwBandInst<I>;
        using Q = typename T::Q;
        *name = intern_name("conv_dw_band<" + std::to_string(T::S) + "," + std::to_string(T::E) + "," + std::to_string(T::E) +
                            "," + std::to_string(T::BR) + "," + std::to_string(T::NQ) + ">");
        const size_t lds = (size_t)4 * Q::REGION * sizeof(float);
        hipLaunchKernelGGL((conv_dw_band<T::S, T::E, T::E, T::BR, T::NQ>), dim3((t.chunks + 3) / 4), dim3(256), lds, s, p, t);
        return hipGetLastError();
    } else {
        return hipErrorNotSupported;
    }
}

bool plan_dw_planes(const ConvParams &p, DwPlan *out) {
    static const bool off = std::getenv("GSPC_NO_DWPLANES") != nullptr;   // tuning aid
    if (off || p.CPG != 1 || p.KPG != 1 || p.in_bf16 || p.KH != 3 || p.KW != 3 || p.pad != 1 ||
        (p.stride != 1 && p.stride != 2))
        return false;
    if (plan_dw_wave(p, out)) return true;
    {
        static const bool off = std::getenv("GSPC_NO_DWBAND") != nullptr;   // tuning aid
        if (!off && plan_dw_band(p, out)) return true;
    }
    out->data[kDwKind] = 0;
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
    static_assert(sizeof(TileD) <= sizeof(int) * kDwInst, "plan storage too small");
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
    if (plan.data[kDwKind] == 2) {
        TileW tw;
        std::memcpy(&tw, plan.data, sizeof(tw));
        return launch_dw_band(plan.data[kDwInst], p, tw, s, name);
    }
    if (plan.data[kDwKind] == 1) {
        TileW tw;
        std::memcpy(&tw, plan.data, sizeof(tw));
        return launch_dw_wave(plan.data[kDwInst], p, tw, s, name);
    }
    TileD t;
    std::memcpy(&t, plan.data, sizeof(t));
    const int wt = dw_row_width(p);
    *name = intern_name("conv_direct_dw<" + std::to_string(p.stride) + "," + std::to_string(wt) + ",f32>");
    if (wt == 28) return launch_dw_inst<2, 28>(p, t, s);
    if (wt == 7) return launch_dw_inst<2, 7>(p, t, s);
    return p.stride == 1 ? launch_dw_inst<1, 0>(p, t, s) : launch_dw_inst<2, 0>(p, t, s);
}

}  // namespace gspc
