// Depthwise 3x3 convolution fused with the pointwise 1x1 convolution that follows it:
// the block of the paper's networks (a grouped or depthwise convolution followed by a
// pointwise standard convolution, Section II and IV-A of arXiv 2006.09791) in one
// kernel, so that the depthwise result never makes the round trip through HBM.
//
// The pointwise layer is the per-image GEMM  Y[k][pixel] = sum_c W2[k][c] * D[c][pixel]
// on v_mfma_f32_16x16x4_f32 (operand layout as in mfma_kernels.hip).  Its B operand, a
// chunk of CK channels x the block's pixels, is not loaded but computed: every staging
// task takes the 3 x (4*SD + 2) input neighbourhood of 4 consecutive depthwise outputs
// of one channel from global memory, applies the channel's nine weights (all depthwise
// weights sit in LDS) and the optional ReLU, and writes the 4 results into the LDS tile
// (and, when the depthwise result is still needed afterwards, to HBM from the blocks of
// the first filter tile).  The loads of chunk i+1 are in flight while chunk i is
// multiplied.  Filters on the M edge, pixels on the N edge; output straight to NCHW.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

struct DwPwParams {
    const float *x;     // depthwise input  [N][C][Hd][Wd]
    const float *wdw;   // depthwise weights: direct section [C][9][kpgd]
    const float *wpw;   // pointwise weights: mfma section [C/4][C2/16][64]
    float *d;           // depthwise output [N][C][H][W], or nullptr when it is not kept
    float *y;           // pointwise output [N][C2][H][W]
    const float *res;   // optional residual of the pointwise layer
    int N, C, Hd, Wd, H, W, C2;
    int kpgd, relu_dw, relu_pw;
};

struct TileP {
    int NB, TH;               // images, rows of the pointwise plane per tile
    int LW, IMG, PLANE;       // LDS row pitch, floats per image / per channel
    int CK, nchunks;
    int row_blocks, img_blocks, oc_blocks, tiles, gx;
    int tpr_log2, tasks, xslots, mtiles;
    int in_floats, w_floats, dw_floats;   // one input buffer; all pointwise filters of the block; depthwise weights
    unsigned m_TH, m_NB, m_ppi, m_W, m_rowb;
    unsigned x_bytes, d_bytes, y_bytes, wdw_bytes, wpw_bytes;
};

// staging slots per thread: four consecutive outputs of one (channel, image, row) each
template <int SD> struct SlotsP { static constexpr int value = SD == 1 ? 4 : 2; };

template <int MI, int NI, int SD>
__global__ __launch_bounds__(256, 2) void conv_dwpw(DwPwParams p, TileP t) {
    constexpr int NT = 256;   // four waves, each on its own 16*NI pixels
    constexpr int TMAX = SlotsP<SD>::value;
    constexpr int RAW = SD == 1 ? 6 : 9;   // input columns per row of a task: index i is column iw - 1 + i
    extern __shared__ f32x4 smem4[];
    float *smem = reinterpret_cast<float *>(smem4);
    const int buf_floats = t.in_floats + 4;          // an input buffer and a spare slot for idle lanes
    float *wsm = smem + 2 * buf_floats;              // pointwise filters [C/4][MI][64]
    float *wl = wsm + t.w_floats;                    // depthwise weights [C][12]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wp = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ob = blockIdx.y;
    const int ppi = t.TH * p.W, tot = t.NB * ppi;
    const unsigned HWd = p.Hd * p.Wd, HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rd = make_rsrc(p.d ? p.d : p.y, p.d ? t.d_bytes : 0u);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, p.res ? t.y_bytes : 0u);

    // ---- once per block: depthwise weights of every channel (nine floats at a pitch of
    // 12) and the block's MI filter tiles of the pointwise layer, all k-steps -> LDS ----
    {
        const __amdgpu_buffer_rsrc_t rwd = make_rsrc(p.wdw, t.wdw_bytes);
        for (int i = tid; i < p.C * 9; i += NT) {
            const int c = fast_div(i, 0x1c71c71du), k = i - c * 9;   // i / 9, exact for i < 2^16
            wl[c * 12 + k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rwd, (unsigned)i * (p.kpgd * 4), 0, 0));
        }
        const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wpw, t.wpw_bytes);
        const unsigned wrow = t.mtiles * 64 * 4;   // bytes per k-step of the packed section
        const int pieces = (p.C / 4) * MI * 16;    // 16-byte pieces
        for (int i = tid; i < pieces; i += NT) {
            const unsigned ks = i / (MI * 16), q = i % (MI * 16);
            smem4[(wsm - smem) / 4 + i] = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, ks * wrow + (ob * MI * 16 + q) * 16, 0, 0));
        }
    }

    // ---- staging plan: task = (channel of the chunk, image, row), 4 columns per thread.
    // What depends on the lane is computed once; a tile adds its origin. ----
    const int rpp = NT >> t.tpr_log2;
    const int row0 = tid >> t.tpr_log2, colv = tid & ((1 << t.tpr_log2) - 1);
    unsigned xlane[TMAX], dlane[TMAX], xlds[TMAX], wsel[TMAX], timg[TMAX], trow[TMAX];
    bool leftok[TMAX], rightok[TMAX];
#pragma unroll
    for (int k = 0; k < TMAX; ++k) {
        const int task = row0 + k * rpp;
        xlane[k] = dlane[k] = wsel[k] = trow[k] = 0;
        timg[k] = 0x7fffffffu;                 // never a valid image: the slot stays idle
        xlds[k] = t.in_floats * 4;             // spare slot
        leftok[k] = rightok[k] = false;
        if (k < t.xslots && task < t.tasks && colv * 4 < p.W) {
            const int cimg = fast_div(task, t.m_TH), r = task - cimg * t.TH;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            const int iw = colv * 4 * SD;
            xlds[k] = (c * t.PLANE + img * t.IMG + r * t.LW + colv * 4) * 4;
            wsel[k] = c * 12;
            timg[k] = img;
            trow[k] = r;
            // byte offset of (image img, channel c, input row r*SD - 1, column iw) relative to the
            // tile's first image and first input row; row -1 wraps and is never used
            xlane[k] = ((((unsigned)img * p.C + c) * p.Hd + r * SD - 1) * p.Wd + iw) * 4;
            dlane[k] = ((((unsigned)img * p.C + c) * p.H + r) * p.W + colv * 4) * 4;
            leftok[k] = iw > 0;
            rightok[k] = iw + 4 * SD < p.Wd;
        }
    }
    // Origin of a tile: first image, first output row.  Uniform.
    struct TileU {
        unsigned n0, oh0;
        bool live;
    };
    auto tile_of = [&](unsigned tg) {
        TileU u;
        const unsigned ib = fast_div(tg, t.m_rowb);
        u.n0 = ib * t.NB;
        u.oh0 = (tg - ib * t.row_blocks) * t.TH;
        u.live = tg < (unsigned)t.tiles;
        return u;
    };

    float raw[TMAX][3][RAW];
    auto fetch_x = [&](const TileU &u, int chunk) __attribute__((always_inline)) {
        const unsigned so = chunk * t.CK * HWd * 4;
        const unsigned xt = ((u.n0 * p.C) * p.Hd + u.oh0 * SD) * p.Wd * 4;
        // every slot loads, idle ones from out-of-range offsets (zeros): with a fixed number of
        // loads in flight the waits further down can count instead of draining the queue
#pragma unroll
        for (int k = 0; k < TMAX; ++k) {
            const bool live = u.live && u.n0 + timg[k] < (unsigned)p.N && u.oh0 + trow[k] < (unsigned)p.H;
            const int ih = (int)(u.oh0 + trow[k]) * SD - 1;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const unsigned o = (live && (unsigned)(ih + kh) < (unsigned)p.Hd) ? xt + xlane[k] + kh * p.Wd * 4 : kOob;
                const f32x4 m0 = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, o, so, 0));
                raw[k][kh][1] = m0.x; raw[k][kh][2] = m0.y; raw[k][kh][3] = m0.z; raw[k][kh][4] = m0.w;
                if (SD == 2) {
                    const f32x4 m1 = __builtin_bit_cast(
                        f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, o != kOob ? o + 16 : kOob, so, 0));
                    raw[k][kh][RAW - 4] = m1.x; raw[k][kh][RAW - 3] = m1.y; raw[k][kh][RAW - 2] = m1.z; raw[k][kh][RAW - 1] = m1.w;
                }
            }
        }
    };
    // Depthwise arithmetic on the fetched neighbourhoods, results -> LDS buffer (and HBM if
    // kept).  The column left of a task's first one and (stride 1) the column right of its
    // last one were loaded by the neighbouring lanes: the lanes of a row are consecutive and
    // a row never straddles a wavefront.  Idle lanes and rows outside the image hold zeros.
    auto commit = [&](const TileU &u, int chunk, int buf) __attribute__((always_inline)) {
        char *bb = reinterpret_cast<char *>(smem) + buf * (buf_floats * 4);
        const unsigned dt = ((u.n0 * p.C) * p.H + u.oh0) * p.W * 4 + chunk * t.CK * HW * 4;
#pragma unroll
        for (int k = 0; k < TMAX; ++k) {
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const float l = __shfl_up(raw[k][kh][4 * SD], 1);
                raw[k][kh][0] = leftok[k] ? l : 0.f;
                if (SD == 1) {
                    const float r = __shfl_down(raw[k][kh][1], 1);
                    raw[k][kh][RAW - 1] = rightok[k] ? r : 0.f;
                }
            }
            const float *wc = wl + chunk * t.CK * 12 + wsel[k];
            const f32x4 w0 = *reinterpret_cast<const f32x4 *>(wc), w1 = *reinterpret_cast<const f32x4 *>(wc + 4);
            const float w8 = wc[8];
            const float w[9] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w, w8};
            f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                    for (int x = 0; x < 4; ++x) o[x] = fmaf(raw[k][kh][x * SD + kw], w[kh * 3 + kw], o[x]);
            if (p.relu_dw) {
#pragma unroll
                for (int x = 0; x < 4; ++x) o[x] = fmaxf(o[x], 0.f);
            }
            *reinterpret_cast<f32x4 *>(bb + xlds[k]) = o;   // idle slots: the spare slot
            if (p.d && ob == 0) {
                const bool live = u.n0 + timg[k] < (unsigned)p.N && u.oh0 + trow[k] < (unsigned)p.H;
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rd, live ? dt + dlane[k] : kOob, 0, 0);
            }
        }
    };

    // ---- per-lane pixel coordinates ------------------------------------------------
    // Operand reads: lane l multiplies pixel l % 16 of each 16-pixel run.  The pixels are
    // the rows of the MFMA product (the tile is its A operand), so lane l ends up with
    // pixels 4*(l/16) .. +3 of filter l % 16 per run: four consecutive elements of an
    // output plane (W is a multiple of 4), one 16-byte store.
    int base[NI];
    unsigned olane[NI], oimg[NI], orem[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * 16 + (lane & 15);
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_W), col = rem - r * p.W;
        base[ni] = (lane >> 4) * t.PLANE + img * t.IMG + r * t.LW + col;
        const int q0 = (wp * NI + ni) * 16 + 4 * (lane >> 4);
        const int qq0 = q0 < tot ? q0 : 0;
        const int img0 = fast_div(qq0, t.m_ppi), rem0 = qq0 - img0 * ppi;
        oimg[ni] = q0 < tot ? img0 : 0x7fffffffu;
        orem[ni] = rem0;
        olane[ni] = (((unsigned)img0 * p.C2 + (lane & 15)) * HW + rem0) * 4;
    }

    // ---- software pipeline over (tile, channel chunk) steps: the loads of step i+1 are
    // in flight while step i multiplies.  A block walks over the tiles blockIdx.x,
    // blockIdx.x + gridDim.x, ... ----
    const int kchunk = t.CK / 4;
    const unsigned oc0 = ob * MI * 16;
    unsigned tg = blockIdx.x;
    int ch = 0, buf = 0;
    TileU cur = tile_of(tg), nxt = cur;
    fetch_x(cur, 0);
    __syncthreads();   // the weights are in LDS
    commit(cur, 0, 0);
    __syncthreads();
    f32x4 acc[MI][NI];
    for (;;) {
        int nch = ch + 1;
        unsigned ntg = tg;
        if (nch == t.nchunks) {
            nch = 0;
            ntg = tg + gridDim.x;
            nxt = tile_of(ntg);
        }
        const bool more = ntg < (unsigned)t.tiles;
        fetch_x(nxt, nch);   // nothing but zeros once the tiles are used up
        __builtin_amdgcn_sched_barrier(0);
        // ---- multiply: the first k-step of a tile starts from zero, so the accumulators
        // (still being read by the previous tile's stores) are only written by the matrix
        // unit, long after those stores were issued ----
        const float *xs = smem + buf * buf_floats;
        const float *ws = wsm + ch * kchunk * MI * 64 + lane;
        auto kstep = [&](int cb, bool fresh) __attribute__((always_inline)) {
            float a[MI], b[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) a[mi] = ws[(cb * MI + mi) * 64];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) b[ni] = xs[cb * 4 * t.PLANE + base[ni]];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                        b[ni], a[mi], fresh ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[mi][ni], 0, 0, 0);
        };
        if (ch == 0) kstep(0, true);
        else kstep(0, false);
        for (int cb = 1; cb < kchunk; ++cb) kstep(cb, false);

        if (ch == t.nchunks - 1) {
            // ---- epilogue: optional residual and ReLU, NCHW store --------------------
            const unsigned ot = ((cur.n0 * p.C2) * HW + cur.oh0 * p.W) * 4, lim = HW - cur.oh0 * p.W;
            unsigned off[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                off[ni] = (cur.n0 + oimg[ni] < (unsigned)p.N && orem[ni] < lim) ? ot + olane[ni] : kOob;
            if (p.res) {
                f32x4 rv[MI][NI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
                        rv[mi][ni] = __builtin_bit_cast(
                            f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, off[ni], (oc0 + mi * 16) * HW * 4, 0));
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) acc[mi][ni] += rv[mi][ni];
            }
            if (p.relu_pw) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[mi][ni][r] = fmaxf(acc[mi][ni][r], 0.f);
            }
            // the stores read the accumulators in place
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[mi][ni]), ry, off[ni],
                                                           (oc0 + mi * 16) * HW * 4, 0);
            // A 16-byte store takes its data a cycle or two after it issues, and one whose data
            // register was rewritten by the very next instruction has been seen to store the new
            // value: keep this wave's vector ALU off the accumulators for a few cycles.
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_sleep(1);
            __builtin_amdgcn_sched_barrier(0);
            if (!more) break;
            // (commit is written out on both paths: here the stores were issued after the loads it
            // waits for, and the wait can leave them in flight)
            commit(nxt, nch, buf ^ 1);
        } else {
            commit(nxt, nch, buf ^ 1);   // that buffer was last read by the multiplication of the step before
        }
        __syncthreads();
        tg = ntg;
        ch = nch;
        buf ^= 1;
        cur = nxt;
    }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

struct CfgP {
    int MI, NI;
};
const CfgP kCfgP[] = {{4, 4}, {4, 2}, {2, 4}, {2, 2}};
constexpr int kNumCfgP = sizeof(kCfgP) / sizeof(kCfgP[0]);
constexpr int kLdsBudgetP = 64 * 1024;   // two blocks per compute unit are resident anyway

bool planP_cfg(const DwPwParams &p, int sd, const CfgP &c, TileP *out) {
    const int MB = 16 * c.MI, PB = 16 * c.NI * 4, NT = 256;
    if (p.C2 % MB || NT % (c.MI * 16)) return false;
    TileP t{};
    ConvParams q{};   // the pointwise plane, for the pixel split
    q.N = p.N; q.Hout = p.H; q.Wout = p.W;
    if (!split_pixels(q, PB, &t.NB, &t.TH)) return false;
    t.LW = round_up(p.W, 4);
    t.IMG = t.TH * t.LW;
    // the four lane groups of a B-operand read are one channel apart: a pitch of 16 mod 32
    // floats puts them on disjoint banks
    t.PLANE = round_up(t.NB * t.IMG, 32) + 16;
    const int cols = p.W / 4;
    t.tpr_log2 = 0;
    while ((1 << t.tpr_log2) < cols) ++t.tpr_log2;
    if (t.tpr_log2 > 6) return false;   // a row's lanes exchange edge columns inside one wavefront
    const int rpp = NT >> t.tpr_log2;
    t.mtiles = p.C2 / 16;
    t.row_blocks = (p.H + t.TH - 1) / t.TH;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.oc_blocks = p.C2 / MB;
    t.dw_floats = p.C * 12;
    t.w_floats = (p.C / 4) * c.MI * 64;
    const int tmax = sd == 1 ? SlotsP<1>::value : SlotsP<2>::value;
    int best = 0;
    for (int d = 1; d <= p.C / 4; ++d) {
        if ((p.C / 4) % d) continue;
        const int CK = 4 * d;
        const size_t in_f = (size_t)CK * t.PLANE;
        if ((2 * (in_f + 4) + t.w_floats + t.dw_floats) * sizeof(float) > (size_t)kLdsBudgetP) continue;
        if ((CK * t.NB * t.TH + rpp - 1) / rpp > tmax) continue;
        best = d;
    }
    if (!best) return false;
    t.CK = 4 * best;
    t.nchunks = p.C / t.CK;
    t.tasks = t.CK * t.NB * t.TH;
    t.xslots = (t.tasks + rpp - 1) / rpp;
    t.in_floats = t.CK * t.PLANE;
    t.m_TH = div_magic(t.TH);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.W);
    t.m_W = div_magic(p.W);
    t.m_rowb = div_magic(t.row_blocks);
    const double xb = (double)p.N * p.C * p.Hd * p.Wd * 4, db = (double)p.N * p.C * p.H * p.W * 4;
    const double yb = (double)p.N * p.C2 * p.H * p.W * 4;
    const double wdb = (double)p.C * 9 * p.kpgd * 4, wpb = (double)(p.C / 4) * t.mtiles * 256;
    if (xb >= (double)kOob || db >= (double)kOob || yb >= (double)kOob || wdb >= (double)kOob || wpb >= (double)kOob)
        return false;
    t.x_bytes = (unsigned)xb;
    t.d_bytes = (unsigned)db;
    t.y_bytes = (unsigned)yb;
    t.wdw_bytes = (unsigned)wdb;
    t.wpw_bytes = (unsigned)wpb;
    if ((long)t.row_blocks * t.img_blocks > 2147483647L - 65536 || t.oc_blocks > 65535) return false;
    if ((double)t.row_blocks * t.img_blocks * t.row_blocks >= 4.0e9 || t.tasks >= 65536 || t.TH * p.W >= 65536 ||
        p.C * 9 >= 65536)
        return false;
    t.tiles = t.row_blocks * t.img_blocks;
    {
        // one resident set of blocks (two per compute unit) walks over the tiles in equal shares
        long cap = 2L * kNumCU / t.oc_blocks;
        cap = cap < 1 ? 1 : cap;
        const long rounds = (t.tiles + cap - 1) / cap;
        t.gx = (int)((t.tiles + rounds - 1) / rounds);
    }
    *out = t;
    return true;
}

template <int MI, int NI>
hipError_t launchP_inst(const DwPwParams &p, const TileP &t, int sd, hipStream_t s) {
    const size_t lds = (2 * ((size_t)t.in_floats + 4) + t.w_floats + t.dw_floats) * sizeof(float);
    const dim3 grid(t.gx, t.oc_blocks);
    if (sd == 1) hipLaunchKernelGGL((conv_dwpw<MI, NI, 1>), grid, dim3(256), lds, s, p, t);
    else hipLaunchKernelGGL((conv_dwpw<MI, NI, 2>), grid, dim3(256), lds, s, p, t);
    return hipGetLastError();
}

}  // namespace

static_assert(sizeof(DwPwParams) <= sizeof(((DwPwPlan *)0)->params), "plan storage too small");
static_assert(sizeof(TileP) <= sizeof(((DwPwPlan *)0)->tile), "plan storage too small");

// layers[first], layers[first + 1]: depthwise 3x3 (pad 1, stride 1 | 2, fp32) whose result
// feeds a 1x1 ungrouped fp32 convolution with Cout a multiple of 16.  Returns 2 when the
// pair runs as one kernel.  The depthwise result is written to its buffer only if the
// rest of the chain can still see it.
int plan_dwpw(const gspc_layer_t *layers, int first, int count, void *const *bufs, DwPwPlan *out) {
    static const bool off = std::getenv("GSPC_NO_DWPW") != nullptr;   // tuning aids
    static const int force_ocb = std::getenv("GSPC_DWPW_OCB") ? std::atoi(std::getenv("GSPC_DWPW_OCB")) : 0;
    static const int max_c = std::getenv("GSPC_DWPW_C") ? std::atoi(std::getenv("GSPC_DWPW_C")) : 128;
    if (off || count < 2) return 0;
    const gspc_layer_t &A = layers[first], &B = layers[first + 1];
    if (A.op != GSPC_OP_CONV || B.op != GSPC_OP_CONV || !A.w || !B.w) return 0;
    if (A.w->dtype != GSPC_F32 || B.w->dtype != GSPC_F32) return 0;
    if (A.KH != 3 || A.KW != 3 || A.pad != 1 || (A.stride != 1 && A.stride != 2) || A.groups != A.Cin ||
        A.Cout != A.Cin || A.src2 >= 0)
        return 0;
    const int H = (A.H + 2 - 3) / A.stride + 1, W = (A.W + 2 - 3) / A.stride + 1;
    if (B.KH != 1 || B.KW != 1 || B.pad != 0 || B.stride != 1 || B.groups != 1 || B.src != A.dst || B.N != A.N ||
        B.Cin != A.Cout || B.H != H || B.W != W)
        return 0;
    if (B.dst == A.dst || B.dst == A.src || B.src2 == A.dst) return 0;
    if (A.Cin % 4 || A.Cin > max_c || B.Cout % 16 || W % 4 || A.W % 4) return 0;
    if (A.stride == 2 && A.W != 2 * W) return 0;
    if (B.w->geom.variant != kMfma16 || !B.w->geom.mfma_bytes) return 0;
    auto misaligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) != 0; };
    if (misaligned(bufs[A.src]) || misaligned(bufs[A.dst]) || misaligned(bufs[B.dst])) return 0;

    DwPwParams p{};
    p.x = static_cast<const float *>(bufs[A.src]);
    p.wdw = static_cast<const float *>(A.w->dev);
    p.wpw = reinterpret_cast<const float *>(static_cast<const char *>(B.w->dev) + B.w->geom.mfma_offset);
    p.y = static_cast<float *>(bufs[B.dst]);
    p.res = B.src2 >= 0 ? static_cast<const float *>(bufs[B.src2]) : nullptr;
    p.N = A.N; p.C = A.Cin; p.Hd = A.H; p.Wd = A.W; p.H = H; p.W = W; p.C2 = B.Cout;
    p.kpgd = A.w->geom.KPGd;
    p.relu_dw = (A.flags & GSPC_FLAG_RELU) ? 1 : 0;
    p.relu_pw = (B.flags & GSPC_FLAG_RELU) ? 1 : 0;
    // Is the depthwise result visible after the pair?  Not if a later step overwrites its
    // buffer before anything reads it.
    bool keep = true;
    for (int m = first + 2; m < first + count; ++m) {
        const gspc_layer_t &L = layers[m];
        if (L.src == A.dst || L.src2 == A.dst) break;
        if (L.dst == A.dst) {
            keep = false;
            break;
        }
    }
    p.d = keep ? static_cast<float *>(bufs[A.dst]) : nullptr;

    // Every filter tile of the pointwise layer recomputes the depthwise tile: fuse only while
    // that is at most two of them (four at stride 2, where a depthwise output costs the same
    // but the unfused pair moves four times the input per output).  Measured break-even; from 256
    // filters on, the dense pointwise layer has its 128-filter blocks and the pair as two kernels is
    // ahead at stride 2 as well (128 channels -> 256 filters at N = 256: 260 against 276 us).
    const int max_ocb = force_ocb ? force_ocb : (A.stride == 2 && B.Cout < 256 ? 4 : 2);
    // The largest tile that still gives every compute unit two blocks, else the shape with the
    // most blocks; with less than one block per compute unit the pair is faster as two
    // kernels, whose finer tiles spread over more of the chip (small batches).
    int best = -1;
    long best_blocks = 0;
    TileP bt{};
    for (int i = 0; i < kNumCfgP; ++i) {
        TileP t;
        if (!planP_cfg(p, A.stride, kCfgP[i], &t) || t.oc_blocks > max_ocb) continue;
        const long blocks = (long)t.tiles * t.oc_blocks;
        if (blocks > best_blocks) {
            best = i;
            best_blocks = blocks;
            bt = t;
        }
        if (blocks >= 2 * kNumCU) break;
    }
    if (best < 0 || best_blocks < kNumCU) return 0;
    out->inst = best;
    out->sd = A.stride;
    std::memcpy(out->params, &p, sizeof(p));
    std::memcpy(out->tile, &bt, sizeof(bt));
    return 2;
}

hipError_t launch_dwpw(const DwPwPlan &plan, hipStream_t s, const char **name) {
    DwPwParams p;
    TileP t;
    std::memcpy(&p, plan.params, sizeof(p));
    std::memcpy(&t, plan.tile, sizeof(t));
    const CfgP &c = kCfgP[plan.inst];
    *name = intern_name("conv_dwpw<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," +
                        std::to_string(plan.sd) + ">");
    switch (plan.inst) {
    case 0: return launchP_inst<4, 4>(p, t, plan.sd, s);
    case 1: return launchP_inst<4, 2>(p, t, plan.sd, s);
    case 2: return launchP_inst<2, 4>(p, t, plan.sd, s);
    case 3: return launchP_inst<2, 2>(p, t, plan.sd, s);
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
