// Per-group implicit-GEMM grouped convolution on the gfx950 matrix cores.
//
// For one group the convolution stage of Algorithm 1 (arXiv 2006.09791) is the
// contraction  Y[oc][pixel] = sum_k W[oc][k] * X[k][pixel],  k = (c, kh, kw),
// pixel = (n, oh, ow).  Filters sit on the M edge of the MFMA tile, output
// pixels on the N edge, and the im2col matrix X[k][pixel] is never built: a
// zero-haloed input tile is staged in LDS (the paper's input reshape, fused)
// and every lane reads its own (pixel, k) element from it.  Results go
// straight to NCHW (the paper's output reshape, fused away).
#include <cstdlib>
#include <cstring>
#include <unordered_map>

#include "conv_common.h"

namespace gspc {

// ---------------------------------------------------------------------------
// 16x16x4 kernel: filters in tiles of 16 (the last tile zero-padded when KPG is not a multiple).
//
// v_mfma_f32_16x16x4_f32 operand layout (lane l of 64):
//   A: filter row l%16, reduction slot l/16      B: slot l/16, pixel column l%16
//   D: register r holds (row 4*(l/16) + r, column l%16)
// One k-step contracts 4 input channels at one kernel tap (kh, kw).
//
// Block = WM x WP waves; a wave owns MI x NI tiles = 16*MI filters x 16*NI
// pixels.  The block's pixels are NB images x TH output rows x Wout columns,
// flattened in that order and cut into runs of 16.  The reduction runs over
// chunks of CK channels; chunk i+1 is fetched from global memory into
// registers while chunk i is multiplied out of LDS (two LDS buffers).
// ---------------------------------------------------------------------------
constexpr int kTmax16 = 4, kTmax16Stem = 10, kWmax16 = 4;

struct Tile16 {
    int NB, TH, IHt;         // images, output rows per block; staged input rows
    int LW, IMG, PLANE, XO;  // LDS row pitch, floats per image / per channel, column of input col 0
    int CK, nchunks;         // channels per chunk (multiple of 4), number of chunks
    int row_blocks, img_blocks, oc_blocks;
    int tpr_log2, vec;       // threads per staged row (log2); 1 = 4-wide loads
    int tasks;               // staged rows per chunk = CK*NB*IHt
    int xslots, wslots;      // staged rows / weight float4 per thread per chunk
    int ksteps, mtiles;      // geometry of the packed weight section
    int in_floats, w_floats; // per LDS buffer (a buffer is in | w | 4 spare floats)
    int ksplit;              // 1: the four waves share one pixel tile and split the reduction
    int vec_out;             // groups of four tile pixels are 16 contiguous, aligned bytes of a plane
    int one_buf;             // single chunk with padded channels: one LDS buffer instead of two
    int flat4;               // 1x1 on a plane of HW % 4 != 0 elements, one image per block: four channels staged as one row
    unsigned m_IHt, m_NB, m_ppi, m_Wout, m_rowb, m_ocb;  // multiply-high reciprocals (0 = divisor 1)
    unsigned x_bytes, w_bytes, y_bytes;                  // extents for the buffer descriptors
};

#ifdef GSPC_PHASE_TIMING
__device__ unsigned long long g_phase[8 * 4096];
#define GSPC_STAMP(i)                                                                      \
    if (threadIdx.x == 0) {                                                                \
        const unsigned bid = blockIdx.x + blockIdx.y * gridDim.x;                          \
        if (bid < 4096) g_phase[bid * 8 + (i)] = __builtin_amdgcn_s_memrealtime();         \
    }
#else
#define GSPC_STAMP(i)
#endif

template <int MI, int NI, int WM, int WP, int KH, int KW, int S, typename TIN, bool VO>
__global__ __launch_bounds__(64 * WM * WP) void conv_mfma16(ConvParams p, Tile16 t) {
    GSPC_STAMP(0)
    constexpr int NT = 64 * WM * WP, TAPS = KH * KW, MIWM = MI * WM;
    // (the 7x7 stem stages nine 224-pixel rows per 4-channel block: more rows per thread)
    constexpr int TMAX = KH == 7 ? kTmax16Stem : kTmax16, WMAX = kWmax16, ES = (int)sizeof(TIN);
    extern __shared__ f32x4 smem4[];
    float *smem = reinterpret_cast<float *>(smem4);
    const int buf_floats = t.in_floats + t.w_floats + 4;
    const unsigned spare = (t.in_floats + t.w_floats) * 4;   // byte offset of a buffer's spare slot

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Normally the WP pixel-side waves own different pixel runs.  With ksplit they
    // all own the same runs and take every fourth 4-channel block of the
    // reduction instead (small batches: more, shorter blocks), and their partial
    // sums are added through LDS at the end.
    const int wm = wave / WP, wp = t.ksplit ? 0 : wave % WP;
    const int wk = t.ksplit ? wave : 0, kstride = t.ksplit ? WM * WP : 1;
    const unsigned ib = fast_div(blockIdx.x, t.m_rowb);
    const int rb = blockIdx.x - ib * t.row_blocks;
    const unsigned j = fast_div(blockIdx.y, t.m_ocb);
    const int ob = blockIdx.y - j * t.oc_blocks;
    const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;
    const unsigned HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wm, t.w_bytes);

    // ---- weights of a chunk: MIWM*kchunk*64 floats, NT float4 per slot --------
    const int kchunk = t.CK / 4 * TAPS;
    const unsigned wrow = t.mtiles * 64 * 4;   // bytes per k-step of the packed section
    const unsigned wblk = ((j * t.ksteps * t.mtiles + ob * MIWM) * 64) * 4;
    const unsigned wvoff = (tid / (MIWM * 16)) * wrow + (tid % (MIWM * 16)) * 16;
    constexpr unsigned kWslot = (NT / (MIWM * 16));   // k-steps advanced per slot
    static_assert(NT % (MIWM * 16) == 0, "a slot must cover whole k-steps");
    // Two register sets: a chunk is fetched two iterations before it is needed.
    f32x4 pin0[TMAX], pw0[WMAX], pin1[TMAX], pw1[WMAX];
    auto fetch_w = [&](int chunk, f32x4 (&pw)[WMAX]) __attribute__((always_inline)) {
        const unsigned so = wblk + chunk * kchunk * wrow;
#pragma unroll
        for (int k = 0; k < WMAX; ++k)
            if (k < t.wslots)
                pw[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff, so + k * kWslot * wrow, 0));
    };
    fetch_w(0, pw0);

    // ---- per-thread input staging plan (identical for every chunk) ---------
    const int rpp = NT >> t.tpr_log2;
    const int row0 = tid >> t.tpr_log2, colv = tid & ((1 << t.tpr_log2) - 1);
    const int vw = t.vec ? 4 : 1;
    unsigned xoff[TMAX], xlds[TMAX];
#pragma unroll
    for (int k = 0; k < TMAX; ++k) {
        const int task = row0 + k * rpp;
        xoff[k] = kOob;
        xlds[k] = spare;
        if (t.flat4) {
            // The four planes of a 4-channel block are 4*HW contiguous floats (16-byte aligned, since the
            // channel count per group is a multiple of 4) both in global memory and in the tile (PLANE = HW):
            // one staged row per block of channels, 16 bytes per thread, whatever HW is.
            if (k < t.xslots && task < t.tasks && colv < p.W) {
                xlds[k] = (task * 4 * t.PLANE + colv * 4) * 4;
                if (n0 < p.N) xoff[k] = ((((unsigned)n0 * p.Cin + j * p.CPG + 4 * task) * HW) + colv * 4) * ES;
            }
        } else if (k < t.xslots && task < t.tasks && colv * vw < p.W) {
            const int cimg = fast_div(task, t.m_IHt), r = task - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            const int ih = ih0 + r, n = n0 + img;
            xlds[k] = (c * t.PLANE + img * t.IMG + r * t.LW + t.XO + colv * vw) * 4;
            if (n < p.N && ih >= 0 && ih < p.H && c < p.CPG)
                xoff[k] = (((n * p.Cin + j * p.CPG + c) * p.H + ih) * p.W + colv * vw) * ES;
        }
    }
    auto fetch_x = [&](int chunk, f32x4 (&pin)[TMAX]) __attribute__((always_inline)) {
        const unsigned so = chunk * t.CK * HW * ES;
#pragma unroll
        for (int k = 0; k < TMAX; ++k)
            if (k < t.xslots) pin[k] = buf_load_in<TIN>(rx, xoff[k], so, t.vec);
    };
    auto commit = [&](int buf, const f32x4 (&pin)[TMAX], const f32x4 (&pw)[WMAX]) __attribute__((always_inline)) {
        char *bb = reinterpret_cast<char *>(smem) + buf * (buf_floats * 4);
#pragma unroll
        for (int k = 0; k < TMAX; ++k) {
            if (k < t.xslots) {
                if (t.vec) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pin[k];
                else *reinterpret_cast<float *>(bb + xlds[k]) = pin[k].x;
            }
        }
        char *wb = bb + t.in_floats * 4 + tid * 16;
#pragma unroll
        for (int k = 0; k < WMAX; ++k)
            if (k < t.wslots) *reinterpret_cast<f32x4 *>(wb + k * NT * 16) = pw[k];
    };
    GSPC_STAMP(1)
    fetch_x(0, pin0);
    if (t.nchunks > 1) {
        fetch_w(1, pw1);
        fetch_x(1, pin1);
    }
    GSPC_STAMP(2)

    // ---- per-lane pixel coordinates ----------------------------------------
    int base[NI];
    unsigned ooff[NI];   // byte offset of this lane's first output element, or kOob
    const unsigned HWo = p.Hout * p.Wout;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * 16 + (lane & 15);
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_Wout), col = rem - r * p.Wout;
        base[ni] = (lane >> 4) * t.PLANE + img * t.IMG + r * S * t.LW + (t.XO - p.pad) + col * S;
        if (VO) {
            // pixels are the rows of the MFMA product: this lane ends up with pixels 4*(l/16) .. +3
            // of the run, four consecutive elements of one output plane, for filter l % 16
            const int q0 = (wp * NI + ni) * 16 + 4 * (lane >> 4);
            const int qq0 = q0 < tot ? q0 : 0;
            const int img0 = fast_div(qq0, t.m_ppi), rem0 = qq0 - img0 * ppi;
            const unsigned n = n0 + img0, e = oh0 * p.Wout + rem0;
            ooff[ni] = (q0 < tot && n < (unsigned)p.N && e < HWo)
                           ? ((n * p.Cout + j * p.KPG + (lane & 15)) * HWo + e) * 4
                           : kOob;
        } else {
            const int n = n0 + img, oh = oh0 + r;
            ooff[ni] = (q < tot && n < p.N && oh < p.Hout)
                           ? (((unsigned)n * p.Cout + j * p.KPG + 4 * (lane >> 4)) * HWo + oh * p.Wout + col) * 4
                           : kOob;
        }
    }

    f32x4 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The staging never writes the halo columns left and right of a row: clear
    // them once, in both buffers (rows = channels x images x staged rows).
    {
        const int per = t.CK * t.NB * t.IHt, rows = (t.one_buf ? 1 : 2) * per;
        const int right = t.XO + p.W;
        for (int i = tid; i < rows; i += NT) {
            const int b = i >= per, rr = i - b * per;
            const int cimg = fast_div(rr, t.m_IHt), r = rr - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            float *row = smem + b * buf_floats + c * t.PLANE + img * t.IMG + r * t.LW;
            for (int x = 0; x < t.XO; ++x) row[x] = 0.f;
            for (int x = right; x < t.LW; ++x) row[x] = 0.f;
        }
    }
    GSPC_STAMP(3)
    commit(0, pin0, pw0);
    __syncthreads();
    GSPC_STAMP(4)

    // Software pipeline: iteration ch multiplies chunk ch out of LDS buffer
    // ch&1; chunk ch+1 moves registers -> the other LDS buffer at its end, and
    // chunk ch+2 is requested from global memory at its start.
    auto compute = [&](int ch) __attribute__((always_inline)) {
        const float *xs = smem + (ch & 1) * buf_floats;
        const float *ws = xs + t.in_floats + (wm * MI) * 64 + lane;
        for (int cb = wk; cb < t.CK / 4; cb += kstride) {
            const float *xrow = xs + cb * 4 * t.PLANE;
            const float *wrw = ws + cb * TAPS * MIWM * 64;
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
#pragma unroll
                for (int kw = 0; kw < KW; ++kw) {
                    float a[MI], b[NI];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) a[mi] = wrw[((kh * KW + kw) * MIWM + mi) * 64];
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) b[ni] = xrow[base[ni] + kh * t.LW + kw];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
                            acc[mi][ni] = VO ? __builtin_amdgcn_mfma_f32_16x16x4f32(b[ni], a[mi], acc[mi][ni], 0, 0, 0)
                                             : __builtin_amdgcn_mfma_f32_16x16x4f32(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
                }
            }
        }
    };
    for (int ch = 0; ch < t.nchunks; ch += 2) {
        // even chunk: set 0 is free (chunk ch is in LDS), set 1 holds chunk ch+1
        if (ch + 2 < t.nchunks) {
            fetch_w(ch + 2, pw0);
            fetch_x(ch + 2, pin0);
        }
        compute(ch);
        if (ch + 1 < t.nchunks) {
            commit((ch + 1) & 1, pin1, pw1);
            __syncthreads();
            // odd chunk: set 1 is free, set 0 holds chunk ch+2
            if (ch + 3 < t.nchunks) {
                fetch_w(ch + 3, pw1);
                fetch_x(ch + 3, pin1);
            }
            compute(ch + 1);
            if (ch + 2 < t.nchunks) {
                commit(ch & 1, pin0, pw0);
                __syncthreads();
            }
        }
    }

    GSPC_STAMP(5)
    if (t.ksplit) {
        __syncthreads();   // staging buffers are free: reuse them for the partial sums
        if (wave != 0) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) smem4[((wave * MI + mi) * NI + ni) * 64 + lane] = acc[mi][ni];
        }
        __syncthreads();
        if (wave != 0) return;
        for (int w = 1; w < WM * WP; ++w)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] += smem4[((w * MI + mi) * NI + ni) * 64 + lane];
    }
    // ---- epilogue: optional residual and ReLU, NCHW store -------------------
    // Register r of tile (mi, ni) is filter 16*(tile row) + 4*(lane/16) + r at
    // this lane's pixel; the 4*(lane/16) part already sits in ooff.
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const unsigned oc0 = (ob * MIWM + wm * MI) * 16;
    // KPG need not be a multiple of 16: the last filter tile is zero-padded in the packed
    // section, and the lanes (registers) of its padding filters get an out-of-range offset.
    if (VO) {
        unsigned om[MI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) om[mi] = oc0 + mi * 16 + (lane & 15) < (unsigned)p.KPG ? 0u : kOob;
        // one 16-byte store per tile: a quarter of the store instructions, and the vector memory
        // path charges per instruction
        if (p.res) {
            const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
            f32x4 rv[MI][NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    rv[mi][ni] = __builtin_bit_cast(
                        f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, ooff[ni] | om[mi], (oc0 + mi * 16) * HWo * 4, 0));
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] += rv[mi][ni];
        }
        if (p.relu) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[mi][ni][r] = fmaxf(acc[mi][ni][r], 0.f);
        }
        // the stores read the accumulators in place; nothing writes a register after them
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[mi][ni]), ry, ooff[ni] | om[mi],
                                                       (oc0 + mi * 16) * HWo * 4, 0);
        GSPC_STAMP(6)
        return;
    }
    const unsigned ocl = oc0 + 4 * (lane >> 4);   // this lane's filter for mi = 0, r = 0
    if (p.res) {
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[mi][ni][r] += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                        rr, ocl + mi * 16 + r < (unsigned)p.KPG ? ooff[ni] : kOob, (oc0 + mi * 16 + r) * HWo * 4, 0));
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[mi][ni][r];
                if (p.relu) v = fmaxf(v, 0.f);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), ry,
                                                      ocl + mi * 16 + r < (unsigned)p.KPG ? ooff[ni] : kOob,
                                                      (oc0 + mi * 16 + r) * HWo * 4, 0);
            }
    GSPC_STAMP(6)
}

#ifdef GSPC_PHASE_TIMING
extern "C" int gspc_debug_phases(unsigned long long *out, int n) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase), sizeof(unsigned long long) * n);
}
#endif

// ---------------------------------------------------------------------------
// Host side: tile planning and instance selection.
// ---------------------------------------------------------------------------
namespace {

constexpr int kLdsBudget16 = 40 * 1024;   // four blocks per CU out of 160 KB
constexpr size_t kLdsMax = 160 * 1024;

struct Cfg16 {
    int MI, NI, WM, WP, ksplit;
};

// Instantiated block shapes, largest first; the ksplit entries reuse the WM = 1,
// WP = 4 instances with all four waves on one 16*MI x 16*NI tile.
const Cfg16 kCfg16[] = {
    {4, 4, 1, 4, 0}, {2, 4, 1, 4, 0}, {4, 2, 1, 4, 0}, {2, 2, 1, 4, 0}, {1, 4, 1, 4, 0}, {2, 2, 2, 2, 0},
    {1, 2, 1, 4, 0}, {2, 1, 1, 4, 0}, {1, 1, 1, 4, 0},
    {2, 2, 1, 4, 1}, {1, 2, 1, 4, 1}, {2, 1, 1, 4, 1}, {1, 1, 1, 4, 1},
    {4, 2, 2, 4, 0},   // eight waves, 128 filters x 128 pixels per block: dense pointwise layers (see plan16)
};
constexpr int kNumCfg16 = sizeof(kCfg16) / sizeof(kCfg16[0]);
constexpr int kFirstKsplit = 9, kEndKsplit = 13;

bool shape_instantiated(int KH, int KW, int S) {
    return (KH == 3 && KW == 3 && (S == 1 || S == 2)) || (KH == 1 && KW == 1 && (S == 1 || S == 2)) ||
           (KH == 7 && KW == 7 && S == 2);
}

// LDS bank conflicts (32 banks of 4 bytes) of the first B-operand read of wave
// 0 for a candidate channel pitch; returns the worst multiplicity of a bank.
int bank_cost(const ConvParams &p, const Tile16 &t, int plane) {
    int worst = 0;
    for (int half = 0; half < 2; ++half) {
        int cnt[32] = {0};
        for (int l = 32 * half; l < 32 * half + 32; ++l) {
            int q = l & 15;
            const int ppi = t.TH * p.Wout;
            if (q >= t.NB * ppi) q = 0;
            const int img = q / ppi, rem = q % ppi, r = rem / p.Wout, col = rem % p.Wout;
            const int a = (l >> 4) * plane + img * t.IMG + r * p.stride * t.LW + col * p.stride;
            ++cnt[a & 31];
        }
        for (int b = 0; b < 32; ++b) worst = cnt[b] > worst ? cnt[b] : worst;
    }
    return worst;
}

bool plan16_cfg(const ConvParams &p, const PackGeom &g, const Cfg16 &c, Tile16 *out, int lds_budget = kLdsBudget16) {
    const int MB = 16 * c.MI * c.WM, PB = 16 * c.NI * (c.ksplit ? 1 : c.WP), NT = 64 * c.WM * c.WP;
    if ((g.mtiles * 16) % MB) return false;   // whole filter tiles only; the last tile may be partly padding
    Tile16 t{};
    t.ksplit = c.ksplit;
    if (!split_pixels(p, PB, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * p.stride + p.KH;
    // 1x1 layers on planes handed over as one row of HW % 4 != 0 elements (7x7, 5x5 ...): one image per
    // block, channel pitch HW exactly, so that four channels can be staged as one aligned row
    t.flat4 = p.KH == 1 && p.KW == 1 && p.stride == 1 && p.pad == 0 && p.H == 1 && p.W % 4 != 0 && !p.in_bf16 &&
              g.CPGp == g.CPG && p.W <= NT && PB < 2 * p.W;
    if (t.flat4) t.NB = 1;
    t.vec = p.W % 4 == 0;
    if (t.vec) {
        t.XO = 4 * ((p.pad + 3) / 4);
        t.LW = round_up(t.XO + p.W + p.pad, 4);
    } else {
        t.XO = p.pad;
        t.LW = p.W + 2 * p.pad;
    }
    t.IMG = t.IHt * t.LW;
    const int plane0 = round_up(t.NB * t.IMG, 4);
    int best_pad = 0, best_cost = 1 << 30;
    for (int pad = 0; pad < 32; pad += 4) {
        const int cost = bank_cost(p, t, plane0 + pad);
        if (cost < best_cost) {
            best_cost = cost;
            best_pad = pad;
        }
    }
    t.PLANE = t.flat4 ? p.W : plane0 + best_pad;
    if (t.flat4) t.vec = 1;   // 16-byte loads and LDS writes
    const int cols = t.vec && !t.flat4 ? p.W / 4 : p.W;
    t.tpr_log2 = 0;
    while ((1 << t.tpr_log2) < cols) ++t.tpr_log2;
    if ((1 << t.tpr_log2) > NT) return false;
    const int rpp = NT >> t.tpr_log2;
    t.ksteps = g.ksteps;
    t.mtiles = g.mtiles;
    t.row_blocks = (p.Hout + t.TH - 1) / t.TH;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.oc_blocks = g.mtiles * 16 / MB;
    const bool check_c = g.CPGp != g.CPG;   // padded channels are masked in the plan: one chunk only
    const int cblks = g.CPGp / 4, taps = p.KH * p.KW;
    int best = 0;
    for (int d = check_c ? cblks : 1; d <= cblks; ++d) {
        if (cblks % d) continue;
        const int CK = 4 * d;
        const int wsl = (c.MI * c.WM * d * taps * 16 + NT - 1) / NT;
        const size_t in_f = (size_t)CK * t.PLANE, w_f = (size_t)wsl * NT * 4;
        // (layers with padded channels run as a single chunk and never touch the second buffer: larger
        // tiles fit, e.g. 18 channels per group on 56-pixel rows)
        if ((check_c ? 1 : 2) * (in_f + w_f + 4) * sizeof(float) > (size_t)(c.ksplit ? 2 * lds_budget : lds_budget)) continue;
        if (((t.flat4 ? d : CK * t.NB * t.IHt) + rpp - 1) / rpp > (p.KH == 7 ? kTmax16Stem : kTmax16)) continue;
        if (wsl > kWmax16) continue;
        best = d;
    }
    if (!best) return false;
    t.CK = 4 * best;
    t.nchunks = cblks / best;
    t.one_buf = check_c ? 1 : 0;
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.Wout);
    t.m_Wout = div_magic(p.Wout);
    t.m_rowb = div_magic(t.row_blocks);
    t.m_ocb = div_magic(t.oc_blocks);
    t.vec_out = (t.TH * p.Wout) % 4 == 0 && (p.Hout * p.Wout) % 4 == 0;
    t.tasks = t.flat4 ? t.CK / 4 : t.CK * t.NB * t.IHt;
    t.xslots = (t.tasks + rpp - 1) / rpp;
    t.wslots = (c.MI * c.WM * best * taps * 16 + NT - 1) / NT;
    t.in_floats = t.CK * t.PLANE;
    t.w_floats = t.wslots * NT * 4;
    const double xb = (double)p.N * p.Cin * p.H * p.W * (p.in_bf16 ? 2 : 4);
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    const double wb = (double)p.groups * g.ksteps * g.mtiles * 256;
    if (xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    if ((long)t.row_blocks * t.img_blocks > 2147483647L || p.groups * t.oc_blocks > 65535) return false;
    if ((double)t.row_blocks * t.img_blocks * t.row_blocks >= 4.0e9 ||
        (double)p.groups * t.oc_blocks * t.oc_blocks >= 4.0e9 || t.tasks >= 65536 || t.TH * p.Wout >= 65536)
        return false;
    *out = t;
    return true;
}

// Picks the block shape: the largest one that still gives every CU two blocks,
// else the one with the most blocks.
bool plan16(const ConvParams &p, const PackGeom &g, int *cfg_idx, Tile16 *t_out) {
    if (!g.mfma_bytes || !p.wm || !shape_instantiated(p.KH, p.KW, p.stride)) return false;
    static const char *force = std::getenv("GSPC_TILE16");
    const int forced = force ? std::atoi(force) : tuned_config(p, 'm');
    if (forced >= 0) {
        const int i = forced;
        // (eight-wave blocks: two per compute unit, hence 64 KB each)
        if (i >= 0 && i < kNumCfg16 &&
            plan16_cfg(p, g, kCfg16[i], t_out, i >= 13 ? 64 * 1024 : kLdsBudget16)) {
            *cfg_idx = i;
            return true;
        }
    }
    int best = -1;
    long best_blocks = -1;
    Tile16 bt{};
    // Among the shapes that fill the chip (four blocks per compute unit), the one whose pixel
    // tiles waste the fewest lanes (a 28x28 plane is 4 tiles of 256 pixels, the last one nearly
    // empty, but exactly 7 tiles of 128: 20 % faster); ties go to the larger shape.
    int full = -1, roomy = -1;
    double full_eff = 0.0;
    Tile16 ft{}, rt{};
    // 1x1 layers (picks of the offline tuner on the MobileNet-shaped pointwise layers at batch 256): planes of
    // up to 64 pixels run 6-15 % faster on the two-by-two wave shape, larger ones on 128-pixel tiles than on 256.
    const bool pointwise = p.KH == 1 && p.KW == 1;
    if (pointwise && p.Hout * p.Wout <= 64) {
        Tile16 t;
        if (plan16_cfg(p, g, kCfg16[5], &t) &&
            (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups >= 2 * kNumCU) {
            *cfg_idx = 5;
            *t_out = t;
            return true;
        }
    }
    // Dense pointwise layers on larger planes: a block of eight waves with 128 filters x 128 pixels reads the input
    // half as often as the 64-filter shapes (two blocks of 64 KB per compute unit).  At N = 256: 128 -> 256 on 56x56
    // 800 -> 705 us, 256 -> 512 on 28x28 602 -> 555 us, 512 -> 1024 on 14x14 627 -> 570 us; wider or taller blocks
    // (128 x 256, 256 x 64) and four-wave blocks of 128 x 128 measured behind it.
    if (pointwise && p.groups == 1 && p.stride == 1) {
        Tile16 t;
        if (plan16_cfg(p, g, kCfg16[kEndKsplit], &t, 64 * 1024) &&
            (long)t.row_blocks * t.img_blocks * t.oc_blocks >= 2 * kNumCU) {
            *cfg_idx = kEndKsplit;
            *t_out = t;
            return true;
        }
    }
    // 3x3 layers whose staged tile is large for its output - stride 2 (four input pixels per output), planes of
    // up to 8x8 pixels (several images and their halos per tile): 32 filters x 64 pixels per block restages the
    // input half as often per multiplication as the 16-filter shapes and won every such layer in the offline
    // tuner's runs (N = 64 and 256: stride-2 stage entries 7-18 % faster, 512-channel 7x7 layers 14 %).
    if (p.KH == 3 && p.KW == 3 && (p.stride == 2 || p.H * p.W <= 64)) {
        for (int i : {7, 6}) {   // 32 x 64, else (16 filters per group) 16 x 128
            Tile16 t;
            if (plan16_cfg(p, g, kCfg16[i], &t) &&
                (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups >= 2 * kNumCU) {
                *cfg_idx = i;
                *t_out = t;
                return true;
            }
        }
    }
    for (int i = 0; i < kFirstKsplit; ++i) {
        Tile16 t;
        if (pointwise && (i == 0 || i == 1)) continue;
        if (!plan16_cfg(p, g, kCfg16[i], &t)) continue;
        const long blocks = (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups;
        if (blocks >= 4 * kNumCU) {
            const Cfg16 &c = kCfg16[i];
            const double eff = (double)p.N * p.Hout * p.Wout /
                               ((double)t.row_blocks * t.img_blocks * 16 * c.NI * c.WP);
            // (only while a wave keeps at least 8 MFMA tiles: smaller shapes lose more in operand reuse)
            if (full < 0 || (eff > full_eff + 0.02 && c.MI * c.NI >= 8)) {
                full = i;
                full_eff = eff;
                ft = t;
            }
            continue;
        }
        if (full >= 0) continue;
        // Smaller launches: the largest shape that still gives 1.5 blocks per compute unit
        // (the autotuner's picks at batch 1 all sit there), else the one with the most blocks.
        if (roomy < 0 && blocks >= 3 * kNumCU / 2) {
            roomy = i;
            rt = t;
        }
        if (blocks >= best_blocks) {   // equal block counts: the smaller tile (less padding)
            best_blocks = blocks;
            best = i;
            bt = t;
        }
    }
    if (full >= 0) {
        *cfg_idx = full;
        *t_out = ft;
        return true;
    }
    // Too few blocks to fill the GPU and a long reduction (small batches): let
    // the waves of a block split the reduction instead of the pixels.
    static const bool no_ksplit = std::getenv("GSPC_NO_KSPLIT") != nullptr;
    if (!no_ksplit && best_blocks < 2 * kNumCU && g.ksteps >= 36) {
        int kbest = -1;
        long kblocks = -1;
        Tile16 kt{};
        for (int i = kFirstKsplit; i < kEndKsplit; ++i) {
            Tile16 t;
            if (!plan16_cfg(p, g, kCfg16[i], &t)) continue;
            const long blocks = (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups;
            if (blocks >= kblocks) {   // equal counts: the smaller tile
                kbest = i;
                kblocks = blocks;
                kt = t;
            }
            if (blocks >= 3 * kNumCU / 2) break;   // the largest tile that gives 1.5 blocks per compute unit
        }
        // else the split shape with the most blocks, unless not splitting gives more
        if (kbest >= 0 && (kblocks >= kNumCU || kblocks >= best_blocks)) {
            *cfg_idx = kbest;
            *t_out = kt;
            return true;
        }
    }
    if (best < 0) {
        // Nothing fits the occupancy-friendly LDS budget (wide rows, 7x7 taps):
        // take the first shape that fits in most of a CU's LDS.
        for (int i = 0; i < kFirstKsplit; ++i) {
            if (plan16_cfg(p, g, kCfg16[i], t_out, 144 * 1024)) {
                *cfg_idx = i;
                return true;
            }
        }
        return false;
    }
    if (roomy >= 0) {
        *cfg_idx = roomy;
        *t_out = rt;
        return true;
    }
    *cfg_idx = best;
    *t_out = bt;
    return true;
}

template <int MI, int NI, int WM, int WP, int KH, int KW, int S, typename TIN, bool VO>
hipError_t launch16_vo(const ConvParams &p, const Tile16 &t, hipStream_t s) {
    size_t lds = (t.one_buf ? 1 : 2) * ((size_t)t.in_floats + t.w_floats + 4) * sizeof(float);
    if (t.ksplit && lds < (size_t)WM * WP * MI * NI * 1024) lds = (size_t)WM * WP * MI * NI * 1024;
    dim3 grid(t.row_blocks * t.img_blocks, p.groups * t.oc_blocks);
    auto kern = conv_mfma16<MI, NI, WM, WP, KH, KW, S, TIN, VO>;
    if (lds > 64 * 1024) {
        static thread_local size_t allowed = 0;   // per instantiation and thread
        if (lds > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
            if (e != hipSuccess) return e;
            allowed = kLdsMax;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(64 * WM * WP), lds, s, p, t);
    return hipGetLastError();
}

template <int MI, int NI, int WM, int WP, int KH, int KW, int S, typename TIN>
hipError_t launch16_inst(const ConvParams &p, const Tile16 &t, hipStream_t s) {
    if constexpr (KH == 7)   // the stem: one layer per network, not worth a second instantiation
        return launch16_vo<MI, NI, WM, WP, KH, KW, S, TIN, false>(p, t, s);
    else
        return t.vec_out ? launch16_vo<MI, NI, WM, WP, KH, KW, S, TIN, true>(p, t, s)
                         : launch16_vo<MI, NI, WM, WP, KH, KW, S, TIN, false>(p, t, s);
}

template <int MI, int NI, int WM, int WP, typename TIN>
hipError_t launch16_shape(const ConvParams &p, const Tile16 &t, hipStream_t s) {
    if (p.KH == 3 && p.stride == 1) return launch16_inst<MI, NI, WM, WP, 3, 3, 1, TIN>(p, t, s);
    if (p.KH == 3 && p.stride == 2) return launch16_inst<MI, NI, WM, WP, 3, 3, 2, TIN>(p, t, s);
    if (p.KH == 1 && p.stride == 1) return launch16_inst<MI, NI, WM, WP, 1, 1, 1, TIN>(p, t, s);
    if (p.KH == 1 && p.stride == 2) return launch16_inst<MI, NI, WM, WP, 1, 1, 2, TIN>(p, t, s);
    if (p.KH == 7 && p.stride == 2) return launch16_inst<MI, NI, WM, WP, 7, 7, 2, TIN>(p, t, s);
    return hipErrorNotSupported;
}

template <typename TIN>
hipError_t launch16_cfg(int i, const ConvParams &p, const Tile16 &t, hipStream_t s) {
    switch (i) {
    case 0: return launch16_shape<4, 4, 1, 4, TIN>(p, t, s);
    case 1: return launch16_shape<2, 4, 1, 4, TIN>(p, t, s);
    case 2: return launch16_shape<4, 2, 1, 4, TIN>(p, t, s);
    case 3: return launch16_shape<2, 2, 1, 4, TIN>(p, t, s);
    case 4: return launch16_shape<1, 4, 1, 4, TIN>(p, t, s);
    case 5: return launch16_shape<2, 2, 2, 2, TIN>(p, t, s);
    case 6: return launch16_shape<1, 2, 1, 4, TIN>(p, t, s);
    case 7: return launch16_shape<2, 1, 1, 4, TIN>(p, t, s);
    case 8: return launch16_shape<1, 1, 1, 4, TIN>(p, t, s);
    case 9: return launch16_shape<2, 2, 1, 4, TIN>(p, t, s);    // ksplit entries
    case 10: return launch16_shape<1, 2, 1, 4, TIN>(p, t, s);
    case 11: return launch16_shape<2, 1, 1, 4, TIN>(p, t, s);
    case 12: return launch16_shape<1, 1, 1, 4, TIN>(p, t, s);
    case 13: return launch16_shape<4, 2, 2, 4, TIN>(p, t, s);
    }
    return hipErrorNotSupported;
}

// Planning costs microseconds of host time, so its outcome is remembered per
// thread, keyed by everything it depends on.
struct PlanKey {
    int v[15];
    bool operator==(const PlanKey &o) const { return std::memcmp(v, o.v, sizeof(v)) == 0; }
};
struct PlanKeyHash {
    size_t operator()(const PlanKey &k) const {
        uint64_t h = 1469598103934665603ull;
        for (int x : k.v) h = (h ^ (uint32_t)x) * 1099511628211ull;
        return (size_t)h;
    }
};
struct Plan {
    int kind;  // 0 none, 32 (bf16), 33 (bf16 row products), 64 (Winograd), 17 (resident filters), 16, 4
    int idx;
    Tile16 t16;
    Mfma4Plan p4;
    MfmaB16Plan pb;
    RowB16Plan pr;
    Mfma16wPlan pw;
    WinoPlan px;
};

const Plan &get_plan(const ConvParams &p, const PackGeom &g) {
    thread_local std::unordered_map<PlanKey, Plan, PlanKeyHash> cache;
    PlanKey k{{p.N, p.Cin, p.H, p.W, p.Cout, p.KH, p.KW, p.stride, p.pad, p.groups, p.in_bf16,
               g.variant, p.wm != nullptr, (p.wb != nullptr) + 2 * (p.wr != nullptr), winograd_mode()}};
    auto it = cache.find(k);
    if (it != cache.end()) return it->second;
    Plan pl{};
    const char fam = tuned_family(p);   // offline tile table: may prefer the plain 16x16x4 kernel
    if ((fam == '\0' || fam == 'r') && plan_row_bf16(p, g, &pl.pr)) pl.kind = 33;
    else if (plan_mfma_bf16(p, g, &pl.pb)) pl.kind = 32;
    else if ((winograd_mode() != 0 || fam == 'x') && (fam == 'x' || fam == '\0') &&
             plan_wino(p, g, winograd_mode() < 0 && fam != 'x', &pl.px))
        pl.kind = 64;
    else if (fam == 'm' && plan16(p, g, &pl.idx, &pl.t16)) pl.kind = 16;
    else if (plan_mfma16w(p, g, &pl.pw)) pl.kind = 17;
    // few filters per group: the 4x4x1 kernel where it has an instance, else padded 16-filter tiles
    else if (g.variant == kMfma4 && fam != 'm' && plan_mfma4(p, g, &pl.p4)) pl.kind = 4;
    else if (plan16(p, g, &pl.idx, &pl.t16)) pl.kind = 16;
    else if (plan_mfma4(p, g, &pl.p4)) pl.kind = 4;
    return cache.emplace(k, pl).first->second;
}

}  // namespace

bool mfma_supported(const ConvParams &p, const PackGeom &g) { return get_plan(p, g).kind != 0; }

hipError_t launch_mfma(const ConvParams &p, const PackGeom &g, hipStream_t s, const char **name) {
    const Plan &pl = get_plan(p, g);
    if (pl.kind == 16) {
        const Cfg16 &c = kCfg16[pl.idx];
        *name = intern_name("conv_mfma16<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," +
                            std::to_string(c.WM) + "," + std::to_string(c.WP) + "," + std::to_string(p.KH) +
                            "," + std::to_string(p.KW) + "," + std::to_string(p.stride) +
                            (p.in_bf16 ? ",bf16," : ",f32,") + (pl.t16.vec_out && p.KH != 7 ? "true>" : "false>") +
                            (c.ksplit ? "/ksplit" : ""));
        return p.in_bf16 ? launch16_cfg<uint16_t>(pl.idx, p, pl.t16, s) : launch16_cfg<float>(pl.idx, p, pl.t16, s);
    }
    if (pl.kind == 32) return launch_mfma_bf16(p, g, pl.pb, s, name);
    if (pl.kind == 33) return launch_row_bf16(p, pl.pr, s, name);
    if (pl.kind == 64) return launch_wino(p, pl.px, s, name);
    if (pl.kind == 17) return launch_mfma16w(p, pl.pw, s, name);
    if (pl.kind == 4) return launch_mfma4(p, pl.p4, s, name);
    return hipErrorNotSupported;
}

}  // namespace gspc
