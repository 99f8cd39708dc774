// bf16 grouped 3x3 convolution on v_mfma_f32_16x16x32_bf16 (fp32 accumulate,
// fp32 NCHW output): the per-group implicit GEMM of mfma_kernels.hip with bf16
// operands, for GSPC_BF16 layers with KPG % 4 == 0 and CPG % 8 == 0 (the last
// 16-filter tile of a group is zero-padded and its surplus rows are not stored).
//
// Operand layout of the instruction (lane l of 64): A = filter row l%16,
// reduction slots 8*(l/16) .. 8*(l/16)+7; B = the same slots of pixel column
// l%16; D register r = (row 4*(l/16) + r, column l%16).  The reduction of a
// chunk of CKB input channels is cut into units of 8 channels at one kernel tap
// (unit u = tap*(CKB/8) + channel block); k-step s feeds unit 4*s + l/16 to lane
// group l/16.  The LDS tile is therefore channel-innermost, [image][row][column]
// [CKB channels], so that a lane's 8 slots are 16 contiguous bytes; the staging
// transposes 8 channels x VW pixels of the NCHW input in registers on the way in
// (the paper's input reshape, fused).  The pixel pitch is padded so that eight
// neighbouring pixels fall into different 16-byte bank groups.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct TileB {
    int NB, TH, IHt, LW;   // images, output rows per block; staged rows; LDS columns (W + 2*pad)
    int PPB, IMGB;         // bytes per pixel / per image in the LDS tile
    int CG;                // column groups of VW pixels per row
    int tasks, tslots;     // staging tasks per chunk (8 channels x VW pixels each), slots per thread
    int wslots;            // 16-byte weight pieces per thread per chunk
    int in_bytes;          // LDS bytes of the input tile (incl. spare area for idle lanes)
    int nchunks, mtiles;
    int row_blocks, img_blocks, oc_blocks;
    int tiles, gx;         // pixel tiles (image groups x row bands); blocks that walk over them
    int wres;              // all chunks' filters stay in LDS
    int vec_out;           // groups of four tile pixels are 16 contiguous, aligned bytes of a plane
    unsigned m_CG, m_IHt, m_NB, m_ppi, m_Wout, m_rowb, m_ocb;
    unsigned x_bytes, w_bytes, y_bytes;
};
static_assert(sizeof(TileB) <= sizeof(((MfmaB16Plan *)0)->data), "plan storage too small");

// Staging widths for which the 16-byte-store instantiation (VO) is the only one built:
// there Wout is a multiple of 4 for a 3x3 window with padding 1 (Wout = W / stride).
constexpr bool always_vec_out(int vw, int stride) { return stride == 1 ? vw >= 4 : vw == 8; }

constexpr int kTmaxB = 4, kWmaxB = 9;
#ifndef GSPC_WAIT_STORES
#define GSPC_WAIT_STORES 1
#endif
constexpr bool kWaitStores = GSPC_WAIT_STORES;   // staging slots per thread (half as many with 8-pixel tasks)

#ifdef GSPC_PHASE_TIMING
__device__ unsigned long long g_phase_b[8 * 4096];
#define GSPC_CLKB(i)                                                   \
    {                                                                  \
        const unsigned long long now = __builtin_amdgcn_s_memtime();   \
        phase_clk[i] += now - phase_t;                                 \
        phase_t = now;                                                 \
    }
#else
#define GSPC_CLKB(i)
#endif

// VW bf16 pixels of one channel row as raw dwords (two pixels per dword).  The vector
// memory path takes a fixed time per wavefront instruction up to 16 bytes per lane, so
// the widest load the row width allows is the cheapest.
template <int VW>
__device__ __forceinline__ u32x4 load_px(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    if (VW == 8) return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    if (VW == 4) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        return u32x4{v.x, v.y, 0u, 0u};
    }
    if (VW == 2) return u32x4{__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0), 0u, 0u, 0u};
    return u32x4{(unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0), 0u, 0u, 0u};
}

template <int MI, int NI, int WM, int WP, int S, int CKB, int VW, bool VO>
__global__ __launch_bounds__(64 * WM * WP, 2) void conv_mfma16b(ConvParams p, TileB t) {
    constexpr int NT = 64 * WM * WP, MIWM = MI * WM;
    constexpr int U8 = CKB / 8, UPC = 9 * U8, KS = (UPC + 3) / 4;
    constexpr int TMAX = VW == 8 ? kTmaxB / 2 : kTmaxB;
    constexpr int WMAX = (KS * MIWM * 64 + NT - 1) / NT;   // 16-byte filter pieces per thread and chunk
    static_assert(WMAX <= kWmaxB, "filter staging slots");
    extern __shared__ f32x4 smem4[];
    char *xs = reinterpret_cast<char *>(smem4);
    char *ws = xs + t.in_bytes;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WP, wp = wave % WP;
    const unsigned j = fast_div(blockIdx.y, t.m_ocb);
    const int ob = blockIdx.y - j * t.oc_blocks;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;
    const unsigned HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wb, t.w_bytes);

    // ---- staging plan: task = ((channel block, image, row), column group).  The part of
    // an address that depends on the lane is computed once; a tile adds its origin. ----
    unsigned xlane[TMAX], xlds[TMAX], ximg[TMAX];
    int xrow[TMAX];
#pragma unroll
    for (int k = 0; k < TMAX; ++k) {
        const int task = tid + k * NT;
        xlane[k] = 0;
        ximg[k] = 0x7fffffffu;              // never a valid image: the slot stays idle
        xrow[k] = 0;
        xlds[k] = t.in_bytes - 8 * t.PPB;   // spare area
        if (k < t.tslots && task < t.tasks) {
            const int rowid = fast_div(task, t.m_CG), cgp = task - rowid * t.CG;
            const int ci = fast_div(rowid, t.m_IHt), r = rowid - ci * t.IHt;
            const int cb8 = fast_div(ci, t.m_NB), img = ci - cb8 * t.NB;
            xlds[k] = ((img * t.IHt + r) * t.LW + cgp * VW + p.pad) * t.PPB + cb8 * 16;
            xlane[k] = (((img * p.Cin + cb8 * 8) * p.H + r) * p.W + cgp * VW) * 2;
            ximg[k] = img;
            xrow[k] = r;
        }
    }
    // weights of a chunk: KS * MIWM kilobytes, contiguous per k-step in the section
    const unsigned wrow = t.mtiles * 1024;   // bytes per k-step
    const unsigned wblk = (j * t.nchunks * KS * t.mtiles + ob * MIWM) * 1024;
    const unsigned wvoff = (tid / (MIWM * 64)) * wrow + (tid % (MIWM * 64)) * 16;
    constexpr int kWstep = NT / (MIWM * 64);   // k-steps advanced per slot
    static_assert(NT % (MIWM * 64) == 0, "a weight slot must cover whole k-steps");
    const unsigned wchunk = t.wslots * NT * 16;   // LDS bytes of one chunk's filters

    // ---- per-lane pixel coordinates and reduction-unit offsets -------------------
    // Operand reads: lane l multiplies pixel (l % 16) of each 16-pixel column block.
    // Results, VO: the pixels are the rows of the MFMA product (the input tile is its A
    // operand), so that lane l holds, per block, pixels 4*(l/16) .. +3 of filter l % 16:
    // four consecutive pixels of one output plane, one 16-byte store.  Otherwise the
    // filters are the rows: lane l holds filters 4*(l/16) .. +3 at pixel l % 16, and a
    // store instruction writes 16 consecutive pixels of 4 planes.
    unsigned pixb[NI], olane[NI], oimg[NI], orem[NI];
    const unsigned HWo = p.Hout * p.Wout;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * 16 + (lane & 15);
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_Wout), col = rem - r * p.Wout;
        pixb[ni] = ((img * t.IHt + r * S) * t.LW + col * S) * t.PPB;
        if (VO) {
            const int q0 = (wp * NI + ni) * 16 + 4 * (lane >> 4);
            const int qq0 = q0 < tot ? q0 : 0;
            const int img0 = fast_div(qq0, t.m_ppi), rem0 = qq0 - img0 * ppi;
            oimg[ni] = q0 < tot ? img0 : 0x7fffffffu;
            orem[ni] = rem0;
            olane[ni] = (((unsigned)img0 * p.Cout + (lane & 15)) * HWo + rem0) * 4;
        } else {
            oimg[ni] = q < tot ? img : 0x7fffffffu;
            orem[ni] = rem;
            olane[ni] = (((unsigned)img * p.Cout + 4 * (lane >> 4)) * HWo + rem) * 4;
        }
    }
    // Byte offset of k-step ks, lane group l/16, inside the tile relative to the pixel.
    // With four channel blocks per chunk a k-step is one tap and the group picks the block:
    // the tap part is uniform.  Otherwise the offsets are per lane.
    constexpr bool TAPK = U8 == 4;
    unsigned uoff[TAPK ? 1 : KS];
    if (TAPK) {
        uoff[0] = (lane >> 4) * 16;
    } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int u = 4 * ks + (lane >> 4);
            const int tap = u / U8, cb8 = u % U8;
            uoff[ks] = u < UPC ? ((tap / 3) * t.LW + tap % 3) * t.PPB + cb8 * 16 : 0u;
        }
    }
    auto unit_off = [&](int ks) -> unsigned {
        return TAPK ? uoff[0] + ((ks / 3) * t.LW + ks % 3) * t.PPB : uoff[ks];
    };

    // Origin of pixel tile tg (an image group and a band of output rows): first image, the
    // number of output elements left in a plane from the band's first row, byte offset of
    // (first image, filter 0 of the group, first row).  Uniform over the block.
    struct TileU {
        unsigned n0, lim, ot;
    };
    // Staging offsets of tile tg; everything is out of range, hence loads zero and stores
    // nothing, when the tile does not exist.
    auto set_tile = [&](unsigned tg, unsigned (&xo)[TMAX], TileU &u) {
        const bool live = tg < (unsigned)t.tiles;
        const unsigned ib = fast_div(tg, t.m_rowb);
        const int rb = tg - ib * t.row_blocks;
        const unsigned n0 = ib * t.NB;
        const int oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
        const unsigned xt = (((n0 * p.Cin + j * p.CPG) * p.H + ih0) * p.W) * 2;
        u.n0 = live ? n0 : 0x7fffffffu;
        u.lim = HWo - oh0 * p.Wout;
        u.ot = ((n0 * p.Cout + j * p.KPG) * HWo + oh0 * p.Wout) * 4;
#pragma unroll
        for (int k = 0; k < TMAX; ++k)
            xo[k] = (live && n0 + ximg[k] < (unsigned)p.N && (unsigned)(ih0 + xrow[k]) < (unsigned)p.H)
                        ? xt + xlane[k]
                        : kOob;
    };

    f32x4 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Halo columns are never written by the staging: clear them once.
    {
        const int pieces = CKB / 8;                      // 16-byte pieces per pixel
        const int halo = 2 * p.pad * pieces, rows = t.NB * t.IHt;
        for (int i = tid; i < rows * halo; i += NT) {
            const int row = i / halo, h = i - row * halo;
            const int hp = h / pieces, pc = h - hp * pieces;
            const int col = hp < p.pad ? hp : p.W + hp;   // left columns, then right columns
            *reinterpret_cast<f32x4 *>(xs + (row * t.LW + col) * t.PPB + pc * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // ---- a block walks over (pixel tile, channel chunk) steps, tiles blockIdx.x,
    // blockIdx.x + gridDim.x, ...; the global loads of step i+1 are in flight while step
    // i multiplies.  With t.wres the filters of every chunk are staged during the first
    // tile only and stay in LDS. ----
    f32x4 pw[WMAX];
    u32x4 v[TMAX][8];
    auto prefetch = [&](const unsigned (&xo)[TMAX], int ch, bool need_w) {
        if (need_w) {
            const unsigned so = wblk + ch * KS * wrow;
#pragma unroll
            for (int k = 0; k < WMAX; ++k)
                if (k < t.wslots)
                    pw[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff, so + k * kWstep * wrow, 0));
        }
#pragma unroll
        for (int k = 0; k < TMAX; ++k)
            if (k < t.tslots)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[k][e] = load_px<VW>(rx, xo[k], (ch * CKB + e) * HW * 2);
    };

    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    const unsigned oc0 = (ob * MIWM + wm * MI) * 16;

    // Tiles in XCD-aware order: workgroups go to the chip's eight XCDs (each with its own L2) in turn,
    // so the blocks of one XCD are given neighbouring tiles - bands of the same image, whose halo rows
    // then meet in that L2 instead of being fetched from memory once per XCD.
    const unsigned bx0 = (gridDim.x & 7) == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    unsigned tg = bx0;
    int ch = 0;
    unsigned xo_n[TMAX];
    TileU tu_n, tu;
    set_tile(tg, xo_n, tu_n);
    prefetch(xo_n, 0, true);
    bool first_step = true;
#ifdef GSPC_PHASE_TIMING
    unsigned long long phase_clk[8] = {0, 0, 0, 0, 0, 0, 0, 0}, phase_t = __builtin_amdgcn_s_memtime();
#endif
    for (;;) {
        const bool first = tg == bx0;
        if (ch == 0) tu = tu_n;
        __syncthreads();   // everyone is done reading the previous step's tile
        GSPC_CLKB(0)
        char *wcur = ws + (t.wres ? ch * wchunk : 0u);
        if (!t.wres || first) {
#pragma unroll
            for (int k = 0; k < WMAX; ++k)
                if (k < t.wslots) *reinterpret_cast<f32x4 *>(wcur + (tid + k * NT) * 16) = pw[k];
        }
        // input: 8 channels x VW pixels per task, transposed in registers
#pragma unroll
        for (int k = 0; k < TMAX; ++k) {
            if (k < t.tslots) {
#pragma unroll
                for (int px = 0; px < VW; ++px) {
                    u32x4 o;
#pragma unroll
                    for (int h = 0; h < 4; ++h)   // channels 2h (low half) and 2h+1 of pixel px
                        o[h] = __builtin_amdgcn_perm(v[k][2 * h + 1][px / 2], v[k][2 * h][px / 2],
                                                     (px & 1) ? 0x07060302u : 0x05040100u);
                    *reinterpret_cast<u32x4 *>(xs + xlds[k] + px * t.PPB) = o;
                }
            }
        }
        GSPC_CLKB(1)
        __syncthreads();
        GSPC_CLKB(2)
        // ---- next step's loads ----------------------------------------------------------
        int nch = ch + 1;
        unsigned ntg = tg;
        if (nch == t.nchunks) {
            nch = 0;
            ntg = tg + gridDim.x;
            set_tile(ntg, xo_n, tu_n);
        }
        const bool more = ntg < (unsigned)t.tiles;
        if (ch == 0 && !first_step) {
            // a new tile: wait for the previous tile's stores (nothing else is in flight
            // here), then clear the accumulators they read from
            if (kWaitStores) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                {
                    asm volatile("" : "+v"(acc[mi][ni]));   // the old value lives in its registers up to here
                    acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
        first_step = false;
        prefetch(xo_n, nch, more && (!t.wres || ntg == bx0));
        __builtin_amdgcn_sched_barrier(0);
        GSPC_CLKB(3)
        // ---- multiply: the operands of k-step s+1 are read from LDS while the matrix
        // unit works on k-step s ----
        // (a wave tile of sixteen MFMAs per k-step would keep one operand set: a second one does not fit the
        // register file; no such instance is built at present - with its staging registers the 64 x 64 tile
        // spills even so, and ran at half the speed of the 32 x 64 one)
        constexpr bool DB = MI * NI < 16;
        bf16x8 opa[DB ? 2 : 1][MI], opb[DB ? 2 : 1][NI];
        auto load_ops = [&](int ks, int set) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                opa[set][mi] = *reinterpret_cast<const bf16x8 *>(wcur + ((ks * MIWM + wm * MI + mi) * 64 + lane) * 16);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                opb[set][ni] = *reinterpret_cast<const bf16x8 *>(xs + pixb[ni] + unit_off(ks));
        };
        if (DB) load_ops(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (!DB) load_ops(ks, 0);
            else if (ks + 1 < KS) load_ops(ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int dummy = 0;
            const int set = DB ? (ks & 1) : dummy;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = VO ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(opb[set][ni], opa[set][mi], acc[mi][ni], 0, 0, 0)
                                     : __builtin_amdgcn_mfma_f32_16x16x32_bf16(opa[set][mi], opb[set][ni], acc[mi][ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        GSPC_CLKB(4)
        if (ch == t.nchunks - 1) {
            // ---- epilogue: optional residual and ReLU, NCHW store; filters past KPG belong
            // to the zero-padded part of the last filter tile ----
            unsigned off[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                off[ni] = (tu.n0 + oimg[ni] < (unsigned)p.N && orem[ni] < tu.lim) ? tu.ot + olane[ni] : kOob;
            if (p.res) {
                f32x4 rv[MI][NI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        if (VO) {
                            rv[mi][ni] = __builtin_bit_cast(
                                f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                           rr, oc0 + mi * 16 + (lane & 15) < (unsigned)p.KPG ? off[ni] : kOob,
                                           (oc0 + mi * 16) * HWo * 4, 0));
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                rv[mi][ni][r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                                    rr, oc0 + mi * 16 + 4 * (lane >> 4) < (unsigned)p.KPG ? off[ni] : kOob,
                                    (oc0 + mi * 16 + r) * HWo * 4, 0));
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
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
            // The stores read the accumulator registers themselves, and those registers are
            // left alone until the stores have completed (see the clearing above): a 16-byte
            // store whose data registers were overwritten right after it has been seen to
            // write the new value of its last dword.
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    if (VO) {
                        __builtin_amdgcn_raw_buffer_store_b128(
                            __builtin_bit_cast(u32x4, acc[mi][ni]), ry,
                            oc0 + mi * 16 + (lane & 15) < (unsigned)p.KPG ? off[ni] : kOob, (oc0 + mi * 16) * HWo * 4, 0);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            __builtin_amdgcn_raw_buffer_store_b32(
                                __float_as_uint(acc[mi][ni][r]), ry,
                                oc0 + mi * 16 + 4 * (lane >> 4) < (unsigned)p.KPG ? off[ni] : kOob,
                                (oc0 + mi * 16 + r) * HWo * 4, 0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        GSPC_CLKB(5)
#ifdef GSPC_PHASE_TIMING
        phase_clk[6] += 1;
#endif
        if (!more) break;
        tg = ntg;
        ch = nch;
    }
#ifdef GSPC_PHASE_TIMING
    if (threadIdx.x == 0) {
        const unsigned bid = blockIdx.x + blockIdx.y * gridDim.x;
        if (bid < 4096)
            for (int i = 0; i < 8; ++i) g_phase_b[bid * 8 + i] = phase_clk[i];
    }
#endif
}

#ifdef GSPC_PHASE_TIMING
extern "C" int gspc_debug_phases_b(unsigned long long *out, int n) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_b), sizeof(unsigned long long) * n);
}
#endif

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

constexpr int kLdsBudgetB = 64 * 1024;   // tile and one chunk of filters
constexpr int kLdsResB = 80 * 1024;      // with every chunk's filters: two blocks per compute unit

struct CfgB {
    int MI, NI, WM, WP;
};
const CfgB kCfgB[] = {{2, 4, 1, 4}, {1, 4, 1, 4}, {2, 2, 1, 4}, {1, 2, 1, 4}, {2, 1, 1, 4}, {1, 1, 1, 4}, {4, 2, 1, 4}};
constexpr int kNumCfgB = sizeof(kCfgB) / sizeof(kCfgB[0]);

int vw_of(int W) { return W % 8 == 0 ? 8 : W % 4 == 0 ? 4 : W % 2 == 0 ? 2 : 1; }

bool planB_cfg(const ConvParams &p, const PackGeom &g, const CfgB &c, TileB *out) {
    const int MB = 16 * c.MI * c.WM, PB = 16 * c.NI * c.WP, NT = 64 * c.WM * c.WP;
    if ((g.mtiles_b * 16) % MB) return false;
    if (c.MI == 4 && g.ckb != 32) return false;
    TileB t{};
    if (!split_pixels(p, PB, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * p.stride + 3;
    t.LW = p.W + 2 * p.pad;
    t.PPB = round_up(g.ckb * 2, 32) + 16;
    t.IMGB = t.IHt * t.LW * t.PPB;
    const int vw = vw_of(p.W);
    t.CG = p.W / vw;
    t.tasks = (g.ckb / 8) * t.NB * t.IHt * t.CG;
    t.tslots = (t.tasks + NT - 1) / NT;
    t.wslots = (g.ks_b * c.MI * c.WM * 64 + NT - 1) / NT;
    if (t.tslots > (vw == 8 ? kTmaxB / 2 : kTmaxB) || t.wslots > kWmaxB) return false;

    t.in_bytes = t.NB * t.IMGB + 8 * t.PPB;
    const size_t wchunk = (size_t)t.wslots * NT * 16;
    // (64-filter blocks carry 36 KB of filters per chunk: they may fill half a compute unit's LDS)
    if (t.in_bytes + wchunk > (size_t)(c.MI == 4 ? kLdsResB : kLdsBudgetB)) return false;
    t.wres = t.in_bytes + g.nchunks_b * wchunk <= (size_t)kLdsResB;
    t.nchunks = g.nchunks_b;
    t.mtiles = g.mtiles_b;
    t.row_blocks = (p.Hout + t.TH - 1) / t.TH;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.oc_blocks = g.mtiles_b * 16 / MB;
    t.m_CG = div_magic(t.CG);
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.Wout);
    t.m_Wout = div_magic(p.Wout);
    t.m_rowb = div_magic(t.row_blocks);
    t.m_ocb = div_magic(t.oc_blocks);
    const double xb = (double)p.N * p.Cin * p.H * p.W * 2;
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    if (xb >= (double)kOob || yb >= (double)kOob || (double)g.bf16_bytes >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)g.bf16_bytes;
    if ((double)t.row_blocks * t.img_blocks * t.row_blocks >= 4.0e9 ||
        (double)p.groups * t.oc_blocks * t.oc_blocks >= 4.0e9 || t.tasks >= 65536 || t.TH * p.Wout >= 65536 ||
        (long)t.row_blocks * t.img_blocks > 2147483647L || p.groups * t.oc_blocks > 65535)
        return false;
    t.tiles = t.row_blocks * t.img_blocks;
    t.vec_out = (t.TH * p.Wout) % 4 == 0 && (p.Hout * p.Wout) % 4 == 0;
    if (always_vec_out(vw, p.stride) && !t.vec_out) return false;   // unusual padding: other kernels
    {
        // one resident set of blocks walks over the tiles in equal shares
        const long gy = (long)p.groups * t.oc_blocks;
        long cap = 2L * kNumCU / gy;   // two blocks per compute unit
        cap = cap < 1 ? 1 : cap;
        const long rounds = (t.tiles + cap - 1) / cap;
        t.gx = (int)((t.tiles + rounds - 1) / rounds);
        if (t.gx >= 8) t.gx = round_up(t.gx, 8);   // the kernel's XCD-aware tile order wants a multiple of 8
    }
    *out = t;
    return true;
}

template <int MI, int NI, int WM, int WP, int S, int CKB, int VW, bool VO>
hipError_t launchB_vo(const ConvParams &p, const TileB &t, hipStream_t s) {
    const size_t lds = (size_t)t.in_bytes + (size_t)(t.wres ? t.nchunks : 1) * t.wslots * 64 * WM * WP * 16;
    dim3 grid(t.gx, p.groups * t.oc_blocks);
    auto kern = conv_mfma16b<MI, NI, WM, WP, S, CKB, VW, VO>;
    if (lds > 64 * 1024) {
        static thread_local bool raised = false;   // per instantiation and thread
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsResB);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(64 * WM * WP), lds, s, p, t);
    return hipGetLastError();
}

template <int MI, int NI, int WM, int WP, int S, int CKB, int VW>
hipError_t launchB_inst(const ConvParams &p, const TileB &t, hipStream_t s) {
    if (t.vec_out) return launchB_vo<MI, NI, WM, WP, S, CKB, VW, true>(p, t, s);
    if constexpr (always_vec_out(VW, S))
        return hipErrorNotSupported;   // the planner does not produce this
    else
        return launchB_vo<MI, NI, WM, WP, S, CKB, VW, false>(p, t, s);
}

template <int MI, int NI, int WM, int WP, int S, int CKB>
hipError_t launchB_vw(int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    if (vw == 8) return launchB_inst<MI, NI, WM, WP, S, CKB, 8>(p, t, s);
    if (vw == 4) return launchB_inst<MI, NI, WM, WP, S, CKB, 4>(p, t, s);
    if (vw == 2) return launchB_inst<MI, NI, WM, WP, S, CKB, 2>(p, t, s);
    return launchB_inst<MI, NI, WM, WP, S, CKB, 1>(p, t, s);
}

template <int MI, int NI, int WM, int WP, int S>
hipError_t launchB_ckb(int ckb, int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    if (ckb == 32) return launchB_vw<MI, NI, WM, WP, S, 32>(vw, p, t, s);
    if constexpr (MI == 4) {   // 64 filters per block: built for the 32-channel chunks of wide groups only
        return hipErrorNotSupported;
    } else {
        if (ckb == 16) return launchB_vw<MI, NI, WM, WP, S, 16>(vw, p, t, s);
        return launchB_vw<MI, NI, WM, WP, S, 8>(vw, p, t, s);
    }
}

template <int MI, int NI, int WM, int WP>
hipError_t launchB_s(int ckb, int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    return p.stride == 1 ? launchB_ckb<MI, NI, WM, WP, 1>(ckb, vw, p, t, s)
                         : launchB_ckb<MI, NI, WM, WP, 2>(ckb, vw, p, t, s);
}

}  // namespace

// The layer as the 16x16x32 section sees it: merged groups (block-diagonal weights).
static ConvParams merged_view(const ConvParams &p0, const PackGeom &g) {
    ConvParams p = p0;
    if (g.bf16_bytes) {
        p.groups = g.gb;
        p.CPG = g.CPGb;
        p.KPG = g.KPGb;
    }
    return p;
}

bool plan_mfma_bf16(const ConvParams &p0, const PackGeom &g, MfmaB16Plan *out) {
    const ConvParams p = merged_view(p0, g);
    if (!p.in_bf16 || !p.wb || !g.bf16_bytes || p.KH != 3 || p.KW != 3 || (p.stride != 1 && p.stride != 2))
        return false;
    static const char *force = std::getenv("GSPC_TILEB");
    int forced = force ? std::atoi(force) : tuned_config(p, 'b');
    {
        TileB t;
        if (!force && forced >= 0 && (forced >= kNumCfgB || !planB_cfg(p, g, kCfgB[forced], &t))) forced = -1;
    }
    int best = -1;
    long best_blocks = -1;
    TileB bt{};
    // Planes of up to 8 x 8 pixels (several images per tile, so a tile's staging is all halo and index
    // work) and stride-2 layers (the staged tile is four times the output tile): 64 filters per block
    // halve the staging per multiplication (N = 256: the 512-channel 7x7 layers 62 -> 46 us for g = 2 and
    // 20 -> 18 us for g = 8; 128 -> 256 on 28x28 stride 2 45 -> 41 us, 256 -> 512 on 14x14 stride 2 44 -> 36 us;
    // on stride-1 planes of 14 x 14 and up it changes nothing).
    if (forced < 0 && (p.H * p.W <= 64 || p.stride == 2)) {
        TileB t;
        if (planB_cfg(p, g, kCfgB[kNumCfgB - 1], &t) &&
            (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups >= 4 * kNumCU) {
            out->inst = kNumCfgB - 1;
            std::memcpy(out->data, &t, sizeof(t));
            return true;
        }
    }
    for (int i = 0; i < kNumCfgB; ++i) {
        TileB t;
        if (forced >= 0 && forced != i) continue;
        if (forced < 0 && kCfgB[i].MI == 4) continue;   // only by the rule above or when asked for
        if (!planB_cfg(p, g, kCfgB[i], &t)) continue;
        const long blocks = (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups;
        if (blocks >= 4 * kNumCU) {
            best = i;
            bt = t;
            break;
        }
        if (blocks > best_blocks) {
            best_blocks = blocks;
            best = i;
            bt = t;
        }
    }
    if (best < 0) return false;
    out->inst = best;
    std::memcpy(out->data, &bt, sizeof(bt));
    return true;
}

hipError_t launch_mfma_bf16(const ConvParams &p0, const PackGeom &g, const MfmaB16Plan &plan, hipStream_t s,
                            const char **name) {
    const ConvParams p = merged_view(p0, g);
    TileB t;
    std::memcpy(&t, plan.data, sizeof(t));
    const CfgB &c = kCfgB[plan.inst];
    const int vw = vw_of(p.W);
    *name = intern_name("conv_mfma16b<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," +
                        std::to_string(c.WM) + "," + std::to_string(c.WP) + "," + std::to_string(p.stride) + "," +
                        std::to_string(g.ckb) + "," + std::to_string(vw) + (t.vec_out ? ",true>" : ",false>") +
                        (g.mb > 1 ? "/merge" + std::to_string(g.mb) : ""));
    switch (plan.inst) {
    case 0: return launchB_s<2, 4, 1, 4>(g.ckb, vw, p, t, s);
    case 1: return launchB_s<1, 4, 1, 4>(g.ckb, vw, p, t, s);
    case 2: return launchB_s<2, 2, 1, 4>(g.ckb, vw, p, t, s);
    case 3: return launchB_s<1, 2, 1, 4>(g.ckb, vw, p, t, s);
    case 4: return launchB_s<2, 1, 1, 4>(g.ckb, vw, p, t, s);
    case 5: return launchB_s<1, 1, 1, 4>(g.ckb, vw, p, t, s);
    case 6: return launchB_s<4, 2, 1, 4>(g.ckb, vw, p, t, s);
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
