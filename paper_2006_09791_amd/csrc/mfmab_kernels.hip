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
    unsigned m_CG, m_IHt, m_NB, m_ppi, m_Wout, m_rowb, m_ocb;
    unsigned x_bytes, w_bytes, y_bytes;
};
static_assert(sizeof(TileB) <= sizeof(((MfmaB16Plan *)0)->data), "plan storage too small");

constexpr int kTmaxB = 4, kWmaxB = 6;

// VW bf16 pixels of one channel row as raw dwords (VW = 4: 2 dwords, else 1).
template <int VW>
__device__ __forceinline__ u32x2 load_px(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    if (VW == 4) return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
    if (VW == 2) return u32x2{__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0), 0u};
    return u32x2{(unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0), 0u};
}

template <int MI, int NI, int WM, int WP, int S, int CKB, int VW>
__global__ __launch_bounds__(64 * WM * WP) void conv_mfma16b(ConvParams p, TileB t) {
    constexpr int NT = 64 * WM * WP, MIWM = MI * WM;
    constexpr int U8 = CKB / 8, UPC = 9 * U8, KS = (UPC + 3) / 4;
    extern __shared__ f32x4 smem4[];
    char *xs = reinterpret_cast<char *>(smem4);
    char *ws = xs + t.in_bytes;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WP, wp = wave % WP;
    const unsigned ib = fast_div(blockIdx.x, t.m_rowb);
    const int rb = blockIdx.x - ib * t.row_blocks;
    const unsigned j = fast_div(blockIdx.y, t.m_ocb);
    const int ob = blockIdx.y - j * t.oc_blocks;
    const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;
    const unsigned HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wb, t.w_bytes);

    // ---- staging plan: task = ((channel block, image, row), column group) ----
    unsigned xoff[kTmaxB], xlds[kTmaxB];
#pragma unroll
    for (int k = 0; k < kTmaxB; ++k) {
        const int task = tid + k * NT;
        xoff[k] = kOob;
        xlds[k] = t.in_bytes - 4 * t.PPB;   // spare area
        if (k < t.tslots && task < t.tasks) {
            const int rowid = fast_div(task, t.m_CG), cgp = task - rowid * t.CG;
            const int ci = fast_div(rowid, t.m_IHt), r = rowid - ci * t.IHt;
            const int cb8 = fast_div(ci, t.m_NB), img = ci - cb8 * t.NB;
            const int ih = ih0 + r, n = n0 + img;
            xlds[k] = ((img * t.IHt + r) * t.LW + cgp * VW + p.pad) * t.PPB + cb8 * 16;
            if (n < p.N && ih >= 0 && ih < p.H)
                xoff[k] = (((n * p.Cin + j * p.CPG + cb8 * 8) * p.H + ih) * p.W + cgp * VW) * 2;
        }
    }
    // weights of a chunk: KS * MIWM kilobytes, contiguous per k-step in the section
    const unsigned wrow = t.mtiles * 1024;   // bytes per k-step
    const unsigned wblk = (j * t.nchunks * KS * t.mtiles + ob * MIWM) * 1024;
    const unsigned wvoff = (tid / (MIWM * 64)) * wrow + (tid % (MIWM * 64)) * 16;
    constexpr int kWstep = NT / (MIWM * 64);   // k-steps advanced per slot
    static_assert(NT % (MIWM * 64) == 0, "a weight slot must cover whole k-steps");

    // ---- per-lane pixel coordinates and reduction-unit offsets -------------------
    unsigned pixb[NI], ooff[NI];
    const unsigned HWo = p.Hout * p.Wout;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * 16 + (lane & 15);
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_Wout), col = rem - r * p.Wout;
        pixb[ni] = ((img * t.IHt + r * S) * t.LW + col * S) * t.PPB;
        const int n = n0 + img, oh = oh0 + r;
        ooff[ni] = (q < tot && n < p.N && oh < p.Hout)
                       ? (((unsigned)n * p.Cout + j * p.KPG + 4 * (lane >> 4)) * HWo + oh * p.Wout + col) * 4
                       : kOob;
    }
    unsigned uoff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int u = 4 * ks + (lane >> 4);
        const int tap = u / U8, cb8 = u % U8;
        uoff[ks] = u < UPC ? ((tap / 3) * t.LW + tap % 3) * t.PPB + cb8 * 16 : 0u;
    }

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

    for (int ch = 0; ch < t.nchunks; ++ch) {
        if (ch) __syncthreads();   // everyone is done reading the previous chunk
        // ---- weights: global -> LDS ---------------------------------------------
        {
            f32x4 pw[kWmaxB];
            const unsigned so = wblk + ch * KS * wrow;
#pragma unroll
            for (int k = 0; k < kWmaxB; ++k)
                if (k < t.wslots)
                    pw[k] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff, so + k * kWstep * wrow, 0));
            // ---- input: 8 channels x VW pixels per task, transposed in registers ------
            u32x2 v[kTmaxB][8];
#pragma unroll
            for (int k = 0; k < kTmaxB; ++k)
                if (k < t.tslots)
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[k][e] = load_px<VW>(rx, xoff[k], (ch * CKB + e) * HW * 2);
#pragma unroll
            for (int k = 0; k < kWmaxB; ++k)
                if (k < t.wslots) *reinterpret_cast<f32x4 *>(ws + (tid + k * NT) * 16) = pw[k];
#pragma unroll
            for (int k = 0; k < kTmaxB; ++k) {
                if (k < t.tslots) {
#pragma unroll
                    for (int px = 0; px < VW; ++px) {
                        u32x4 o;
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            const unsigned lo = px < 2 ? v[k][2 * h].x : v[k][2 * h].y;
                            const unsigned hi = px < 2 ? v[k][2 * h + 1].x : v[k][2 * h + 1].y;
                            o[h] = (px & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
                        }
                        *reinterpret_cast<u32x4 *>(xs + xlds[k] + px * t.PPB) = o;
                    }
                }
            }
        }
        __syncthreads();
        // ---- multiply ------------------------------------------------------------------
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a[MI], b[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                a[mi] = *reinterpret_cast<const bf16x8 *>(ws + ((ks * MIWM + wm * MI + mi) * 64 + lane) * 16);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) b[ni] = *reinterpret_cast<const bf16x8 *>(xs + pixb[ni] + uoff[ks]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        }
    }

    // ---- epilogue: optional residual and ReLU, NCHW store (as in the fp32 kernel) ----
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const unsigned oc0 = (ob * MIWM + wm * MI) * 16;
    if (p.res) {
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[mi][ni][r] += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                        rr, oc0 + mi * 16 + 4 * (lane >> 4) < (unsigned)p.KPG ? ooff[ni] : kOob,
                        (oc0 + mi * 16 + r) * HWo * 4, 0));
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[mi][ni][r];
                if (p.relu) v = fmaxf(v, 0.f);
                // rows past KPG belong to the zero-padded part of the last filter tile
                __builtin_amdgcn_raw_buffer_store_b32(
                    __float_as_uint(v), ry, oc0 + mi * 16 + 4 * (lane >> 4) < (unsigned)p.KPG ? ooff[ni] : kOob,
                    (oc0 + mi * 16 + r) * HWo * 4, 0);
            }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

constexpr int kLdsBudgetB = 64 * 1024;

struct CfgB {
    int MI, NI, WM, WP;
};
const CfgB kCfgB[] = {{2, 4, 1, 4}, {1, 4, 1, 4}, {2, 2, 1, 4}, {1, 2, 1, 4}, {2, 1, 1, 4}, {1, 1, 1, 4}};
constexpr int kNumCfgB = sizeof(kCfgB) / sizeof(kCfgB[0]);

bool planB_cfg(const ConvParams &p, const PackGeom &g, const CfgB &c, TileB *out) {
    const int MB = 16 * c.MI * c.WM, PB = 16 * c.NI * c.WP, NT = 64 * c.WM * c.WP;
    if ((g.mtiles_b * 16) % MB) return false;
    TileB t{};
    if (!split_pixels(p, PB, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * p.stride + 3;
    t.LW = p.W + 2 * p.pad;
    t.PPB = round_up(g.ckb * 2, 32) + 16;
    t.IMGB = t.IHt * t.LW * t.PPB;
    const int vw = p.W % 4 == 0 ? 4 : p.W % 2 == 0 ? 2 : 1;
    t.CG = p.W / vw;
    t.tasks = (g.ckb / 8) * t.NB * t.IHt * t.CG;
    t.tslots = (t.tasks + NT - 1) / NT;
    t.wslots = (g.ks_b * c.MI * c.WM * 64 + NT - 1) / NT;
    if (t.tslots > kTmaxB || t.wslots > kWmaxB) return false;
    t.in_bytes = t.NB * t.IMGB + 4 * t.PPB;
    const size_t lds = (size_t)t.in_bytes + (size_t)t.wslots * NT * 16;
    if (lds > (size_t)kLdsBudgetB) return false;
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
    *out = t;
    return true;
}

template <int MI, int NI, int WM, int WP, int S, int CKB, int VW>
hipError_t launchB_inst(const ConvParams &p, const TileB &t, hipStream_t s) {
    const size_t lds = (size_t)t.in_bytes + (size_t)t.wslots * 64 * WM * WP * 16;
    dim3 grid(t.row_blocks * t.img_blocks, p.groups * t.oc_blocks);
    hipLaunchKernelGGL((conv_mfma16b<MI, NI, WM, WP, S, CKB, VW>), grid, dim3(64 * WM * WP), lds, s, p, t);
    return hipGetLastError();
}

template <int MI, int NI, int WM, int WP, int S, int CKB>
hipError_t launchB_vw(int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    if (vw == 4) return launchB_inst<MI, NI, WM, WP, S, CKB, 4>(p, t, s);
    if (vw == 2) return launchB_inst<MI, NI, WM, WP, S, CKB, 2>(p, t, s);
    return launchB_inst<MI, NI, WM, WP, S, CKB, 1>(p, t, s);
}

template <int MI, int NI, int WM, int WP, int S>
hipError_t launchB_ckb(int ckb, int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    if (ckb == 32) return launchB_vw<MI, NI, WM, WP, S, 32>(vw, p, t, s);
    if (ckb == 16) return launchB_vw<MI, NI, WM, WP, S, 16>(vw, p, t, s);
    return launchB_vw<MI, NI, WM, WP, S, 8>(vw, p, t, s);
}

template <int MI, int NI, int WM, int WP>
hipError_t launchB_s(int ckb, int vw, const ConvParams &p, const TileB &t, hipStream_t s) {
    return p.stride == 1 ? launchB_ckb<MI, NI, WM, WP, 1>(ckb, vw, p, t, s)
                         : launchB_ckb<MI, NI, WM, WP, 2>(ckb, vw, p, t, s);
}

}  // namespace

bool plan_mfma_bf16(const ConvParams &p, const PackGeom &g, MfmaB16Plan *out) {
    if (!p.in_bf16 || !p.wb || !g.bf16_bytes || p.KH != 3 || p.KW != 3 || (p.stride != 1 && p.stride != 2))
        return false;
    static const char *force = std::getenv("GSPC_TILEB");
    int best = -1;
    long best_blocks = -1;
    TileB bt{};
    for (int i = 0; i < kNumCfgB; ++i) {
        TileB t;
        if (force && std::atoi(force) != i) continue;
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

hipError_t launch_mfma_bf16(const ConvParams &p, const PackGeom &g, const MfmaB16Plan &plan, hipStream_t s,
                            const char **name) {
    TileB t;
    std::memcpy(&t, plan.data, sizeof(t));
    const CfgB &c = kCfgB[plan.inst];
    const int vw = p.W % 4 == 0 ? 4 : p.W % 2 == 0 ? 2 : 1;
    *name = intern_name("conv_mfma16b<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," +
                        std::to_string(c.WM) + "," + std::to_string(c.WP) + "," + std::to_string(p.stride) + "," +
                        std::to_string(g.ckb) + "," + std::to_string(vw) + ">");
    switch (plan.inst) {
    case 0: return launchB_s<2, 4, 1, 4>(g.ckb, vw, p, t, s);
    case 1: return launchB_s<1, 4, 1, 4>(g.ckb, vw, p, t, s);
    case 2: return launchB_s<2, 2, 1, 4>(g.ckb, vw, p, t, s);
    case 3: return launchB_s<1, 2, 1, 4>(g.ckb, vw, p, t, s);
    case 4: return launchB_s<2, 1, 1, 4>(g.ckb, vw, p, t, s);
    case 5: return launchB_s<1, 1, 1, 4>(g.ckb, vw, p, t, s);
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
