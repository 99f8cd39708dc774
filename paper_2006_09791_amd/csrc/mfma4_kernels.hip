// Grouped 3x3 convolution for groups with few filters (KPG a multiple of 4 but
// not of 16) on the 4x4x1 matrix-core instruction.
//
// v_mfma_f32_4x4x1_16b_f32 performs sixteen independent 4x4 outer products:
// lane l belongs to block l/4, supplies A row l%4 and B column l%4, and
// receives D register r = (row r, column l%4) of its block.  Here every block
// gets the same four filters as A (lane l holds filter l%4), so one instruction
// updates 4 filters x 64 pixels for one (c, kh, kw) of the convolution stage of
// Algorithm 1 (arXiv 2006.09791).  The group's whole filter bank
// (KPG x CPG x 9 values) lives in registers for the lifetime of a wave (it gets
// there through LDS: one coalesced copy per block, then wide LDS reads); the
// pixel operand comes from a zero-haloed LDS tile of the group's input slab.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

struct Tile4 {
    int NB, TH, IHt;          // images, output rows per block; staged input rows
    int LW, IMG, PLANE, XO;   // LDS row pitch, floats per image / channel, column of input col 0
    int row_blocks, img_blocks;
    int tpr_log2, vec, tasks, xslots;
    int in_floats;
    unsigned m_IHt, m_NB, m_ppi, m_Wout, m_rowb;
    unsigned x_bytes, w_bytes, y_bytes;
};
static_assert(sizeof(Tile4) <= sizeof(((Mfma4Plan *)0)->data), "plan storage too small");

constexpr int kTmax4 = 12;   // staged rows per thread

// Block = 4 waves; a wave owns NTILE runs of 64 pixels and all KPG = 4*MT
// filters of the group.  Grid: x = (image block, row block), y = group.
template <int CPG, int MT, int NTILE, int S, typename TIN>
__global__ __launch_bounds__(256) void conv_mfma4r(ConvParams p, Tile4 t) {
    constexpr int NT = 256, TAPS = 9, ES = (int)sizeof(TIN);
    extern __shared__ f32x4 smem4[];
    float *xs = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned ib = fast_div(blockIdx.x, t.m_rowb);
    const int rb = blockIdx.x - ib * t.row_blocks;
    const unsigned j = blockIdx.y;
    const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;

    // ---- filter bank: global -> LDS, transposed to [filter%4][k][mt] ----------
    // One 16-byte unit of the direct section is W[k][4*mt .. 4*mt+3]; behind the
    // barrier below lane l reads its K*MT operands a[k][mt] = W[j*KPG + 4*mt + l%4][k]
    // as one contiguous run.  (One dword load per operand and lane would keep the
    // CU's vector memory path busy for longer than the whole convolution.)
    constexpr int K = CPG * TAPS, WROW = K * MT + 4;   // +4 floats: the four rows start in different banks
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wd, t.w_bytes);
    float *wl = xs + t.in_floats + 4;
    {
        const unsigned wbase = j * K * p.KPGd * 4;
        for (int u = tid; u < K * MT; u += NT) {
            const int k = u / MT, mt = u - k * MT;
            const f32x4 v = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, (k * p.KPGd + mt * 4) * 4, wbase, 0));
#pragma unroll
            for (int f = 0; f < 4; ++f) wl[f * WROW + k * MT + mt] = v[f];
        }
    }

    // ---- stage the group's input slab with a zero halo -----------------------
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    {
        const int rpp = NT >> t.tpr_log2;
        const int row0 = tid >> t.tpr_log2, colv = tid & ((1 << t.tpr_log2) - 1);
        const int vw = t.vec ? 4 : 1;
        f32x4 pin[kTmax4];
        unsigned xlds[kTmax4];
#pragma unroll
        for (int k = 0; k < kTmax4; ++k) {
            if (k < t.xslots) {
                const int task = row0 + k * rpp;
                unsigned xoff = kOob;
                xlds[k] = t.in_floats * 4;   // spare slot behind the tile
                if (task < t.tasks && colv * vw < p.W) {
                    const int cimg = fast_div(task, t.m_IHt), r = task - cimg * t.IHt;
                    const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
                    const int ih = ih0 + r, n = n0 + img;
                    xlds[k] = (c * t.PLANE + img * t.IMG + r * t.LW + t.XO + colv * vw) * 4;
                    if (n < p.N && ih >= 0 && ih < p.H)
                        xoff = (((n * p.Cin + j * CPG + c) * p.H + ih) * p.W + colv * vw) * ES;
                }
                pin[k] = buf_load_in<TIN>(rx, xoff, 0, t.vec);
            }
        }
        // halo columns left and right of every staged row
        const int rows = CPG * t.NB * t.IHt, right = t.XO + p.W;
        for (int i = tid; i < rows; i += NT) {
            const int cimg = fast_div(i, t.m_IHt), r = i - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            float *row = xs + c * t.PLANE + img * t.IMG + r * t.LW;
            for (int x = 0; x < t.XO; ++x) row[x] = 0.f;
            for (int x = right; x < t.LW; ++x) row[x] = 0.f;
        }
        char *bb = reinterpret_cast<char *>(xs);
#pragma unroll
        for (int k = 0; k < kTmax4; ++k) {
            if (k < t.xslots) {
                if (t.vec) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pin[k];
                else *reinterpret_cast<float *>(bb + xlds[k]) = pin[k].x;
            }
        }
    }

    // ---- per-lane pixels -------------------------------------------------------
    int base[NTILE];
    unsigned ooff[NTILE];
    const unsigned HWo = p.Hout * p.Wout;
#pragma unroll
    for (int nt = 0; nt < NTILE; ++nt) {
        const int q = (wave * NTILE + nt) * 64 + lane;
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_Wout), col = rem - r * p.Wout;
        base[nt] = img * t.IMG + r * S * t.LW + (t.XO - p.pad) + col * S;
        const int n = n0 + img, oh = oh0 + r;
        ooff[nt] = (q < tot && n < p.N && oh < p.Hout)
                       ? (((unsigned)n * p.Cout + j * (4 * MT)) * HWo + oh * p.Wout + col) * 4
                       : kOob;
    }
    f32x4 acc[NTILE][MT];
#pragma unroll
    for (int nt = 0; nt < NTILE; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();

    float a[K][MT];
    {
        const float *wr = wl + (lane & 3) * WROW;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[k][mt] = wr[k * MT + mt];
    }

#pragma unroll
    for (int c = 0; c < CPG; ++c) {
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const float *xr = xs + c * t.PLANE + kh * t.LW;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                float b[NTILE];
#pragma unroll
                for (int nt = 0; nt < NTILE; ++nt) b[nt] = xr[base[nt] + kw];
#pragma unroll
                for (int nt = 0; nt < NTILE; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_4x4x1f32(a[(c * 3 + kh) * 3 + kw][mt], b[nt],
                                                                        acc[nt][mt], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: register r of (nt, mt) is filter 4*mt + r at this lane's pixel
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    if (p.res) {
        // all residual loads in flight before the first one is consumed
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
        float rv[NTILE][MT][4];
#pragma unroll
        for (int nt = 0; nt < NTILE; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    rv[nt][mt][r] =
                        __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, ooff[nt], (mt * 4 + r) * HWo * 4, 0));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int nt = 0; nt < NTILE; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[nt][mt][r] += rv[nt][mt][r];
    }
#pragma unroll
    for (int nt = 0; nt < NTILE; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[nt][mt][r];
                if (p.relu) v = fmaxf(v, 0.f);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), ry, ooff[nt], (mt * 4 + r) * HWo * 4, 0);
            }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

constexpr int kLdsBudget4 = 64 * 1024;

struct Inst4 {
    int CPG, MT, NTILE, S;
    const char *name;
};

// Bank conflicts (32 banks) of one 32-lane group reading consecutive pixels.
int bank_cost4(const ConvParams &p, const Tile4 &t, int lw) {
    int cnt[32] = {0}, worst = 0;
    const int ppi = t.TH * p.Wout;
    for (int l = 0; l < 32; ++l) {
        const int q = l < t.NB * ppi ? l : 0;
        const int img = q / ppi, rem = q % ppi, r = rem / p.Wout, col = rem % p.Wout;
        ++cnt[(img * t.IHt * lw + r * p.stride * lw + col * p.stride) & 31];
    }
    for (int b = 0; b < 32; ++b) worst = cnt[b] > worst ? cnt[b] : worst;
    return worst;
}

bool plan4_tile(const ConvParams &p, const PackGeom &g, int NTILE, Tile4 *out) {
    const int PB = 256 * NTILE, NT = 256;
    Tile4 t{};
    if (!split_pixels(p, PB, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * p.stride + 3;
    t.vec = p.W % 4 == 0;
    int lw0;
    if (t.vec) {
        t.XO = 4 * ((p.pad + 3) / 4);
        lw0 = round_up(t.XO + p.W + p.pad, 4);
    } else {
        t.XO = p.pad;
        lw0 = p.W + 2 * p.pad;
    }
    // Row pitch: smallest conflict count within the LDS budget.
    int best_lw = 0, best_cost = 1 << 30;
    for (int lw = lw0; lw < lw0 + 32; lw += t.vec ? 4 : 1) {
        const size_t bytes = ((size_t)round_up(g.CPG * t.NB * t.IHt * lw, 4) + 4 + 4 * (g.Kred * (g.KPG / 4) + 4)) * sizeof(float);
        if (bytes > (size_t)kLdsBudget4) break;
        const int cost = bank_cost4(p, t, lw);
        if (cost < best_cost) {
            best_cost = cost;
            best_lw = lw;
        }
    }
    if (!best_lw) return false;
    t.LW = best_lw;
    t.IMG = t.IHt * t.LW;
    t.PLANE = round_up(t.NB * t.IMG, 4);
    t.in_floats = g.CPG * t.PLANE;
    const int cols = t.vec ? p.W / 4 : p.W;
    while ((1 << t.tpr_log2) < cols) ++t.tpr_log2;
    if ((1 << t.tpr_log2) > NT) return false;
    const int rpp = NT >> t.tpr_log2;
    t.tasks = g.CPG * t.NB * t.IHt;
    t.xslots = (t.tasks + rpp - 1) / rpp;
    if (t.xslots > kTmax4) return false;
    t.row_blocks = (p.Hout + t.TH - 1) / t.TH;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.Wout);
    t.m_Wout = div_magic(p.Wout);
    t.m_rowb = div_magic(t.row_blocks);
    const double xb = (double)p.N * p.Cin * p.H * p.W * (p.in_bf16 ? 2 : 4);
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    const double wb = (double)p.groups * g.Kred * g.KPGd * 4;
    if (xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    if ((double)t.row_blocks * t.img_blocks * t.row_blocks >= 4.0e9 || t.tasks >= 65536 ||
        t.TH * p.Wout >= 65536 || p.groups > 65535)
        return false;
    *out = t;
    return true;
}

template <int CPG, int MT, int NTILE, int S, typename TIN>
hipError_t launch4_inst(const ConvParams &p, const Tile4 &t, hipStream_t s) {
    const size_t lds = ((size_t)t.in_floats + 4 + 4 * (CPG * 9 * MT + 4)) * sizeof(float);   // tile, spare slot, filter bank
    dim3 grid(t.row_blocks * t.img_blocks, p.groups);
    hipLaunchKernelGGL((conv_mfma4r<CPG, MT, NTILE, S, TIN>), grid, dim3(256), lds, s, p, t);
    return hipGetLastError();
}

template <int CPG, int MT, typename TIN>
hipError_t launch4_nt(int NTILE, int S, const ConvParams &p, const Tile4 &t, hipStream_t s) {
    if (S == 1) {
        if (NTILE == 1) return launch4_inst<CPG, MT, 1, 1, TIN>(p, t, s);
        if (NTILE == 2) return launch4_inst<CPG, MT, 2, 1, TIN>(p, t, s);
        if (NTILE == 4) return launch4_inst<CPG, MT, 4, 1, TIN>(p, t, s);
    } else {
        if (NTILE == 1) return launch4_inst<CPG, MT, 1, 2, TIN>(p, t, s);
        if (NTILE == 2) return launch4_inst<CPG, MT, 2, 2, TIN>(p, t, s);
        if (NTILE == 4) return launch4_inst<CPG, MT, 4, 2, TIN>(p, t, s);
    }
    return hipErrorNotSupported;
}

template <typename TIN>
hipError_t launch4_any(int CPG, int MT, int NTILE, int S, const ConvParams &p, const Tile4 &t, hipStream_t s) {
#define GSPC_I4(C, M) \
    if (CPG == C && MT == M) return launch4_nt<C, M, TIN>(NTILE, S, p, t, s);
    GSPC_I4(1, 1) GSPC_I4(2, 1) GSPC_I4(4, 1) GSPC_I4(8, 1)
    GSPC_I4(1, 2) GSPC_I4(2, 2) GSPC_I4(4, 2) GSPC_I4(8, 2)
    GSPC_I4(2, 3) GSPC_I4(4, 3)
#undef GSPC_I4
    return hipErrorNotSupported;
}

bool inst_exists(int CPG, int MT) {
    if (MT == 1 || MT == 2) return CPG == 1 || CPG == 2 || CPG == 4 || CPG == 8;
    if (MT == 3) return CPG == 2 || CPG == 4;
    return false;
}

}  // namespace

bool plan_mfma4(const ConvParams &p, const PackGeom &g, Mfma4Plan *out) {
    if (g.variant != kMfma4 || p.KH != 3 || p.KW != 3 || (p.stride != 1 && p.stride != 2)) return false;
    const int MT = g.KPG / 4;
    if (!inst_exists(g.CPG, MT)) return false;
    static const char *force = std::getenv("GSPC_TILE4");
    // Most pixel runs per wave (more independent accumulators, fewer filter-bank
    // loads, less halo re-staging) while a block still works on a single image:
    // images share nothing, so packing several into a block only costs blocks.
    int chosen = 0;
    Tile4 best{};
    int forced = force ? std::atoi(force) : tuned_config(p, 'q');
    {
        Tile4 t;
        if (!force && forced >= 0 && ((forced != 1 && forced != 2 && forced != 4) || !plan4_tile(p, g, forced, &t))) forced = -1;
    }
    for (int nt : {4, 2, 1}) {
        Tile4 t;
        if (forced >= 0 && forced != nt) continue;
        if (!plan4_tile(p, g, nt, &t)) continue;
        const long blocks = (long)t.row_blocks * t.img_blocks * p.groups;
        chosen = nt;
        best = t;
        // heavy filter banks (8 channels x 8 filters per group: 144 MFMAs per pixel run) want
        // the launch spread over more, shorter blocks (autotuner: 10.6 -> 8.9 us at N = 64)
        const long enough = g.Kred * MT >= 144 ? 4L * kNumCU : kNumCU / 2;
        // several images per block only when the launch is plentiful anyway (large batches); with the
        // heavy banks four pixel runs per filter-bank read pay from two blocks per compute unit on
        // (64 -> 64 on 16x16 in 8 groups at N = 256: 21.0 -> 15.1 us)
        if ((t.NB == 1 && blocks >= enough) || blocks >= 4L * kNumCU ||
            (nt == 4 && g.Kred * MT >= 144 && blocks >= 2L * kNumCU))
            break;
    }
    // Stride 2: the staged tile is four times the outputs it feeds, so one pixel run per wave keeps
    // more blocks resident (8-13 % at N = 64 and 256 on the 56x56 and 32x32 planes).
    if (forced < 0 && chosen > 1 && p.stride == 2) {
        Tile4 t;
        if (plan4_tile(p, g, 1, &t)) {
            chosen = 1;
            best = t;
        }
    }
    if (!chosen) return false;
    // Half the pixel runs per wave when that cuts the plane into tiles with clearly fewer idle lanes
    // (a 56x56 plane is 4 tiles of 1024 pixels at 77 % or 7 of 512 at 88 %; the offline tuner's pick, 5-10 %).
    // Heavy filter banks only: with lighter ones the saving did not repeat at batch 256.
    if (forced < 0 && chosen > 1 && g.Kred * MT >= 144) {
        Tile4 t;
        if (plan4_tile(p, g, chosen / 2, &t)) {
            const double px = (double)p.N * p.Hout * p.Wout;
            const double eff0 = px / ((double)best.row_blocks * best.img_blocks * 256 * chosen);
            const double eff1 = px / ((double)t.row_blocks * t.img_blocks * 128 * chosen);
            if (t.NB == 1 && best.NB == 1 && eff1 >= eff0 + 0.08) {
                chosen /= 2;
                best = t;
            }
        }
    }
    out->inst = chosen;
    std::memcpy(out->data, &best, sizeof(best));
    return true;
}

hipError_t launch_mfma4(const ConvParams &p, const Mfma4Plan &plan, hipStream_t s, const char **name) {
    Tile4 t;
    std::memcpy(&t, plan.data, sizeof(t));
    *name = intern_name("conv_mfma4r<" + std::to_string(p.CPG) + "," + std::to_string(p.KPG / 4) + "," +
                        std::to_string(plan.inst) + "," + std::to_string(p.stride) +
                        (p.in_bf16 ? ",bf16>" : ",f32>"));
    const int MT = p.KPG / 4;
    return p.in_bf16 ? launch4_any<uint16_t>(p.CPG, MT, plan.inst, p.stride, p, t, s)
                     : launch4_any<float>(p.CPG, MT, plan.inst, p.stride, p, t, s);
}

}  // namespace gspc
