// Depth fusion of consecutive grouped 3x3 convolutions of a layer chain.
//
// A grouped convolution only mixes the channels of one group (Section II and
// Fig. 2 of arXiv 2006.09791; Section III-A: there is no data dependency
// between groups, which is what Algorithm 1 parallelises over).  When consecutive layers have the same shape and the same g, stride 1
// and Cin = Cout, group j of every one of them depends on group j of the
// chain's input alone: the whole run can be evaluated per (image, group) with
// the activations never leaving the CU.  One block owns one (image, group): its
// CPG x H x W slabs live in LDS tiles with a zero halo, a layer reads one tile
// (and a residual tile), writes another, and only the values a buffer still
// holds when the run ends are written to HBM.  Weights of the next layer are
// fetched while the current one is computed.
#include <cstdlib>
#include <cstring>
#include <vector>

#include "conv_common.h"

namespace gspc {

constexpr int kFuseMaxUnits = 32 * 9 * 32 / 4;   // 16-byte units of the largest layer's weights (CPG = 32)

// ---------------------------------------------------------------------------
// One block per (image, group).  A layer is a [KPG x CPG*9] by [CPG*9 x H*W]
// product on v_mfma_f32_16x16x4_f32: filters on the M edge (zero rows past
// KPG), runs of 16 output pixels on the N edge, 4 channels at one tap per
// k-step (zero past CPG).  Both operands come from LDS: the layer's weights in
// their [c][tap][KPGd] order (lane l reads filter l%16 of channel 4*cb + l/16),
// the activations from the source tile.  A wave owns NI pixel runs of one
// 16-filter tile at a time.  NW waves per block: with one block per CU (large tiles)
// sixteen, so that LDS latency and the epilogues of some waves hide behind the
// MFMAs of others; eight when several blocks share a CU.
// ---------------------------------------------------------------------------
#ifdef GSPC_PHASE_TIMING
__device__ unsigned long long g_phase_f[16 * 8];
#define GSPC_STAMPF(l, i)                                                                  \
    if (threadIdx.x == 0 && blockIdx.x == 0 && (l) < 16) g_phase_f[(l) * 8 + (i)] = __builtin_amdgcn_s_memrealtime();
extern "C" int gspc_debug_phases_f(unsigned long long *out, int n) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_f), sizeof(unsigned long long) * n);
}
#else
#define GSPC_STAMPF(l, i)
#endif

template <int NI, int NW>
__global__ __launch_bounds__(64 * NW) void conv_fused_run(FusedRun r) {
    constexpr int kFuseThreads = 64 * NW, kFuseWaves = NW;
    constexpr int kFuseMaxW = (kFuseMaxUnits + kFuseThreads - 1) / kFuseThreads;
    extern __shared__ f32x4 smem4[];
    float *smem = reinterpret_cast<float *>(smem4);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned n = fast_div(blockIdx.x, r.m_groups);
    const int j = blockIdx.x - n * r.groups;
    const int HW = r.H * r.W;
    const size_t slab = ((size_t)n * r.C + (size_t)j * r.CPG) * HW;   // first element of this block's channels

    float *tiles = smem;
    float *wbuf = smem + r.ntiles * r.TILE;

    // ---- clear the tiles (halos stay zero for the whole run) ----------------
    {
        const int n4 = r.ntiles * r.TILE / 4;
        for (int i = tid; i < n4; i += kFuseThreads) smem4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // ---- weights of the first layer ----------------------------------------
    const int wunits = r.wfloats / 4;
    f32x4 pw[kFuseMaxW];
    auto fetch_w = [&](int l) __attribute__((always_inline)) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(r.L[l].w + (size_t)j * r.wfloats);
#pragma unroll
        for (int k = 0; k < kFuseMaxW; ++k) {
            const int u = k * kFuseThreads + tid;
            if (u < wunits) pw[k] = src[u];
        }
    };
    auto commit_w = [&](int buf) __attribute__((always_inline)) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(wbuf + buf * r.wfloats);
#pragma unroll
        for (int k = 0; k < kFuseMaxW; ++k) {
            const int u = k * kFuseThreads + tid;
            if (u < wunits) dst[u] = pw[k];
        }
    };
    fetch_w(0);
    __syncthreads();   // tiles cleared before the inputs land
    // ---- run inputs: global -> tile interiors --------------------------------
    for (int i = 0; i < r.ninputs; ++i) {
        const float *src = r.in_ptr[i] + slab;
        float *tile = tiles + r.in_tile[i] * r.TILE;
        if (r.vec) {
            const int wq = r.W / 4, total = r.CPG * r.H * wq;
            for (int e = tid; e < total; e += kFuseThreads) {
                const int c = fast_div(e, r.m_hwq), rem = e - c * (r.H * wq);
                const int h = fast_div(rem, r.m_wq), q = rem - h * wq;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(src + (size_t)c * HW + h * r.W + q * 4);
                *reinterpret_cast<f32x4 *>(tile + c * r.PLANE + (h + 1) * r.LW + r.XO + q * 4) = v;
            }
        } else {
            const int total = r.CPG * HW;
            for (int e = tid; e < total; e += kFuseThreads) {
                const int c = fast_div(e, r.m_hw), rem = e - c * HW;
                const int h = fast_div(rem, r.m_w), x = rem - h * r.W;
                tile[c * r.PLANE + (h + 1) * r.LW + r.XO + x] = src[e];
            }
        }
    }
    commit_w(0);
    __syncthreads();

    const int lrow = lane & 15, lk = lane >> 4;   // MFMA operand coordinates of this lane
    const int cblocks = (r.CPG + 3) >> 2;
    for (int l = 0; l < r.nlayers; ++l) {
        GSPC_STAMPF(l, 0)
        // the layer's descriptor, read once (scalar loads share a wait counter with LDS)
        const int l_src = r.L[l].src, l_res = r.L[l].res, l_dst = r.L[l].dst, l_relu = r.L[l].relu;
        float *const l_y = r.L[l].y;
        if (l + 1 < r.nlayers) fetch_w(l + 1);
        const float *wl = wbuf + (l & 1) * r.wfloats;
        const float *src = tiles + l_src * r.TILE;
        for (int item = wave; item < r.nitems; item += kFuseWaves) {
            const int mt = fast_div(item, r.m_rgroups), rg = item - mt * r.rgroups;
            // B operand: pixel (rg*NI + ni)*16 + lrow of channel 4*cb + lk
            int base[NI], prow[NI], pcol[NI];
            bool pvalid[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int p = (rg * NI + ni) * 16 + lrow;
                pvalid[ni] = p < HW;
                const int pp = pvalid[ni] ? p : 0;
                prow[ni] = fast_div(pp, r.m_w);
                pcol[ni] = pp - prow[ni] * r.W;
                base[ni] = prow[ni] * r.LW + (r.XO - 1) + pcol[ni];
            }
            // A operand: filter mt*16 + lrow, channel 4*cb + lk; zero outside the group's extent
            const int f = mt * 16 + lrow;
            const bool fvalid = f < r.CPG;
            f32x4 acc[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) acc[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int cb = 0; cb < cblocks; ++cb) {
                const int c = cb * 4 + lk;
                const bool avalid = fvalid && c < r.CPG;
                const int cc = c < r.CPG ? c : r.CPG - 1;
                const float *wp = wl + cc * 9 * r.KPGd + (fvalid ? f : 0);
                const float *xp = src + cc * r.PLANE;
#pragma unroll
                for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        const float wv = wp[(kh * 3 + kw) * r.KPGd];
                        const float a = avalid ? wv : 0.f;
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const float b = xp[base[ni] + kh * r.LW + kw];
                            acc[ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[ni], 0, 0, 0);
                        }
                    }
            }
            GSPC_STAMPF(l, 1 + 2 * ((item - wave) / kFuseWaves > 0))
            // ---- epilogue: register q of acc[ni] is filter mt*16 + 4*lk + q at pixel (rg*NI + ni)*16 + lrow.
            // Addresses first, then all residual reads, then all writes: no wait between the accesses.
            int eoff[NI][4];    // float offset inside a tile
            bool eok[NI][4];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int oc = mt * 16 + 4 * lk + q;
                    eok[ni][q] = pvalid[ni] && oc < r.CPG;
                    eoff[ni][q] = (eok[ni][q] ? oc : 0) * r.PLANE + (prow[ni] + 1) * r.LW + r.XO + pcol[ni];
                }
            float v[NI][4];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) v[ni][q] = acc[ni][q];
            if (l_res >= 0) {
                const float *rt = tiles + l_res * r.TILE;
                float rv[NI][4];
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) rv[ni][q] = rt[eoff[ni][q]];
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[ni][q] += rv[ni][q];
            }
            if (l_relu) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[ni][q] = fmaxf(v[ni][q], 0.f);
            }
            if (l_dst >= 0) {
                float *dt = tiles + l_dst * r.TILE;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (eok[ni][q]) dt[eoff[ni][q]] = v[ni][q];
            }
            if (l_y) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (eok[ni][q])
                            l_y[slab + (size_t)(mt * 16 + 4 * lk + q) * HW + prow[ni] * r.W + pcol[ni]] = v[ni][q];
            }
            GSPC_STAMPF(l, 2 + 2 * ((item - wave) / kFuseWaves > 0))
        }
        GSPC_STAMPF(l, 5)
        if (l + 1 < r.nlayers) commit_w((l + 1) & 1);
        GSPC_STAMPF(l, 6)
        __syncthreads();
        GSPC_STAMPF(l, 7)
    }
}

// ---------------------------------------------------------------------------
// Host side: run detection, tile allocation, launch.
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kFuseLds = 150 * 1024;

template <int NI, int NW>
hipError_t launch_core(const FusedRun &r, size_t lds, hipStream_t s) {
    auto kern = conv_fused_run<NI, NW>;
    if (lds > 64 * 1024) {
        static thread_local bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3(r.N * r.groups), dim3(64 * NW), lds, s, r);
    return hipGetLastError();
}

// The layer as the fused kernel multiplies it: its widest merged direct section if it has one
// (block-diagonal groups of up to 8 channels fill more of each matrix-core instruction), else its own
// direct section.
struct FuseView {
    int groups, CPG, KPGd;
    const float *w;
};
FuseView fuse_view(const gspc_layer_t &L) {
    const PackGeom &g = L.w->geom;
    for (int which = 1; which >= 0; --which)
        if (g.md[which].m && g.md[which].groups >= 2)
            return FuseView{g.md[which].groups, g.md[which].CPG, g.md[which].KPGd,
                            reinterpret_cast<const float *>(static_cast<const char *>(L.w->dev) + g.md[which].offset)};
    return FuseView{L.groups, L.Cin / L.groups, g.KPGd, reinterpret_cast<const float *>(L.w->dev)};
}

bool fusable_layer(const gspc_layer_t &L) {
    if (L.op != GSPC_OP_CONV || !L.w) return false;
    if (L.KH != 3 || L.KW != 3 || L.stride != 1 || L.pad != 1 || L.Cin != L.Cout) return false;
    if (L.w->dtype != GSPC_F32) return false;
    const int CPG = L.Cin / L.groups;
    if (L.groups < 2 || CPG > 32) return false;
    return true;
}

}  // namespace

// Tries to turn layers [first, first + count) into one fused run.  Returns the
// number of leading layers it covers (0 = not worth fusing / does not fit).
int plan_fused_run(const gspc_layer_t *layers, int first, int count, void *const *bufs, FusedPlan *out) {
    static const bool off = std::getenv("GSPC_NO_FUSE") != nullptr;   // tuning aid
    if (off || count < 2 || !fusable_layer(layers[first])) return 0;
    const gspc_layer_t &A = layers[first];
    int n = 1;
    while (n < count && n < kFuseMaxLayers) {
        const gspc_layer_t &B = layers[first + n];
        if (!fusable_layer(B) || B.N != A.N || B.Cin != A.Cin || B.H != A.H || B.W != A.W || B.groups != A.groups)
            break;
        ++n;
    }
    if (n < 2) return 0;

    FusedRun r{};
    r.N = A.N;
    r.C = A.Cin;
    r.H = A.H;
    r.W = A.W;
    const FuseView av = fuse_view(A);
    r.groups = av.groups;
    r.CPG = av.CPG;
    r.KPGd = av.KPGd;
    r.vec = A.W % 4 == 0;
    r.XO = 4;
    r.LW = round_up(r.XO + r.W + 1, 4);
    r.PLANE = (r.H + 2) * r.LW;
    r.TILE = r.CPG * r.PLANE;
    r.wfloats = r.CPG * 9 * r.KPGd;
    if (r.wfloats % 4 || r.wfloats / 4 > kFuseMaxUnits) return 0;
    if ((double)r.N * r.C * r.H * r.W >= 2147483648.0) return 0;
    if ((double)r.N * r.groups * r.groups >= 4.0e9) return 0;

    // Value numbering and tile allocation, shrinking the run until it fits.
    for (; n >= 2; --n) {
        struct Val {
            int buf, producer, last_read, tile;   // producer -1: value from before the run
        };
        std::vector<Val> vals;
        auto find_val = [&](int buf) -> int {   // current value of a buffer
            for (int v = (int)vals.size() - 1; v >= 0; --v)
                if (vals[v].buf == buf) return v;
            vals.push_back({buf, -1, -1, -1});
            return (int)vals.size() - 1;
        };
        std::vector<int> src_v(n), res_v(n), dst_v(n);
        for (int l = 0; l < n; ++l) {
            const gspc_layer_t &L = layers[first + l];
            src_v[l] = find_val(L.src);
            vals[src_v[l]].last_read = l;
            res_v[l] = -1;
            if (L.src2 >= 0) {
                res_v[l] = find_val(L.src2);
                vals[res_v[l]].last_read = l;
            }
            vals.push_back({L.dst, l, -1, -1});
            dst_v[l] = (int)vals.size() - 1;
        }
        // A tile holds a value up to and including the layer tile_free_at[t].
        int ninputs = 0;
        bool ok = true;
        std::vector<int> tile_free_at(kFuseMaxTiles, -1);
        std::vector<bool> tile_used(kFuseMaxTiles, false);
        // run inputs occupy their tiles from the start
        for (size_t v = 0; v < vals.size() && ok; ++v) {
            if (vals[v].producer >= 0) continue;
            int t = -1;
            for (int c = 0; c < kFuseMaxTiles && t < 0; ++c)
                if (!tile_used[c]) t = c;
            if (t < 0 || ninputs == kFuseMaxInputs) {
                ok = false;
                break;
            }
            vals[v].tile = t;
            tile_used[t] = true;
            tile_free_at[t] = vals[v].last_read;
            r.in_ptr[ninputs] = static_cast<const float *>(bufs[vals[v].buf]);
            r.in_tile[ninputs] = t;
            ++ninputs;
        }
        for (int l = 0; l < n && ok; ++l) {
            const gspc_layer_t &L = layers[first + l];
            FusedLayer &F = r.L[l];
            F.w = fuse_view(L).w;
            F.src = (short)vals[src_v[l]].tile;
            F.res = (short)(res_v[l] >= 0 ? vals[res_v[l]].tile : -1);
            F.relu = (L.flags & GSPC_FLAG_RELU) ? 1 : 0;
            Val &d = vals[dst_v[l]];
            // the value still sits in its buffer when the run ends -> HBM
            bool final_value = true;
            for (int m = l + 1; m < n; ++m)
                if (layers[first + m].dst == L.dst) final_value = false;
            F.y = final_value ? static_cast<float *>(bufs[L.dst]) : nullptr;
            F.dst = -1;
            if (d.last_read >= 0) {
                // a tile that is free during layer l: its last reader is an earlier layer, or it is the
                // residual's tile and this layer is the residual's last reader (element-wise reuse)
                int t = -1;
                for (int c = 0; c < kFuseMaxTiles && t < 0; ++c) {
                    if (c == F.src) continue;
                    const bool free_now = !tile_used[c] || tile_free_at[c] < l ||
                                          (c == F.res && tile_free_at[c] == l);
                    if (free_now) t = c;
                }
                if (t < 0) {
                    ok = false;
                    break;
                }
                d.tile = t;
                tile_used[t] = true;
                tile_free_at[t] = d.last_read;
                F.dst = (short)t;
            }
        }
        int ntiles = 0;
        for (int t = 0; t < kFuseMaxTiles; ++t)
            if (tile_used[t]) ntiles = t + 1;
        const size_t lds = ((size_t)ntiles * r.TILE + 2 * (size_t)r.wfloats) * sizeof(float);
        if (ok && lds <= kFuseLds) {
            r.nlayers = n;
            r.ninputs = ninputs;
            r.ntiles = ntiles;
            break;
        }
    }
    if (n < 2) return 0;
    const size_t lds = ((size_t)r.ntiles * r.TILE + 2 * (size_t)r.wfloats) * sizeof(float);

    // Worth it?  Both sides are fits to measurements on this GPU (stage by stage, N = 1 and 64).  A
    // fused layer costs a round of co-resident blocks about 2 us (barrier, epilogues, pipeline fill)
    // plus 5.7 ns per MFMA of the blocks that share a CU (32 cycles each over four SIMDs, x 1.4); a
    // separate launch costs about 4.2 us of launch and pipeline latency plus the layer at the speed of
    // the kernel that would take it.
    {
        long per_cu = (long)(160 * 1024 / lds);
        per_cu = per_cu < 1 ? 1 : per_cu > 8 ? 8 : per_cu;
        const long blocks = (long)r.N * r.groups;
        const long rounds = (blocks + kNumCU * per_cu - 1) / (kNumCU * per_cu);
        long share = (blocks + kNumCU - 1) / kNumCU;   // blocks that share a CU at a time
        share = share > per_cu ? per_cu : share;
        const double mfmas = (double)((r.CPG + 15) / 16) * ((r.H * r.W + 15) / 16) * ((r.CPG + 3) / 4) * 9.0;
        const double fused_us = (2.0 + 0.0057 * share * mfmas) * rounds;
        const double macs = (double)r.CPG * r.CPG * 9.0 * r.H * r.W * blocks;
        const double macs_per_us = r.W % 4 ? 20.0e6 : r.CPG >= 16 ? 45.0e6 : 25.0e6;
        const double unfused_us = (r.CPG <= 2 ? 6.0 : 4.2) + macs / macs_per_us;   // CPG <= 2 runs on the plain-ALU kernel
        if (fused_us >= unfused_us) return 0;
    }

    // 16-byte global accesses need 16-byte aligned tensors (weights are 256-byte aligned by contract).
    {
        auto misaligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) != 0; };
        for (int i = 0; i < r.ninputs; ++i)
            if (misaligned(r.in_ptr[i])) r.vec = 0;
        for (int l = 0; l < r.nlayers; ++l)
            if (misaligned(r.L[l].w)) return 0;
    }

    // Pixel runs per wave item: as many as still give every wave an item.
    const int runs = (r.H * r.W + 15) / 16, mtiles = (r.CPG + 15) / 16;
    // one block per CU (by LDS size, or because there are no more blocks than CUs): sixteen waves
    const int nw = (160 * 1024 / lds >= 2 && (long)r.N * r.groups > kNumCU) ? 8 : 16;
    int ni = 4;
    while (ni > 1 && (long)mtiles * ((runs + ni - 1) / ni) < nw) ni >>= 1;
    r.rgroups = (runs + ni - 1) / ni;
    r.nitems = mtiles * r.rgroups;
    r.m_groups = div_magic(r.groups);
    r.m_rgroups = div_magic(r.rgroups);
    r.m_hw = div_magic(r.H * r.W);
    r.m_w = div_magic(r.W);
    r.m_hwq = div_magic(r.H * (r.W / 4 > 0 ? r.W / 4 : 1));
    r.m_wq = div_magic(r.W / 4 > 0 ? r.W / 4 : 1);
    out->core = ni;
    out->waves = nw;
    out->lds = lds;
    out->run = r;
    return n;
}

hipError_t launch_fused_run(const FusedPlan &pl, hipStream_t s, const char **name) {
    *name = intern_name("conv_fused_run<" + std::to_string(pl.core) + "," + std::to_string(pl.waves) + ">x" +
                        std::to_string(pl.run.nlayers));
    if (pl.waves == 16) {
        switch (pl.core) {
        case 4: return launch_core<4, 16>(pl.run, pl.lds, s);
        case 2: return launch_core<2, 16>(pl.run, pl.lds, s);
        case 1: return launch_core<1, 16>(pl.run, pl.lds, s);
        }
    } else {
        switch (pl.core) {
        case 4: return launch_core<4, 8>(pl.run, pl.lds, s);
        case 2: return launch_core<2, 8>(pl.run, pl.lds, s);
        case 1: return launch_core<1, 8>(pl.run, pl.lds, s);
        }
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
