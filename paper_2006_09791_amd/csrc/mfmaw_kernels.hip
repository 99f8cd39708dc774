// Per-group implicit-GEMM grouped convolution, 3x3, with the group's filter
// tile resident in LDS and wave-private input tiles.
//
// Same contraction as conv_mfma16 (the convolution stage of Algorithm 1,
// arXiv 2006.09791, with the paper's input and output reshapes fused in), but
// organised for layers whose whole job is a few microseconds of matrix-core
// work: one wave per SIMD, every wave owns 16*MI filters x 16*NI output pixels
// for the whole reduction, and after the weights have landed no wave ever
// waits for another one.
//
//   * The block's 16*MI filters (all CPG channels, 9 taps) are copied once
//     from the packed matrix-core section into LDS, in MFMA A-operand order.
//     The k-steps of the first chunk are committed first so that the first
//     MFMA does not wait for the rest; the rest follows behind one more
//     barrier after the first chunk has been multiplied.
//   * Each wave stages the input rows of its own pixel tile in a private
//     two-stage LDS ring (zero halo columns, rows outside the image arrive as
//     zeros from the buffer loads), two chunks ahead through registers.
//     LDS operations of one wave execute in order, so the ring needs no
//     barrier.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "conv_common.h"

namespace gspc {

constexpr int kTmaxW = 4;    // most input staging slots (16 bytes per lane each) per chunk (stride 1)
constexpr int kTmaxW2 = 8;   // the same for stride 2, whose tiles span twice the input rows at twice the width
constexpr int kWmaxW = 20;   // weight staging slots (16 bytes per thread each) of a 256-thread block, whole reduction

struct Tile16w {
    int NB, TH, IHt;         // images, output rows per wave tile; staged input rows
    int LW, IMG, PLANE, XO;  // LDS row pitch, floats per image / per channel, column of input col 0
    int nchunks;             // chunks of 4*CKB channels
    int row_blocks, img_blocks, oc_blocks, wave_tiles, tile_groups;   // tile_groups = ceil(wave_tiles / 4)
    int tpr_log2;            // lanes per staged row (log2), 16 bytes per lane
    int tasks, xslots;       // staged rows per chunk, rows per lane per chunk
    int xs;                  // staging slots the instance is built for (>= xslots)
    int wslots;              // weight slots in total (the first chunk's count is static)
    int ksteps, mtiles;      // geometry of the packed weight section
    int w_floats, stage_floats;
    unsigned m_IHt, m_NB, m_ppi, m_Wout, m_rowb, m_ocb;
    unsigned x_bytes, w_bytes, y_bytes;
};

#ifdef GSPC_PHASE_TIMING
__device__ unsigned long long g_phase_w[8 * 4096];
#define GSPC_STAMPW(i)                                                                     \
    if (threadIdx.x == 0) {                                                                \
        const unsigned bid = blockIdx.x + blockIdx.y * gridDim.x;                          \
        if (bid < 4096) g_phase_w[bid * 8 + (i)] = __builtin_amdgcn_s_memrealtime();       \
    }
#else
#define GSPC_STAMPW(i)
#endif

// 64 lanes x 16 bytes from global memory straight into LDS: lane l's bytes land at byte offset dst + 16 l of
// the dynamic LDS array (dst wave-uniform).  (A device-only function: the host pass does not know that this
// GPU takes 16 bytes per lane in this instruction, and inside a lambda it would be checked there.)
__device__ __forceinline__ void load_to_lds16(__amdgpu_buffer_rsrc_t r, f32x4 *lds_base, unsigned dst, unsigned voff,
                                              unsigned soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        r, (__attribute__((address_space(3))) void *)(reinterpret_cast<char *>(lds_base) + dst), 16, voff, soff, 0, 0);
}

template <int MI, int NI, int S, int CKB, bool PERSIST, int XS, typename TIN>
__global__ __launch_bounds__(256) void conv_mfma16w(ConvParams p, Tile16w t) {
    GSPC_STAMPW(0)
    constexpr int NT = 256, TAPS = 9, CK = 4 * CKB, KCHUNK = CKB * TAPS, ES = (int)sizeof(TIN);
    constexpr int TMAX = XS, WMAX = kWmaxW;
    extern __shared__ f32x4 smem4[];
    float *smem = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned j = fast_div(blockIdx.y, t.m_ocb);
    const int ob = blockIdx.y - j * t.oc_blocks;
    const int ppi = t.TH * p.Wout, tot = t.NB * ppi;
    const unsigned HW = p.H * p.W, HWo = p.Hout * p.Wout;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wm, t.w_bytes);

    // ---- weights: thread tid copies 16-byte unit k*NT + tid of the block's
    // [k-step][MI][64] array; a slot of NT units covers NT / (16 MI) k-steps.
    constexpr unsigned kStepsPerSlot = NT / (MI * 16);
    const unsigned wrow = t.mtiles * 64 * 4;   // bytes per k-step of the packed section
    const unsigned wblk = ((j * t.ksteps * t.mtiles + ob * MI) * 64) * 4;
    const unsigned wvoff = (tid / (MI * 16)) * wrow + (tid % (MI * 16)) * 16;
    // The weights go straight from global memory into LDS (buffer loads with the LDS modifier: lane l of
    // a wave-level load writes its 16 bytes at the wave's LDS base + 16 l, which is exactly the
    // [unit k*NT + tid] order), all of them requested here, before anything else: no registers, no
    // LDS write instructions, and no memory instruction left in the multiply phase for them.  All
    // blocks fetch their filters at the same moment and the level-2 cache then delivers about 25
    // bytes per clock to each compute unit: that stream (1.4 us for 74 KB per block) is what the
    // time to the barrier is made of, and the index arithmetic below runs while it lasts.  (Letting
    // later chunks' weights arrive behind a second barrier, one load every few k-steps, was measured
    // and is slower: a wave that finds the memory path full waits with its MFMAs.  The same loads for
    // the input tiles, into a ring of three or four stages, were measured too: stride-2 layers gained
    // 8-15 %, stride-1 layers lost 5-7 % - the halo columns then travel as out-of-range lanes, twice
    // the load count on 8-pixel rows.)
    // Slots past the end are skipped (a wave-uniform branch): a load with an out-of-range offset
    // moves no data but still takes its turn in the memory path.
#pragma unroll
    for (int k = 0; k < WMAX; ++k)
        if (k < t.wslots)
            load_to_lds16(rw, smem4, (k * NT + wave * 64) * 16, wvoff, wblk + k * kStepsPerSlot * wrow);

    // ---- private input ring: every wave owns two stages ----------------------
    // (a stage ends with a spare 16-byte slot per lane that absorbs the writes of idle lanes and idle
    // slots: one shared slot would make those writes a 64-way conflict on a single bank)
    float *ring = smem + t.w_floats + wave * (2 * t.stage_floats);
    const unsigned spare = (t.stage_floats - 256) * 4 + lane * 16;   // byte offset of the lane's spare slot in a stage
    const int rpp = 64 >> t.tpr_log2;
    const int row0 = lane >> t.tpr_log2, colv = lane & ((1 << t.tpr_log2) - 1);
    // What depends on the lane alone: where a staged row goes in the ring, its
    // offset from the tile's first input element, and where the lane's pixels sit.
    unsigned xlds[TMAX];
    int xrow[TMAX], ximg[TMAX], xlane[TMAX];   // staged row k of this lane: row and image inside the tile, byte offset
#pragma unroll
    for (int k = 0; k < TMAX; ++k) {
        const int task = row0 + k * rpp;
        xlds[k] = spare;
        xrow[k] = -(1 << 20);   // never in range
        ximg[k] = 0;
        xlane[k] = 0;
        if (k < t.xslots && task < t.tasks && colv * 4 < p.W) {
            const int cimg = fast_div(task, t.m_IHt), r = task - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            xlds[k] = (c * t.PLANE + img * t.IMG + r * t.LW + t.XO + colv * 4) * 4;
            xrow[k] = r;
            ximg[k] = img;
            xlane[k] = (((img * p.Cin + c) * p.H + r) * p.W + colv * 4) * ES;
        }
    }
    int base[NI], pimg[NI], prow[NI], olane[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = ni * 16 + (lane & 15);
        const int qq = q < tot ? q : 0;
        const int img = fast_div(qq, t.m_ppi), rem = qq - img * ppi;
        const int r = fast_div(rem, t.m_Wout), col = rem - r * p.Wout;
        base[ni] = (lane >> 4) * t.PLANE + img * t.IMG + r * S * t.LW + (t.XO - p.pad) + col * S;
        pimg[ni] = img;
        prow[ni] = q < tot ? r : 1 << 20;   // rows of idle lanes are never in range
        olane[ni] = ((img * p.Cout + 4 * (lane >> 4)) * HWo + r * p.Wout + col) * 4;
    }
    // What depends on the pixel tile: global offsets of the staged rows and of
    // the outputs (kOob = no access).  A wave past the last tile loads zeros and
    // stores nothing.
    unsigned xoff[TMAX], ooff[NI];
    auto set_tile = [&](int tile_group) __attribute__((always_inline)) {
        const int wt = tile_group * 4 + wave;
        const bool live = wt < t.wave_tiles;
        const unsigned ib = fast_div(live ? wt : 0, t.m_rowb);
        const int rb = (live ? wt : 0) - ib * t.row_blocks;
        const int n0 = ib * t.NB, oh0 = rb * t.TH, ih0 = oh0 * S - p.pad;
        const int nleft = live ? p.N - n0 : 0;   // images of this tile that exist
        const int xtile = (((n0 * p.Cin + j * p.CPG) * p.H + ih0) * p.W) * ES;
        const int otile = ((n0 * p.Cout + j * p.KPG) * HWo + oh0 * p.Wout) * 4;
#pragma unroll
        for (int k = 0; k < TMAX; ++k)
            xoff[k] = (ximg[k] < nleft && xrow[k] >= -ih0 && xrow[k] < p.H - ih0) ? (unsigned)(xtile + xlane[k]) : kOob;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            ooff[ni] = (pimg[ni] < nleft && prow[ni] < p.Hout - oh0) ? (unsigned)(otile + olane[ni]) : kOob;
    };
    set_tile(blockIdx.x);
    f32x4 pin0[TMAX], pin1[TMAX];
    auto fetch_x = [&](int c, f32x4 (&pin)[TMAX]) __attribute__((always_inline)) {
        const unsigned so = c * CK * HW * ES;
        const bool on = c < t.nchunks;
#pragma unroll
        for (int k = 0; k < TMAX; ++k) pin[k] = buf_load_in<TIN>(rx, on ? xoff[k] : kOob, so, 1);
    };
    auto commit_x = [&](int stage, const f32x4 (&pin)[TMAX]) __attribute__((always_inline)) {
        char *bb = reinterpret_cast<char *>(ring) + (stage ? t.stage_floats * 4 : 0);
#pragma unroll
        for (int k = 0; k < TMAX; ++k) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pin[k];   // idle slots: the spare one
    };

    // First and second chunk's input of the first tile (the first chunk's weights are on their way).
    fetch_x(0, pin0);
    fetch_x(1, pin1);
    GSPC_STAMPW(1)

    f32x4 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Halo columns of both stages are never written by the staging: clear once.
    {
        const int rows = CK * t.NB * t.IHt;
        const int right = t.XO + p.W;
        for (int i = lane; i < 2 * rows; i += 64) {
            const int b = i >= rows, rr = i - b * rows;
            const int cimg = fast_div(rr, t.m_IHt), r = rr - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            float *row = ring + b * t.stage_floats + c * t.PLANE + img * t.IMG + r * t.LW;
            for (int x = 0; x < t.XO; ++x) row[x] = 0.f;
            for (int x = right; x < t.LW; ++x) row[x] = 0.f;
        }
    }

    // The reduction of a chunk is a sequence of R = 3*CKB rows (one filter row of
    // one 4-channel block: 3 k-steps).  The operands of row i+1 are read from
    // LDS while row i is multiplied (two register sets), across chunk borders
    // too, so that the matrix core does not wait for LDS.
    constexpr int R = 3 * CKB, KS = 3 * R;
    float opa[2][3][MI], opb[2][3][NI];
    // One k-step (tap kw of a row of chunk c) of operands, and of MFMAs.
    auto load_kw = [&](int c, int row, int kw, float (&a)[3][MI], float (&b)[3][NI]) __attribute__((always_inline)) {
        const int cb = row / 3, khh = row - 3 * cb;
        const float *xrow = ring + (c & 1) * t.stage_floats + cb * 4 * t.PLANE + khh * t.LW;
        const float *ws = smem + (c * KCHUNK + row * 3) * (MI * 64) + lane;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a[kw][mi] = ws[(kw * MI + mi) * 64];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) b[kw][ni] = xrow[base[ni] + kw];
    };
    auto load_row = [&](int c, int row, float (&a)[3][MI], float (&b)[3][NI]) __attribute__((always_inline)) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) load_kw(c, row, kw, a, b);
    };
    auto mfma_kw = [&](int kw, const float (&a)[3][MI], const float (&b)[3][NI]) __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kw][mi], b[kw][ni], acc[mi][ni], 0, 0, 0);
    };
    // One chunk (no barriers): chunk c is multiplied out of stage c&1 while chunk c+2 is requested
    // from global memory into the register set pf and chunk c+1 moves from the register set pc
    // into the other stage.  Row i is multiplied while row i+1 is read, tap by tap: the reads of a
    // tap follow that tap's MFMAs, so they issue while the matrix unit works (a burst of all reads
    // in front of a row's MFMAs left the unit idle for the time the burst takes to issue).  The loads
    // and the LDS writes are dealt out one per k-step the same way; the writes come before the last
    // row, whose operand reads already belong to chunk c+1.  Every slot is always requested and always committed (idle slots
    // and chunks past the end carry zeros into the spare slots or into a stage nobody reads again),
    // so the body holds no branch and the compiler can tell at every wait which loads are in flight.
    auto chunk = [&](int c, auto par, auto io, f32x4 (&pf)[TMAX], const f32x4 (&pc)[TMAX], int cstage)
                     __attribute__((always_inline)) {
        constexpr int P = decltype(par)::value;
        constexpr bool IO = decltype(io)::value;
        const unsigned so = (c + 2) * CK * HW * ES;
        const bool on = c + 2 < t.nchunks;
        const int cn = c + 1 < t.nchunks ? c + 1 : c;   // the last chunk's look-ahead re-reads its own first row (unused)
        char *bb = reinterpret_cast<char *>(ring) + (cstage ? t.stage_floats * 4 : 0);
#pragma unroll
        for (int i = 0; i < R; ++i) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int s = i * 3 + kw;
                mfma_kw(kw, opa[(P + i) & 1], opb[(P + i) & 1]);
                if (IO) {
#pragma unroll
                    for (int k = 0; k < TMAX; ++k) {
                        const int fs = k < KS ? k : KS - 1;
                        const int cs = KS - 4 - (TMAX - 1 - k) > 0 ? KS - 4 - (TMAX - 1 - k) : 0;
                        if (fs == s) pf[k] = buf_load_in<TIN>(rx, on ? xoff[k] : kOob, so, 1);
                        if (cs == s) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pc[k];
                    }
                }
                load_kw(i + 1 < R ? c : cn, i + 1 < R ? i + 1 : 0, kw, opa[(P + i + 1) & 1], opb[(P + i + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // ---- the one barrier: weights and every wave's first chunk are in LDS -----
    // (memory loads return in order: waiting for all of them covers the weights, whose arrival no
    // register dependence would otherwise make the wave wait for)
    commit_x(0, pin0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    GSPC_STAMPW(2)
    GSPC_STAMPW(3)
    GSPC_STAMPW(4)
#ifdef GSPC_PHASE_TIMING
    const unsigned long long clk0 = __builtin_amdgcn_s_memtime();
#endif
    constexpr int P1 = R & 1;   // register set that holds row 0 of an odd chunk
    load_row(0, 0, opa[0], opb[0]);

    // Chunk pairs (even chunk: pin0 is free, pin1 holds the next one; odd chunk: the other way
    // round), then a last even chunk with nothing left to request or to commit.
    auto steady = [&]() __attribute__((always_inline)) {
        using std::integral_constant;
        const integral_constant<bool, true> yes{};
        const integral_constant<bool, false> no{};
        int c = 0;
        for (; c + 1 < t.nchunks; c += 2) {
            chunk(c, integral_constant<int, 0>{}, yes, pin0, pin1, 1);
            chunk(c + 1, integral_constant<int, P1>{}, yes, pin1, pin0, 0);
        }
        if (c < t.nchunks) chunk(c, integral_constant<int, 0>{}, no, pin0, pin1, 1);
    };
    // ---- epilogue: optional residual and ReLU, NCHW store -------------------
    // Register r of tile (mi, ni) is filter 16*(tile row) + 4*(lane/16) + r at
    // this lane's pixel; the 4*(lane/16) part already sits in ooff.
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const unsigned oc0 = ob * MI * 16;
    auto epilogue = [&](const unsigned (&ooff)[NI]) __attribute__((always_inline)) {
    if (p.res) {
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res, t.y_bytes);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[mi][ni][r] += __uint_as_float(
                        __builtin_amdgcn_raw_buffer_load_b32(rr, ooff[ni], (oc0 + mi * 16 + r) * HWo * 4, 0));
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[mi][ni][r];
                if (p.relu) v = fmaxf(v, 0.f);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), ry, ooff[ni],
                                                      (oc0 + mi * 16 + r) * HWo * 4, 0);
            }
    };

    steady();
#ifdef GSPC_PHASE_TIMING
    if (threadIdx.x == 0) {
        const unsigned bid = blockIdx.x + blockIdx.y * gridDim.x;
        if (bid < 4096) g_phase_w[bid * 8 + 7] = (__builtin_amdgcn_s_memtime() - clk0) & 0xffffffffull;
    }
#endif

    // ---- further pixel tiles of this block (large batches): the filters stay ----
    // The next tile's first two chunks are requested before the results of the
    // current one are stored, so their latency hides behind the epilogue.
    if (!PERSIST) {   // one tile group per block: the common, latency-bound case, kept lean
        GSPC_STAMPW(5)
        epilogue(ooff);
        GSPC_STAMPW(6)
        return;
    }
    for (int tg = blockIdx.x;;) {
        const int next = tg + gridDim.x;
        unsigned ooff_done[NI];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) ooff_done[ni] = ooff[ni];
        const bool more = next < t.tile_groups;
        if (more) {
            set_tile(next);
            fetch_x(0, pin0);
            fetch_x(1, pin1);
        }
        epilogue(ooff_done);
        if (!more) break;
        tg = next;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
        commit_x(0, pin0);
        load_row(0, 0, opa[0], opb[0]);
        steady();
    }
    GSPC_STAMPW(6)
}

#ifdef GSPC_PHASE_TIMING
extern "C" int gspc_debug_phases_w(unsigned long long *out, int n) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_w), sizeof(unsigned long long) * n);
}
#endif

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kLdsMaxW = 160 * 1024;

struct CfgW {
    int MI, NI;
};
// Largest wave tile first.
const CfgW kCfgW[] = {{2, 4}, {2, 2}, {1, 4}, {1, 2}, {1, 1}};
constexpr int kNumCfgW = sizeof(kCfgW) / sizeof(kCfgW[0]);

// Worst bank multiplicity (32 banks of 4 bytes) of a B-operand read for a
// candidate channel pitch.
int bank_cost_w(const ConvParams &p, const Tile16w &t, int plane) {
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

bool planW_cfg(const ConvParams &p, const PackGeom &g, const CfgW &c, int ckb, Tile16w *out) {
    const int MB = 16 * c.MI, PW = 16 * c.NI, CK = 4 * ckb;
    if ((g.mtiles * 16) % MB || g.CPG % CK) return false;
    Tile16w t{};
    if (!split_pixels(p, PW, &t.NB, &t.TH)) return false;
    t.IHt = (t.TH - 1) * p.stride + 3;
    t.XO = 4 * ((p.pad + 3) / 4);
    t.LW = round_up(t.XO + p.W + p.pad, 4);
    t.IMG = t.IHt * t.LW;
    const int plane0 = round_up(t.NB * t.IMG, 4);
    int best_pad = 0, best_cost = 1 << 30;
    for (int pad = 0; pad < 32; pad += 4) {
        const int cost = bank_cost_w(p, t, plane0 + pad);
        if (cost < best_cost) {
            best_cost = cost;
            best_pad = pad;
        }
    }
    t.PLANE = plane0 + best_pad;
    const int cols = p.W / 4;
    t.tpr_log2 = 0;
    while ((1 << t.tpr_log2) < cols) ++t.tpr_log2;
    if ((1 << t.tpr_log2) > 64) return false;
    const int rpp = 64 >> t.tpr_log2;
    t.tasks = CK * t.NB * t.IHt;
    t.xslots = (t.tasks + rpp - 1) / rpp;
    const int tmax = p.stride == 2 ? kTmaxW2 : kTmaxW;
    if (t.xslots > tmax) return false;
    t.xs = t.xslots <= tmax / 2 ? tmax / 2 : tmax;     // the instances are built for half and for all of the slots
    t.ksteps = g.ksteps;
    t.mtiles = g.mtiles;
    t.nchunks = g.CPG / CK;
    const int units = g.ksteps * c.MI * 16;            // 16-byte units of the block's weights
    t.wslots = (units + 255) / 256;
    if (t.wslots > kWmaxW) return false;
    t.w_floats = t.wslots * 256 * 4;
    t.stage_floats = CK * t.PLANE + 256;   // tile, then a spare 16-byte slot per lane
    const size_t lds = ((size_t)t.w_floats + 8 * (size_t)t.stage_floats) * sizeof(float);
    if (lds > kLdsMaxW) return false;
    t.row_blocks = (p.Hout + t.TH - 1) / t.TH;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.oc_blocks = g.mtiles * 16 / MB;
    const long wt = (long)t.row_blocks * t.img_blocks;
    if (wt > 1000000000L || p.groups * t.oc_blocks > 65535) return false;
    t.wave_tiles = (int)wt;
    t.tile_groups = (t.wave_tiles + 3) / 4;
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_ppi = div_magic(t.TH * p.Wout);
    t.m_Wout = div_magic(p.Wout);
    t.m_rowb = div_magic(t.row_blocks);
    t.m_ocb = div_magic(t.oc_blocks);
    const double xb = (double)p.N * p.Cin * p.H * p.W * (p.in_bf16 ? 2 : 4);
    const double yb = (double)p.N * p.Cout * p.Hout * p.Wout * 4;
    const double wb = (double)p.groups * g.ksteps * g.mtiles * 256;
    if (xb >= (double)kOob || yb >= (double)kOob || wb >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)wb;
    if ((double)wt * t.row_blocks >= 4.0e9 || (double)p.groups * t.oc_blocks * t.oc_blocks >= 4.0e9 ||
        t.tasks >= 65536 || t.TH * p.Wout >= 65536)
        return false;
    *out = t;
    return true;
}

// One block per group of four wave tiles while the chip can hold them all at once; beyond that
// every block walks over several tile groups, keeping its filters.
long grid_x_w(const ConvParams &p, const Tile16w &t, size_t lds) {
    const long gy = (long)p.groups * t.oc_blocks;
    long per_cu = (long)(kLdsMaxW / lds);
    per_cu = per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu;
    const long cap = kNumCU * per_cu, total = (long)t.tile_groups * gy;
    if (total <= cap) return t.tile_groups;
    const long rounds = (total + cap - 1) / cap;
    return (t.tile_groups + rounds - 1) / rounds;
}

size_t lds_bytes_w(const Tile16w &t);

size_t lds_bytes_w(const Tile16w &t) {
    return ((size_t)t.w_floats + 8 * (size_t)t.stage_floats) * sizeof(float);
}

template <int MI, int NI, int S, int CKB, bool PERSIST, int XS>
hipError_t launchW_kernel(const ConvParams &p, const Tile16w &t, dim3 grid, size_t lds, hipStream_t s) {
    auto kern = conv_mfma16w<MI, NI, S, CKB, PERSIST, XS, float>;
    if (lds > 64 * 1024) {
        static thread_local bool raised = false;   // per instantiation and thread
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMaxW);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, p, t);
    return hipGetLastError();
}

template <int MI, int NI, int S, int CKB, int XS>
hipError_t launchW_inst(const ConvParams &p, const Tile16w &t, hipStream_t s) {
    const size_t lds = lds_bytes_w(t);
    const long gx = grid_x_w(p, t, lds), gy = (long)p.groups * t.oc_blocks;
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (gx < t.tile_groups) return launchW_kernel<MI, NI, S, CKB, true, XS>(p, t, grid, lds, s);
    return launchW_kernel<MI, NI, S, CKB, false, XS>(p, t, grid, lds, s);
}

template <int MI, int NI, int S>
hipError_t launchW_xs(int ckb, const ConvParams &p, const Tile16w &t, hipStream_t s) {
    constexpr int TM = S == 2 ? kTmaxW2 : kTmaxW;
    if (t.xs == TM / 2)
        return ckb == 2 ? launchW_inst<MI, NI, S, 2, TM / 2>(p, t, s) : launchW_inst<MI, NI, S, 1, TM / 2>(p, t, s);
    return ckb == 2 ? launchW_inst<MI, NI, S, 2, TM>(p, t, s) : launchW_inst<MI, NI, S, 1, TM>(p, t, s);
}

template <int MI, int NI>
hipError_t launchW_shape(int stride, int ckb, const ConvParams &p, const Tile16w &t, hipStream_t s) {
    return stride == 1 ? launchW_xs<MI, NI, 1>(ckb, p, t, s) : launchW_xs<MI, NI, 2>(ckb, p, t, s);
}

}  // namespace

bool plan_mfma16w(const ConvParams &p, const PackGeom &g, Mfma16wPlan *out) {
    static const bool off = std::getenv("GSPC_NO_RESIDENT") != nullptr;   // tuning aid
    if (off || g.variant != kMfma16 || !p.wm || p.in_bf16 || p.KH != 3 || p.KW != 3 ||
        (p.stride != 1 && p.stride != 2) || p.W % 4 || g.CPG % 4 || g.CPGp != g.CPG)
        return false;
    // Findings of the tile-table autotuner for stride-2 layers: the plain 16x16x4 kernel is 6-20 %
    // faster with at most 16 channels per group and 10-25 % faster at batch 16 and below; at batch 64
    // this kernel wins by up to 30 %; at batch 128 and above it wins (7-17 %, with the larger
    // stride-2 tiles that eight staging slots allow) from 64 channels per group on and loses
    // below.  A table can overrule.
    const bool asked = tuned_family(p) == 'w';
    if (p.stride == 2 && !asked && (g.CPG <= 16 || (p.N >= 128 && g.CPG <= 32) || p.N <= 16)) return false;
    static const char *force = std::getenv("GSPC_TILEW");
    const int ckb = g.CPG % 8 == 0 ? 2 : 1;
    int forced = force ? std::atoi(force) : tuned_config(p, 'w');
    {
        Tile16w t;
        if (!force && forced >= 0 && (forced >= kNumCfgW || !planW_cfg(p, g, kCfgW[forced], ckb, &t))) forced = -1;
    }
    int best = -1;
    long best_waves = -1;
    Tile16w bt{};
    for (int i = 0; i < kNumCfgW; ++i) {
        Tile16w t;
        if (forced >= 0 && forced != i) continue;
        if (!planW_cfg(p, g, kCfgW[i], ckb, &t)) continue;
        const long waves = (long)t.wave_tiles * t.oc_blocks * p.groups;
        if (waves >= 4 * kNumCU) {   // every SIMD has a wave: take the largest such tile
            best = i;
            best_waves = waves;
            bt = t;
            break;
        }
        if (waves > best_waves) {
            best_waves = waves;
            best = i;
            bt = t;
        }
    }
    if (best < 0) return false;
    // Fewer than two waves per compute unit and a long reduction (batch 1): the plain kernel, which
    // then lets the four waves of a block split the reduction, is 10-15 % faster.
    if (!asked && !force && best_waves >= 0 && best_waves < 2 * kNumCU && g.ksteps >= 36) return false;
    out->inst = best;
    out->ckb = ckb;
    static_assert(sizeof(Tile16w) <= sizeof(out->data), "plan storage too small");
    std::memcpy(out->data, &bt, sizeof(bt));
    return true;
}

hipError_t launch_mfma16w(const ConvParams &p, const Mfma16wPlan &plan, hipStream_t s, const char **name) {
    Tile16w t;
    std::memcpy(&t, plan.data, sizeof(t));
    const CfgW &c = kCfgW[plan.inst];
    const bool persist = grid_x_w(p, t, lds_bytes_w(t)) < t.tile_groups;
    *name = intern_name("conv_mfma16w<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," +
                        std::to_string(p.stride) + "," + std::to_string(plan.ckb) + "," +
                        (persist ? "true" : "false") + "," + std::to_string(t.xs) + ",f32>");
    switch (plan.inst) {
    case 0: return launchW_shape<2, 4>(p.stride, plan.ckb, p, t, s);
    case 1: return launchW_shape<2, 2>(p.stride, plan.ckb, p, t, s);
    case 2: return launchW_shape<1, 4>(p.stride, plan.ckb, p, t, s);
    case 3: return launchW_shape<1, 2>(p.stride, plan.ckb, p, t, s);
    case 4: return launchW_shape<1, 1>(p.stride, plan.ckb, p, t, s);
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
