// Grouped Winograd F(2x2, 3x3) convolution on the gfx950 matrix cores.
//
// The paper (arXiv 2006.09791, Section VI) names a grouped Winograd convolution as the
// next step after GSPC.  For one group, a 2x2 block of outputs of filter k is
//     Y = A^T [ sum_c (G g_kc G^T) .* (B^T d_c B) ] A
// with d_c the 4x4 input patch of channel c and g_kc the 3x3 filter (Lavin & Gray's
// minimal filtering F(2x2, 3x3)): 16 multiplications per channel instead of 36.  The sum
// over c is, for each of the 16 positions (xi, nu) of the transformed domain, the
// contraction  M[xi,nu][k][tile] = sum_c U[xi,nu][k][c] * V[xi,nu][c][tile]:
// sixteen independent GEMMs per group, run here as v_mfma_f32_16x16x4_f32 with
// filters on the M edge and 2x2 output tiles on the N edge.
//
//   U = G g G^T is computed once, at packing time (the paper's kernel reshape stage),
//       and stored in MFMA A-operand order.
//   V = B^T d B is computed per block from a zero-haloed input tile staged in LDS
//       (the input reshape stage, fused) and kept in LDS as the B operand.
//   A wave keeps all sixteen M accumulators of its (filters x tiles) sub-block in
//   registers, so the inverse transform A^T M A needs no exchange between lanes; the
//   2x2 results go straight to NCHW (output reshape fused away).
//
//   Where a wave holds one product tile (16 filters x 16 output tiles), V never goes through LDS
//   (template argument RT): lane l of the wave needs, as the B operand of the sixteen MFMAs of a
//   k-step, the sixteen transformed values of channel l/16, tile l%16 - exactly what one 4x4 patch
//   gives - so every lane reads its own patch from the staged tile and transforms it in registers,
//   the next k-step's while the current one multiplies.  No V buffer, no LDS writes, one barrier per
//   chunk (the staged tile is double-buffered).
//
// Stride 1, pad 1, fp32, KPG >= 12 (the last filter tile zero-padded), CPG a multiple of 4.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "conv_common.h"

namespace gspc {

struct TileX {
    int NB, TR, TC, TRtot;   // images and tile rows per block; tile columns and rows of a plane
    int tpi, P;              // tiles per image in a block (TR*TC); tiles per block (NB*tpi)
    int IHt, LW, IMG, PLANE, XO;   // staged rows (2*TR+2), row pitch, floats per image / channel, column of input col 0
    int nchunks;             // chunks of CK = 4*CKB channels
    int row_blocks, img_blocks, oc_blocks;
    int tpr_log2, vec, tasks, xslots;
    int cblks, mtiles;       // CPG/4, KPG/16: geometry of the packed section
    int raw_floats;
    int wodd;                // odd plane width: 4-byte stores with a column check
    int rt;                  // V transformed in registers by the wave that multiplies it (one product tile per wave)
    unsigned m_IHt, m_NB, m_tpi, m_TC, m_rowb, m_ocb;
    unsigned x_bytes, u_bytes, y_bytes;
};

constexpr int kTmaxX = 4;

template <int MI, int NI, int WM, int WP, int CKB, bool RT>
__global__ __launch_bounds__(64 * WM * WP, 2) void conv_wino(ConvParams p, TileX t) {
    static_assert(!RT || (MI == 1 && NI == 1), "the register transform serves one product tile per wave");
    constexpr int NT = 64 * WM * WP, PT = 16 * NI * WP, VP = PT + 16, MIWM = MI * WM, CK = 4 * CKB;
    constexpr int TMAX = kTmaxX;
    constexpr int CPP = NT / PT;                  // channels transformed per pass of the block
    constexpr int TPASS = (CK + CPP - 1) / CPP;
    extern __shared__ f32x4 smem4[];
    float *raw = reinterpret_cast<float *>(smem4);   // [CK][PLANE] (RT: two of them)
    float *V = raw + t.raw_floats;                   // [16][CK][VP]; VP = 16 mod 32: conflict-free operand reads
    const unsigned spare = RT ? 2 * t.raw_floats * 4 : (t.raw_floats + 16 * CK * VP) * 4;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WP, wp = wave % WP;
    const unsigned ib = fast_div(blockIdx.x, t.m_rowb);
    const int rb = blockIdx.x - ib * t.row_blocks;
    const unsigned j = fast_div(blockIdx.y, t.m_ocb);
    const int ob = blockIdx.y - j * t.oc_blocks;
    const int n0 = ib * t.NB, tr0 = rb * t.TR, ih0 = 2 * tr0 - 1;
    const unsigned HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t ru = make_rsrc(p.wx, t.u_bytes);

    // ---- input staging plan (identical for every chunk) ----------------------
    const int rpp = NT >> t.tpr_log2;
    const int row0 = tid >> t.tpr_log2, colv = tid & ((1 << t.tpr_log2) - 1);
    const int vw = t.vec ? 4 : 1;
    unsigned xoff[TMAX], xlds[TMAX];
    // (the first chunk's load of a slot is requested as soon as the slot's offset is known: the index
    // arithmetic of the other slots then runs under its latency)
    f32x4 pin[TMAX];
#pragma unroll
    for (int k = 0; k < TMAX; ++k) {
        const int task = row0 + k * rpp;
        xoff[k] = kOob;
        xlds[k] = spare;
        if (k < t.xslots && task < t.tasks && colv * vw < p.W) {
            const int cimg = fast_div(task, t.m_IHt), r = task - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            const int ih = ih0 + r, n = n0 + img;
            // rows above and below the image load as zero: the halo rows are rewritten with every chunk
            if (n < p.N && ih >= 0 && ih < p.H)
                xoff[k] = ((((unsigned)n * p.Cin + j * p.CPG + c) * p.H + ih) * p.W + colv * vw) * 4;
            xlds[k] = (c * t.PLANE + img * t.IMG + r * t.LW + t.XO + colv * vw) * 4;
        }
        if (k < t.xslots) pin[k] = buf_load_in<float>(rx, xoff[k], 0, t.vec);
        __builtin_amdgcn_sched_barrier(0);
    }
    auto fetch_x = [&](int chunk) __attribute__((always_inline)) {
        const unsigned so = chunk * CK * HW * 4;
#pragma unroll
        for (int k = 0; k < TMAX; ++k)
            if (k < t.xslots) pin[k] = buf_load_in<float>(rx, xoff[k], so, t.vec);
    };

    // ---- U operand: [g][cblk][mtile][4][64 lanes] float4, four consecutive (xi, nu) per float4 ----
    f32x4 ua[CKB][MI][4];
    auto fetch_u = [&](int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < CKB; ++cb)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const unsigned mt = ob * MIWM + wm * MI + mi;
                const unsigned so = (((j * t.cblks + chunk * CKB + cb) * t.mtiles + mt) * 4) * 1024;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    ua[cb][mi][qd] = __builtin_bit_cast(
                        f32x4, __builtin_amdgcn_raw_buffer_load_b128(ru, lane * 16, so + qd * 1024, 0));
            }
    };

    // ---- this thread's tile in the transform pass ----
    const int tq = tid % PT, tc0 = tid / PT;
    int pbase;
    {
        const int qq = tq < t.P ? tq : 0;
        const int img = fast_div(qq, t.m_tpi), rem = qq - img * t.tpi;
        const int tr = fast_div(rem, t.m_TC), tc = rem - tr * t.TC;
        pbase = img * t.IMG + 2 * tr * t.LW + (t.XO - 1) + 2 * tc;
    }

    // Halo columns left and right of a staged row are never written by the staging: clear them once.
    {
        const int rows = CK * t.NB * t.IHt, right = t.XO + p.W;
        for (int i = tid; i < (RT ? 2 : 1) * rows; i += NT) {
            const int b = i >= rows, ii = i - b * rows;
            const int cimg = fast_div(ii, t.m_IHt), r = ii - cimg * t.IHt;
            const int c = fast_div(cimg, t.m_NB), img = cimg - c * t.NB;
            float *row = raw + b * t.raw_floats + c * t.PLANE + img * t.IMG + r * t.LW;
            for (int x = 0; x < t.XO; ++x) row[x] = 0.f;
            for (int x = right; x < t.LW; ++x) row[x] = 0.f;
        }
    }

    f32x4 acc[16][MI][NI];
#pragma unroll
    for (int xn = 0; xn < 16; ++xn)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) acc[xn][mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    if constexpr (RT) {
        // ---- register transform: this lane's patch (channel lane/16 of the k-step, tile lane%16 of the wave) ----
        int pbase_r;
        {
            const int q = wp * 16 + (lane & 15);
            const int qq = q < t.P ? q : 0;
            const int img = fast_div(qq, t.m_tpi), rem = qq - img * t.tpi;
            const int tr = fast_div(rem, t.m_TC), tc = rem - tr * t.TC;
            pbase_r = (lane >> 4) * t.PLANE + img * t.IMG + 2 * tr * t.LW + (t.XO - 1) + 2 * tc;
        }
        f32x4 ub[2][CKB][4];   // U of this chunk and of the next one
        float vb[2][16];       // V of this k-step and of the next one
        float d[4][4], w[4][4];
        auto fetch_ub = [&](int chunk, f32x4 (&u)[CKB][4]) __attribute__((always_inline)) {
#pragma unroll
            for (int cb = 0; cb < CKB; ++cb) {
                const unsigned mt = ob * MIWM + wm;
                const unsigned so = (((j * t.cblks + chunk * CKB + cb) * t.mtiles + mt) * 4) * 1024;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    u[cb][qd] = __builtin_bit_cast(
                        f32x4, __builtin_amdgcn_raw_buffer_load_b128(ru, lane * 16, so + qd * 1024, 0));
            }
        };
        // B^T d B in sixteen slices, one behind each MFMA of the k-step before: rows of the patch are read in
        // slices 0-3, the column pass runs in slices 8-11 (by then the reads have returned), the row pass in 12-15.
        auto slice = [&](int i, const float *src, float (&out)[16]) __attribute__((always_inline)) {
            if (i < 4) {
#pragma unroll
                for (int x = 0; x < 4; ++x) d[i][x] = src[i * t.LW + x];
            } else if (i >= 8 && i < 12) {
                const int x = i - 8;
                w[0][x] = d[0][x] - d[2][x];
                w[1][x] = d[1][x] + d[2][x];
                w[2][x] = d[2][x] - d[1][x];
                w[3][x] = d[1][x] - d[3][x];
            } else if (i >= 12) {
                const int xi = i - 12;
                out[xi * 4 + 0] = w[xi][0] - w[xi][2];
                out[xi * 4 + 1] = w[xi][1] + w[xi][2];
                out[xi * 4 + 2] = w[xi][2] - w[xi][1];
                out[xi * 4 + 3] = w[xi][1] - w[xi][3];
            }
        };
        auto commit_x = [&](int ch) __attribute__((always_inline)) {
            char *bb = reinterpret_cast<char *>(raw + (ch & 1) * t.raw_floats);
#pragma unroll
            for (int k = 0; k < TMAX; ++k) {
                if (k < t.xslots) {
                    if (t.vec) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pin[k];
                    else *reinterpret_cast<float *>(bb + xlds[k]) = pin[k].x;
                }
            }
        };
        // One chunk.  On entry vb[VB0] holds V of its first k-step, ub[PB] its U, and the input of chunk ch+1 is
        // on its way into pin.  The sixteen MFMAs of a k-step carry, one slice or one load each: the transform of
        // the next k-step; the loads of chunk ch+1's U (first k-step) and of chunk ch+2's input (last k-step, after
        // pin has been committed).  Before the last k-step chunk ch+1 is committed to the other staged tile and the
        // block meets at its one barrier per chunk, so that the last k-step can already transform chunk ch+1's first
        // one.  (The other tile was last read before the previous barrier.)
        auto chunk = [&](int ch, auto par) __attribute__((always_inline)) {
            constexpr int PB = decltype(par)::value, VB0 = CKB % 2 ? PB : 0;
            const bool more = ch + 1 < t.nchunks;
            const float *src = raw + (ch & 1) * t.raw_floats + pbase_r;
            const float *nxt = raw + ((ch + 1) & 1) * t.raw_floats + pbase_r;
            const unsigned xso = (ch + 2) * CK * HW * 4;
            const bool xon = ch + 2 < t.nchunks;
#pragma unroll
            for (int cb = 0; cb < CKB; ++cb) {
                const bool last = cb == CKB - 1;
                if (last && more) {
                    commit_x(ch + 1);
                    __syncthreads();
                }
                const float *srcn = last ? nxt : src + (cb + 1) * 4 * t.PLANE;
#pragma unroll
                for (int xn = 0; xn < 16; ++xn) {
                    acc[xn][0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(ub[PB][cb][xn >> 2][xn & 3],
                                                                       vb[(VB0 + cb) & 1][xn], acc[xn][0][0], 0, 0, 0);
                    slice(xn, srcn, vb[(VB0 + cb + 1) & 1]);
                    if (cb == 0 && xn % 2 == 1 && xn / 2 < CKB * 4) {   // U of the next chunk: CKB * 4 loads
                        const int l = xn / 2, ucb = l / 4, qd = l % 4;
                        const unsigned mt = ob * MIWM + wm;
                        const unsigned so = (((j * t.cblks + (ch + 1) * CKB + ucb) * t.mtiles + mt) * 4) * 1024;
                        ub[PB ^ 1][ucb][qd] = __builtin_bit_cast(
                            f32x4, __builtin_amdgcn_raw_buffer_load_b128(ru, lane * 16, so + qd * 1024, 0));
                    }
                    if (last && xn >= 4 && xn < 4 + TMAX) {             // input of chunk ch+2
                        const int k = xn - 4;
                        if (k < t.xslots) pin[k] = buf_load_in<float>(rx, xon ? xoff[k] : kOob, xso, t.vec);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        fetch_ub(0, ub[0]);
        commit_x(0);
        __syncthreads();
        if (t.nchunks > 1) fetch_x(1);
#pragma unroll
        for (int i = 0; i < 16; ++i) slice(i, raw + pbase_r, vb[0]);
        int ch = 0;
        for (; ch + 1 < t.nchunks; ch += 2) {
            chunk(ch, std::integral_constant<int, 0>{});
            chunk(ch + 1, std::integral_constant<int, 1>{});
        }
        if (ch < t.nchunks) chunk(ch, std::integral_constant<int, 0>{});
    } else {
        const float *vrd = V + (lane >> 4) * VP + wp * NI * 16 + (lane & 15);
        for (int ch = 0; ch < t.nchunks; ++ch) {
            fetch_u(ch);   // needed after the transform: its latency passes meanwhile
            {
                char *bb = reinterpret_cast<char *>(raw);
#pragma unroll
                for (int k = 0; k < TMAX; ++k) {
                    if (k < t.xslots) {
                        if (t.vec) *reinterpret_cast<f32x4 *>(bb + xlds[k]) = pin[k];
                        else *reinterpret_cast<float *>(bb + xlds[k]) = pin[k].x;
                    }
                }
            }
            __syncthreads();
            if (ch + 1 < t.nchunks) fetch_x(ch + 1);
            // ---- V = B^T d B for (channel, tile) pairs ----
#pragma unroll
            for (int k = 0; k < TPASS; ++k) {
                const int c = tc0 + k * CPP;
                if (CK % CPP == 0 || c < CK) {
                    const float *d = raw + c * t.PLANE + pbase;
                    float w[4][4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const float d0 = d[x], d1 = d[t.LW + x], d2 = d[2 * t.LW + x], d3 = d[3 * t.LW + x];
                        w[0][x] = d0 - d2;
                        w[1][x] = d1 + d2;
                        w[2][x] = d2 - d1;
                        w[3][x] = d1 - d3;
                    }
                    float *vo = V + c * VP + tq;
#pragma unroll
                    for (int xi = 0; xi < 4; ++xi) {
                        vo[(xi * 4 + 0) * CK * VP] = w[xi][0] - w[xi][2];
                        vo[(xi * 4 + 1) * CK * VP] = w[xi][1] + w[xi][2];
                        vo[(xi * 4 + 2) * CK * VP] = w[xi][2] - w[xi][1];
                        vo[(xi * 4 + 3) * CK * VP] = w[xi][1] - w[xi][3];
                    }
                }
            }
            __syncthreads();
            // ---- sixteen GEMM steps per 4-channel block ----
#pragma unroll
            for (int cb = 0; cb < CKB; ++cb)
#pragma unroll
                for (int xn = 0; xn < 16; ++xn) {
                    float b[NI];
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) b[ni] = vrd[(xn * CK + cb * 4) * VP + ni * 16];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
                            acc[xn][mi][ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(ua[cb][mi][xn >> 2][xn & 3], b[ni],
                                                                                   acc[xn][mi][ni], 0, 0, 0);
                }
            // the next chunk's staging writes `raw` (free since the second barrier) and, after
            // its first barrier, V (every wave is past this loop by then)
        }
    }

    // ---- inverse transform Y = A^T M A, optional residual and ReLU, NCHW stores ----
    // Register r of an accumulator is filter 16*(tile row) + 4*(lane/16) + r at tile lane%16.
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);
    const unsigned oc0 = (ob * MIWM + wm * MI) * 16;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int q = (wp * NI + ni) * 16 + (lane & 15);
        const int qq = q < t.P ? q : 0;
        const int img = fast_div(qq, t.m_tpi), rem = qq - img * t.tpi;
        const int tr = fast_div(rem, t.m_TC), tc = rem - tr * t.TC;
        const int n = n0 + img, oh = 2 * (tr0 + tr), ow = 2 * tc;
        const bool ok = q < t.P && n < p.N && oh < p.H;
        const unsigned o0 = ok ? (((unsigned)n * p.Cout + j * p.KPG + 4 * (lane >> 4)) * HW + oh * p.W + ow) * 4 : kOob;
        const unsigned o1 = ok && oh + 1 < p.H ? o0 + p.W * 4 : kOob;
        const bool c1 = ow + 1 < p.W;   // second column exists (always, for even widths)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float s0[4], s1[4];   // A^T M: rows 0 and 1, four columns
#pragma unroll
                for (int nu = 0; nu < 4; ++nu) {
                    const float m0 = acc[nu][mi][ni][r], m1 = acc[4 + nu][mi][ni][r], m2 = acc[8 + nu][mi][ni][r],
                                m3 = acc[12 + nu][mi][ni][r];
                    s0[nu] = m0 + m1 + m2;
                    s1[nu] = m1 - m2 - m3;
                }
                float y00 = s0[0] + s0[1] + s0[2], y01 = s0[1] - s0[2] - s0[3];
                float y10 = s1[0] + s1[1] + s1[2], y11 = s1[1] - s1[2] - s1[3];
                const unsigned so = (oc0 + mi * 16 + r) * HW * 4;
                // filters past KPG in a zero-padded last tile neither load a residual nor store
                const bool fk = oc0 + mi * 16 + 4 * (lane >> 4) + r < (unsigned)p.KPG;
                const unsigned p0 = fk ? o0 : kOob, p1 = fk ? o1 : kOob;
                if (!t.wodd) {
                    if (p.res) {
                        const u32x2 ra = __builtin_amdgcn_raw_buffer_load_b64(rr, p0, so, 0);
                        const u32x2 rb2 = __builtin_amdgcn_raw_buffer_load_b64(rr, p1, so, 0);
                        y00 += __uint_as_float(ra.x);
                        y01 += __uint_as_float(ra.y);
                        y10 += __uint_as_float(rb2.x);
                        y11 += __uint_as_float(rb2.y);
                    }
                    if (p.relu) {
                        y00 = fmaxf(y00, 0.f);
                        y01 = fmaxf(y01, 0.f);
                        y10 = fmaxf(y10, 0.f);
                        y11 = fmaxf(y11, 0.f);
                    }
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{__float_as_uint(y00), __float_as_uint(y01)}, ry, p0, so, 0);
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{__float_as_uint(y10), __float_as_uint(y11)}, ry, p1, so, 0);
                } else {
                    const unsigned o0b = c1 ? p0 + 4 : kOob, o1b = c1 ? p1 + 4 : kOob;
                    if (p.res) {
                        y00 += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, p0, so, 0));
                        y01 += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, o0b, so, 0));
                        y10 += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, p1, so, 0));
                        y11 += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rr, o1b, so, 0));
                    }
                    if (p.relu) {
                        y00 = fmaxf(y00, 0.f);
                        y01 = fmaxf(y01, 0.f);
                        y10 = fmaxf(y10, 0.f);
                        y11 = fmaxf(y11, 0.f);
                    }
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y00), ry, p0, so, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y01), ry, o0b, so, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y10), ry, p1, so, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y11), ry, o1b, so, 0);
                }
            }
    }
}


// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

struct CfgX {
    int MI, NI, WM, WP;
};
// filters x tiles per block: 32 x 64, 64 x 32, 32 x 32, 16 x 128, 16 x 64, 16 x 32, 16 x 16
const CfgX kCfgX[] = {{1, 2, 2, 2}, {2, 1, 2, 2}, {1, 1, 2, 2}, {1, 2, 1, 4}, {1, 1, 1, 4}, {1, 1, 1, 2}, {1, 1, 1, 1}};
constexpr int kNumCfgX = sizeof(kCfgX) / sizeof(kCfgX[0]);
constexpr int kLdsBudgetX = 64 * 1024;

// LDS of a block: the staged tile and V, or (register transform) two staged tiles; a spare 16 bytes.
size_t lds_bytes_x(int raw_floats, int CK, int VP, bool rt) {
    return ((rt ? 2 * (size_t)raw_floats : (size_t)raw_floats + 16 * CK * VP) + 4) * sizeof(float);
}

// The register transform is taken where a wave holds one product tile, except for very large launches, where the
// matrix cores are the bound and the V buffer's single transform is ahead: from sixteen blocks per compute unit on
// with two waves per tile set (each repeats the transform; 8 % at 32 -> 32 on 32x32, N = 1024), from forty-eight on
// with one (6 % at 64 -> 64 on 56x56 in 4 groups, N = 256).  Tuning aid: GSPC_WINO_RT=0 / 1.
bool use_rt(const CfgX &c, long blocks) {
    static const char *env = std::getenv("GSPC_WINO_RT");
    if (c.MI != 1 || c.NI != 1) return false;
    if (env) return std::atoi(env) != 0;
    return blocks < (c.WM == 1 ? 48L : 16L) * kNumCU;
}

bool planx_cfg(const ConvParams &p, const PackGeom &g, const CfgX &c, int ckb, bool rt, TileX *out) {
    const int PT = 16 * c.NI * c.WP, NT = 64 * c.WM * c.WP, MIWM = c.MI * c.WM, CK = 4 * ckb, VP = PT + 16;
    TileX t{};
    t.cblks = g.CPG / 4;
    t.mtiles = (g.KPG + 15) / 16;
    // Whole filter tiles per block; an odd tile count may leave up to a third of the tile count empty in the last block's
    // tiles empty (its U loads then read rows of other tiles or, past the section, zeros: products
    // that the store mask drops).
    const int spill = (MIWM - t.mtiles % MIWM) % MIWM;
    if (spill * 3 > t.mtiles || t.cblks % ckb) return false;
    t.TC = (p.W + 1) / 2;
    t.TRtot = (p.H + 1) / 2;
    if (t.TC > PT) return false;
    if (t.TC * t.TRtot <= PT) {
        t.TR = t.TRtot;
        t.NB = PT / (t.TC * t.TRtot);
        if (t.NB > p.N) t.NB = p.N;
    } else {
        t.NB = 1;
        const int trmax = PT / t.TC;
        const int rbk = (t.TRtot + trmax - 1) / trmax;
        t.TR = (t.TRtot + rbk - 1) / rbk;
    }
    t.tpi = t.TR * t.TC;
    t.P = t.NB * t.tpi;
    t.IHt = 2 * t.TR + 2;
    t.vec = p.W % 4 == 0;
    t.XO = t.vec ? 4 : 1;
    t.LW = round_up(t.XO + p.W + 2, 4);
    // the tiles of a wave read their patches together; with several tile rows among them (planes of 8x8 and less)
    // a row pitch of 16 floats would put every tile row on the same banks
    if (t.TC < 16 && (2 * t.LW) % 32 == 0) t.LW += 4;
    t.IMG = t.IHt * t.LW;
    t.PLANE = round_up(t.NB * t.IMG, 4);
    t.raw_floats = CK * t.PLANE;
    if (lds_bytes_x(t.raw_floats, CK, VP, rt) > (size_t)kLdsBudgetX) return false;
    t.nchunks = t.cblks / ckb;
    const int cols = t.vec ? p.W / 4 : p.W;
    while ((1 << t.tpr_log2) < cols) ++t.tpr_log2;
    if ((1 << t.tpr_log2) > NT) return false;
    const int rpp = NT >> t.tpr_log2;
    t.tasks = CK * t.NB * t.IHt;
    t.xslots = (t.tasks + rpp - 1) / rpp;
    if (t.xslots > kTmaxX) return false;
    t.row_blocks = (t.TRtot + t.TR - 1) / t.TR;
    t.img_blocks = (p.N + t.NB - 1) / t.NB;
    t.oc_blocks = (t.mtiles + MIWM - 1) / MIWM;
    t.wodd = p.W % 2;
    t.rt = rt;
    t.m_IHt = div_magic(t.IHt);
    t.m_NB = div_magic(t.NB);
    t.m_tpi = div_magic(t.tpi);
    t.m_TC = div_magic(t.TC);
    t.m_rowb = div_magic(t.row_blocks);
    t.m_ocb = div_magic(t.oc_blocks);
    const double xb = (double)p.N * p.Cin * p.H * p.W * 4, yb = (double)p.N * p.Cout * p.H * p.W * 4;
    const double ub = (double)p.groups * t.cblks * t.mtiles * 4096;
    if (xb >= (double)kOob || yb >= (double)kOob || ub >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.u_bytes = (unsigned)ub;
    if ((long)t.row_blocks * t.img_blocks > 2147483647L || p.groups * t.oc_blocks > 65535) return false;
    // fast_div exactness: numerator * divisor < 2^32
    if ((double)t.row_blocks * t.img_blocks * t.row_blocks >= 4.0e9 ||
        (double)p.groups * t.oc_blocks * t.oc_blocks >= 4.0e9 || (double)t.tasks * t.IHt >= 4.0e9 ||
        (double)t.tasks * t.NB >= 4.0e9 || (double)PT * t.tpi >= 4.0e9)
        return false;
    *out = t;
    return true;
}

template <int MI, int NI, int WM, int WP, int CKB>
hipError_t launchx_inst(const ConvParams &p, const TileX &t, bool rt, hipStream_t s) {
    constexpr int PT = 16 * NI * WP, VP = PT + 16, CK = 4 * CKB;
    const size_t lds = lds_bytes_x(t.raw_floats, CK, VP, rt);
    dim3 grid(t.row_blocks * t.img_blocks, p.groups * t.oc_blocks);
    if constexpr (MI == 1 && NI == 1) {
        if (rt) {
            hipLaunchKernelGGL((conv_wino<MI, NI, WM, WP, CKB, true>), grid, dim3(64 * WM * WP), lds, s, p, t);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((conv_wino<MI, NI, WM, WP, CKB, false>), grid, dim3(64 * WM * WP), lds, s, p, t);
    return hipGetLastError();
}

template <int CKB>
hipError_t launchx_cfg(int i, const ConvParams &p, const TileX &t, bool rt, hipStream_t s) {
    switch (i) {
    case 0: return launchx_inst<1, 2, 2, 2, CKB>(p, t, rt, s);
    case 1: return launchx_inst<2, 1, 2, 2, CKB>(p, t, rt, s);
    case 2: return launchx_inst<1, 1, 2, 2, CKB>(p, t, rt, s);
    case 3: return launchx_inst<1, 2, 1, 4, CKB>(p, t, rt, s);
    case 4: return launchx_inst<1, 1, 1, 4, CKB>(p, t, rt, s);
    case 5: return launchx_inst<1, 1, 1, 2, CKB>(p, t, rt, s);
    case 6: return launchx_inst<1, 1, 1, 1, CKB>(p, t, rt, s);
    }
    return hipErrorNotSupported;
}

}  // namespace

bool plan_wino(const ConvParams &p, const PackGeom &g, bool must_fill, WinoPlan *out) {
    if (!p.wx || !g.wino_bytes || p.in_bf16 || p.KH != 3 || p.KW != 3 || p.stride != 1 || p.pad != 1) return false;
    static const char *force = std::getenv("GSPC_TILEX");   // tuning aid: configuration index
    const int forced = force ? std::atoi(force) : tuned_config(p, 'x');
    const int ckb = g.CPG % 8 == 0 ? 2 : 1;
    // Measured order of preference: as many filters per block as the group has (the V transform of
    // a tile is repeated by every filter block), then the smaller tile count (more blocks in
    // flight per compute unit, whose transform and multiply phases overlap).
    static const int order_default[kNumCfgX] = {1, 2, 0, 4, 5, 3, 6};
    // A plane of 33..64 tiles (14x14 pixels) is one block of the 64-tile shape but two ragged ones of the
    // 32-tile shape: the larger shape first (offline tuner: 33.7 -> 25.2 us on the 256-channel g = 8 layer).
    static const int order_mid[kNumCfgX] = {1, 0, 2, 4, 5, 3, 6};
    const int plane_tiles = ((p.H + 1) / 2) * ((p.W + 1) / 2);
    const int *order = plane_tiles > 32 && plane_tiles <= 64 ? order_mid : order_default;
    // (Eq. 2; below about 128 MMAC a layer sits on the launch floor of the direct kernels, which
    // Winograd's longer prologue and epilogue cannot reach)
    const double macs = (double)p.N * p.Cout * g.CPG * 9 * p.H * p.W;
    int best = -1, best_ckb = 0;
    long best_blocks = -1;
    bool filled = false;
    TileX bt{};
    for (int o = 0; o < kNumCfgX; ++o) {
        const int i = order[o];
        if (forced >= 0 && i != forced) continue;
        // shapes with fewer filters than the group has (up to 32) repeat the V transform of a tile for
        // every filter block and do not beat the direct kernels: only on request
        const int filters = 16 * kCfgX[i].MI * kCfgX[i].WM;
        if (must_fill && forced < 0 && filters < (g.KPG < 32 ? g.KPG : 32)) continue;
        TileX t;
        int k = ckb;
        // (the block count does not depend on the form; the staged tile's LDS does)
        bool rt = use_rt(kCfgX[i], 0);
        if (!planx_cfg(p, g, kCfgX[i], k, rt, &t)) {
            k = 1;
            if (ckb == 1 || !planx_cfg(p, g, kCfgX[i], k, rt, &t)) continue;
        }
        const long blocks = (long)t.row_blocks * t.img_blocks * t.oc_blocks * p.groups;
        if (rt && !use_rt(kCfgX[i], blocks)) {
            TileX t2;
            if (planx_cfg(p, g, kCfgX[i], k, false, &t2)) t = t2;
        }
        if (blocks > best_blocks) {
            best = i;
            best_ckb = k;
            best_blocks = blocks;
            bt = t;
        }
        // the first shape that gives every compute unit two blocks - or one, for short reductions with at
        // most two filter blocks (the offline tuner's picks among the 16x16-pixel layers at batch 64)
        // (planes of less than 64 pixels - 7x7: a quarter of the 2x2 output tiles' area lies outside the plane -
        // need four blocks per unit: at two the plain kernel's 32-filter shape is 14 % ahead, 512 channels at N = 64)
        const long fill = p.H * p.W < 64 ? 4 * kNumCU : 2 * kNumCU;
        if (blocks >= fill || (blocks >= kNumCU && t.oc_blocks <= 2 && t.cblks <= 16 && p.H * p.W >= 64)) {
            best = i;
            best_ckb = k;
            best_blocks = blocks;
            bt = t;
            filled = true;
            break;
        }
    }
    if (best < 0) return false;
    // With fewer blocks the direct kernels (which can split the reduction over waves) were faster in
    // every measured case: left to them unless Winograd is asked for explicitly.
    if (must_fill && forced < 0 && (!filled || macs < 128.0e6)) return false;
    out->inst = best;
    out->ckb = best_ckb;
    static_assert(sizeof(TileX) <= sizeof(out->data), "plan storage too small");
    std::memcpy(out->data, &bt, sizeof(bt));
    return true;
}

hipError_t launch_wino(const ConvParams &p, const WinoPlan &plan, hipStream_t s, const char **name) {
    TileX t;
    std::memcpy(&t, plan.data, sizeof(t));
    const CfgX &c = kCfgX[plan.inst];
    const bool rt = t.rt != 0;
    *name = intern_name("conv_wino<" + std::to_string(c.MI) + "," + std::to_string(c.NI) + "," + std::to_string(c.WM) +
                        "," + std::to_string(c.WP) + "," + std::to_string(plan.ckb) + "," + (rt ? "true" : "false") + ">");
    return plan.ckb == 2 ? launchx_cfg<2>(plan.inst, p, t, rt, s) : launchx_cfg<1>(plan.inst, p, t, rt, s);
}

}  // namespace gspc
