// bf16 grouped 3x3 convolution (stride 1, pad 1) for few channels per group, as a
// stream of row products on v_mfma_f32_16x16x32_bf16 with no LDS and no barriers.
//
// Layers with 2..16 channels per group are far below the bf16 ridge: what has to be
// fast is moving the input once and the output once.  The kernel therefore never
// rearranges the input.  For one input row ih, four input channels and a window of
// eight consecutive columns, the 16 bytes a lane loads from NCHW memory ARE its B
// operand: reduction slot (channel c, column iw) with the column innermost.  The
// kernel taps along the row are folded into the A operand instead: a banded
// (Toeplitz) matrix T[(filter f, column ow)][(c, iw)] = w[f][c][kh][iw - ow + 1],
// built once by gspc_pack_weights for each kernel row kh.  A window starts at column
// 4n - 2 and yields the output columns 4n .. 4n + 3, so the product of one
// instruction is 4 filters x 4 columns x 16 windows, and the accumulator of a lane
// (rows 4*(l/16) .. +3 of the product) is four consecutive output columns of one
// filter: one 16-byte store, 256 contiguous bytes per filter row over 16 lanes.
// Five eighths of the multiplications hit the zeros of the band; the matrix cores are
// otherwise idle in these layers (Section IV-B of arXiv 2006.09791: the fewer MACs a
// grouped layer has, the more its time is memory), so that is the cheap resource.
//
// A wave owns (image set, merged group, filter block, row band): it keeps the banded
// operands of its filters in registers for the whole launch, walks down the input rows
// with the loads a few rows ahead, and feeds each row to the three output rows it
// belongs to (kh = 0, 1, 2); four accumulator sets rotate so that a set is not written
// again until a full step after its row was stored.  Groups with fewer than 8 channels are merged by
// the pack step into block-diagonal groups of 8 (zero weights between channels and
// filters of different groups, Section II / Fig. 2), which costs only idle
// multiplications.
#include <cstdlib>
#include <cstring>

#include "conv_common.h"

namespace gspc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct TileR {
    int WPR, wpr_shift, SPW;   // window slots per row (power of two, 16 / WPR images per wave)
    int nwin;                  // windows per row = W / 4
    int bands, TH;             // row bands per plane, output rows per band
    int gt, CPGt, KPGt;        // merged groups, channels and filters per merged group
    int FS, FQT;               // filter blocks per merged group, filter quads per merged group
    unsigned items;            // wave work items
    unsigned m_FS, m_bands, m_gt;
    unsigned x_bytes, y_bytes, w_bytes;
};
static_assert(sizeof(TileR) <= sizeof(((RowB16Plan *)0)->data), "plan storage too small");

// CQ: channel quads per merged group, FQ: filter quads per wave, D: input rows in flight,
// EPI: with the residual / ReLU epilogue (its residual rows travel through registers of their own).
template <int CQ, int FQ, int D, int OCC, bool EPI>
__global__ __launch_bounds__(256, OCC) void conv_row16b(ConvParams p, TileR t) {
    static_assert(D % 4 == 0, "the accumulator rotation has period 4");
    const int lane = threadIdx.x & 63;
    const unsigned wi = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wi >= t.items) return;   // uniform over the wave; the kernel has no barriers
    const unsigned q1 = fast_div(wi, t.m_FS);
    const int fs = wi - q1 * t.FS;
    const unsigned q2 = fast_div(q1, t.m_bands);
    const int band = q1 - q2 * t.bands;
    const unsigned is = fast_div(q2, t.m_gt);
    const int j = q2 - is * t.gt;
    const int oh0 = band * t.TH;
    const int oh1 = oh0 + t.TH < p.H ? oh0 + t.TH : p.H;
    const int nsteps = oh1 - oh0 + 2;   // input rows oh0 - 1 .. oh1

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wr, t.w_bytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);

    // Lane l: window slot l % 16 (image sub = slot / WPR of the wave's set, window slot % WPR),
    // channel (loads) or filter (stores) l / 16 of the current quad.
    const int nslot = lane & 15, cl = lane >> 4;
    const int win = nslot & (t.WPR - 1);
    const unsigned img = is * t.SPW + (nslot >> t.wpr_shift);
    const bool live = win < t.nwin && img < (unsigned)p.N;
    // The first window of a row would start two columns before the row and the last one end
    // two columns behind it: they load the row's first / last eight columns instead (always
    // inside the tensor) and shift the dwords into place, zeros entering at the border.
    const bool is_first = win == 0, is_last = win == t.nwin - 1;
    const unsigned HW = p.H * p.W;
    const unsigned colb = is_first ? 0u : is_last ? (p.W - 8) * 2u : (win * 4 - 2) * 2u;
    const unsigned xv = live ? ((img * p.Cin + j * t.CPGt + cl) * HW) * 2u + colb : kOob;
    const unsigned yv = live ? ((img * p.Cout + j * t.KPGt + fs * FQ * 4 + cl) * HW) * 4u + win * 16u : kOob;

    // Banded operands of this wave's filters: [filter quad][kh][channel quad], 16 bytes per lane.
    bf16x8 A[FQ][3][CQ];
    {
        const unsigned abase = ((unsigned)(j * t.FQT + fs * FQ) * 3 * CQ * 64 + lane) * 16u;
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int cq = 0; cq < CQ; ++cq)
                    A[fq][kh][cq] = __builtin_bit_cast(
                        bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rw, abase, ((fq * 3 + kh) * CQ + cq) * 1024, 0));
        // The operands arrive before the first input row is requested: otherwise the loop's first
        // wait, which must cover every way into the loop, would also cover these loads and drain
        // the input rows in flight once per trip.
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int cq = 0; cq < CQ; ++cq) asm volatile("" : "+v"(A[fq][kh][cq]));
        __builtin_amdgcn_sched_barrier(0);
    }

    // Every step issues the same vector-memory instructions in the same order - CQ input loads,
    // FQ residual loads (EPI only), FQ stores - and the prologue issues that pattern too (with out-of-range
    // offsets, which load zeros and store nothing), so that the wait counts the compiler derives are
    // the same on every path into the loop and a step waits for its own row only, never for the
    // rows requested behind it.
    u32x4 B[D][CQ];
    f32x4 R[2][EPI ? FQ : 1];
    f32x4 acc[4][FQ];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq) acc[s][fq] = f32x4{0.f, 0.f, 0.f, 0.f};
    const unsigned rv_off = p.res ? yv : kOob;

    // Input row of step `step` (row oh0 - 1 + step); rows outside the image and steps past the
    // band read zeros.
    auto issue = [&](int step, u32x4(&dst)[CQ]) {
        const int ih = oh0 - 1 + step;
        const bool ok = step < nsteps && (unsigned)ih < (unsigned)p.H;
        const unsigned vo = ok ? xv : kOob;
        const unsigned so = ok ? (unsigned)ih * p.W * 2u : 0u;
#pragma unroll
        for (int cq = 0; cq < CQ; ++cq) dst[cq] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo, so + cq * 4 * HW * 2, 0);
    };
    // Residual of the output row that is stored at step `step` (relative row step - 2), zeros
    // without a residual.
    auto issue_res = [&](int step, f32x4(&dst)[EPI ? FQ : 1]) {
        if (!EPI) return;
        const bool ok = step >= 2 && step < nsteps;
        const unsigned vo = ok ? rv_off : kOob;
        const unsigned so = ok ? (unsigned)(oh0 + step - 2) * p.W * 4u : 0u;
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
            dst[fq] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, vo, so + fq * 4 * HW * 4, 0));
    };
    auto store_row = [&](int step, const f32x4(&src)[FQ]) {
        const bool ok = step >= 2 && step < nsteps;
        const unsigned vo = ok ? yv : kOob;
        const unsigned so = ok ? (unsigned)(oh0 + step - 2) * p.W * 4u : 0u;
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, src[fq]), ry, vo, so + fq * 4 * HW * 4, 0);
    };

#pragma unroll
    for (int u = 0; u < D - 1; ++u) {
        issue(u, B[u]);
        issue_res(u - (D - 1) + 1, R[(u + 1) & 1]);   // nothing to fetch yet: keeps the pattern
        store_row(-1, acc[0]);
    }

#pragma clang loop unroll(disable)
    for (int t0 = 0; t0 < nsteps; t0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int step = t0 + u;
            // (steps past the band, up to D - 1 of them, run on zeros and store nothing: an exit from
            // the middle of the trip would give the loop head a path with fewer requests in flight)
            // the steps stay in program order: requests first, stores last
            __builtin_amdgcn_sched_barrier(0);
            issue(step + D - 1, B[(u + D - 1) % D]);
            issue_res(step + 1, R[(u + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            // Output row `step` (relative to oh0) starts at this step (kh = 0), row step - 1
            // takes its middle kernel row and row step - 2 its last one and is complete.
            const int s_new = u % 4, s_mid = (u + 3) % 4, s_end = (u + 2) % 4;
#pragma unroll
            for (int cq = 0; cq < CQ; ++cq) {
                const u32x4 raw = B[u % D][cq];
                u32x4 b;
                b.x = is_first ? 0u : is_last ? raw.y : raw.x;
                b.y = is_first ? raw.x : is_last ? raw.z : raw.y;
                b.z = is_first ? raw.y : is_last ? raw.w : raw.z;
                b.w = is_first ? raw.z : is_last ? 0u : raw.w;
                const bf16x8 bv = __builtin_bit_cast(bf16x8, b);
#pragma unroll
                for (int fq = 0; fq < FQ; ++fq) {
                    acc[s_new][fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        A[fq][0][cq], bv, cq == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[s_new][fq], 0, 0, 0);
                    acc[s_mid][fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[fq][1][cq], bv, acc[s_mid][fq], 0, 0, 0);
                    acc[s_end][fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[fq][2][cq], bv, acc[s_end][fq], 0, 0, 0);
                }
            }
            if (EPI) {
#pragma unroll
                for (int fq = 0; fq < FQ; ++fq) acc[s_end][fq] += R[u & 1][fq];
            }
            if (EPI && p.relu) {
#pragma unroll
                for (int fq = 0; fq < FQ; ++fq)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[s_end][fq][r] = fmaxf(acc[s_end][fq][r], 0.f);
            }
            __builtin_amdgcn_sched_barrier(0);
            store_row(step, acc[s_end]);
        }
    }
}

// 4x4 transpose between four registers and the four 16-lane rows of a wavefront:
// afterwards register i, row r holds what register r, row i held.  v_permlane16_swap
// exchanges the odd rows of its first operand with the even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second.
__device__ __forceinline__ void transpose_rows(unsigned &a0, unsigned &a1, unsigned &a2, unsigned &a3) {
    const auto p01 = __builtin_amdgcn_permlane16_swap(a0, a1, false, false);
    const auto p23 = __builtin_amdgcn_permlane16_swap(a2, a3, false, false);
    const auto q02 = __builtin_amdgcn_permlane32_swap(p01[0], p23[0], false, false);
    const auto q13 = __builtin_amdgcn_permlane32_swap(p01[1], p23[1], false, false);
    a0 = q02[0];
    a2 = q02[1];
    a1 = q13[0];
    a3 = q13[1];
}
template <typename V> __device__ __forceinline__ void transpose_rows4(V &a0, V &a1, V &a2, V &a3) {
    u32x4 b0 = __builtin_bit_cast(u32x4, a0), b1 = __builtin_bit_cast(u32x4, a1), b2 = __builtin_bit_cast(u32x4, a2),
          b3 = __builtin_bit_cast(u32x4, a3);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        unsigned c0 = b0[e], c1 = b1[e], c2 = b2[e], c3 = b3[e];
        transpose_rows(c0, c1, c2, c3);
        b0[e] = c0;
        b1[e] = c1;
        b2[e] = c2;
        b3[e] = c3;
    }
    a0 = __builtin_bit_cast(V, b0);
    a1 = __builtin_bit_cast(V, b1);
    a2 = __builtin_bit_cast(V, b2);
    a3 = __builtin_bit_cast(V, b3);
}

// The same row products with memory touched four rows at a time.  conv_row16b asks for one
// row of four channels per load and writes one row of four filters per store: pieces of 2*W
// and 4*W bytes, each in a different plane.  Here a load instruction fetches four consecutive
// rows of ONE channel (lane group = row: 8*W contiguous bytes) and a store instruction writes
// four consecutive rows of ONE filter (16*W contiguous bytes); a 4x4 exchange between
// registers and lane groups (transpose_rows) turns four such loads into the four channels x
// one row operands the products want, and four finished output rows back into the store
// layout.  A trip of the loop is eight steps: two input quads, two output quads, eight
// accumulator sets (output row r lives in set r % 8).
template <int CQ, int FQ, bool EPI>
__global__ __launch_bounds__(256, 2) void conv_row16q(ConvParams p, TileR t) {
    const int lane = threadIdx.x & 63;
    const unsigned wi = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wi >= t.items) return;   // uniform over the wave; the kernel has no barriers
    const unsigned q1 = fast_div(wi, t.m_FS);
    const int fs = wi - q1 * t.FS;
    const unsigned q2 = fast_div(q1, t.m_bands);
    const int band = q1 - q2 * t.bands;
    const unsigned is = fast_div(q2, t.m_gt);
    const int j = q2 - is * t.gt;
    const int oh0 = band * t.TH;
    const int oh1 = oh0 + t.TH < p.H ? oh0 + t.TH : p.H;
    const int rows = oh1 - oh0, nsteps = rows + 2;   // input rows oh0 - 1 .. oh1
    const int ntrips = (4 * ((rows + 3) / 4) + 2 + 7) / 8;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, t.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wr, t.w_bytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.y, t.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res ? p.res : p.y, t.y_bytes);

    // Lane l: window slot l % 16 as in conv_row16b; lane group l / 16 is a row of the quad in
    // memory instructions and a channel / filter of the quad in the products.
    const int nslot = lane & 15, g4 = lane >> 4;
    const int win = nslot & (t.WPR - 1);
    const unsigned img = is * t.SPW + (nslot >> t.wpr_shift);
    const bool live = win < t.nwin && img < (unsigned)p.N;
    const bool is_first = win == 0, is_last = win == t.nwin - 1;
    const unsigned HW = p.H * p.W;
    const unsigned colb = is_first ? 0u : is_last ? (p.W - 8) * 2u : (win * 4 - 2) * 2u;
    const unsigned xb = ((img * p.Cin + j * t.CPGt) * HW) * 2u + colb;
    const unsigned yb = ((img * p.Cout + j * t.KPGt + fs * FQ * 4) * HW) * 4u + win * 16u;

    bf16x8 A[FQ][3][CQ];
    {
        const unsigned abase = ((unsigned)(j * t.FQT + fs * FQ) * 3 * CQ * 64 + lane) * 16u;
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int cq = 0; cq < CQ; ++cq)
                    A[fq][kh][cq] = __builtin_bit_cast(
                        bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rw, abase, ((fq * 3 + kh) * CQ + cq) * 1024, 0));
        __builtin_amdgcn_sched_barrier(0);   // see conv_row16b: the operands arrive before the first request
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int cq = 0; cq < CQ; ++cq) asm volatile("" : "+v"(A[fq][kh][cq]));
        __builtin_amdgcn_sched_barrier(0);
    }

    u32x4 L[2][4 * CQ];          // two input quads: [channel] with lane group = row until transposed
    f32x4 R[EPI ? 4 * FQ : 1];   // residual of the output quad stored next, in store layout
    f32x4 acc[8][FQ];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq) acc[s][fq] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Input quad q: rows oh0 - 1 + 4q .. + 3, every channel of the merged group.
    auto issue_quad = [&](int q, u32x4(&dst)[4 * CQ]) {
        const int st = 4 * q + g4, row = oh0 - 1 + st;
        const bool ok = live && st < nsteps && (unsigned)row < (unsigned)p.H;
        const unsigned vo = ok ? xb + (unsigned)row * p.W * 2u : kOob;
#pragma unroll
        for (int c = 0; c < 4 * CQ; ++c) dst[c] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo, c * HW * 2, 0);
    };
    // Output quad m: rows oh0 + 4m .. + 3 of this wave's filters (m = -1: nothing).
    auto quad_offset = [&](int m) -> unsigned {
        const int orow = 4 * m + g4;
        return live && m >= 0 && orow < rows ? yb + (unsigned)(oh0 + orow) * p.W * 4u : kOob;
    };
    auto issue_res = [&](int m) {
        if (!EPI) return;
        const unsigned vo = p.res ? quad_offset(m) : kOob;
#pragma unroll
        for (int k = 0; k < 4 * FQ; ++k)
            R[EPI ? k : 0] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, vo, k * HW * 4, 0));
    };
    auto store_quad = [&](int m, f32x4(&a0)[FQ], f32x4(&a1)[FQ], f32x4(&a2)[FQ], f32x4(&a3)[FQ]) {
        const unsigned vo = quad_offset(m);
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq) {
            transpose_rows4(a0[fq], a1[fq], a2[fq], a3[fq]);   // register i: filter 4*fq + i, lane group = row
            f32x4 *o[4] = {&a0[fq], &a1[fq], &a2[fq], &a3[fq]};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (EPI) *o[i] += R[EPI ? fq * 4 + i : 0];
                if (EPI && p.relu) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) (*o[i])[r] = fmaxf((*o[i])[r], 0.f);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int fq = 0; fq < FQ; ++fq) {
            const f32x4 *o[4] = {&a0[fq], &a1[fq], &a2[fq], &a3[fq]};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, *o[i]), ry, vo, (fq * 4 + i) * HW * 4, 0);
        }
    };
    // One step: the row in `raw` (lane group = channel) goes to the output row that starts here
    // (set s_new, kh = 0), the one in its middle (kh = 1) and the one it completes (kh = 2).
    auto step_fn = [&](const u32x4(&rowops)[4 * CQ], int r, f32x4(&a_new)[FQ], f32x4(&a_mid)[FQ], f32x4(&a_end)[FQ]) {
#pragma unroll
        for (int cq = 0; cq < CQ; ++cq) {
            const u32x4 raw = rowops[4 * cq + r];
            u32x4 b;
            b.x = is_first ? 0u : is_last ? raw.y : raw.x;
            b.y = is_first ? raw.x : is_last ? raw.z : raw.y;
            b.z = is_first ? raw.y : is_last ? raw.w : raw.z;
            b.w = is_first ? raw.z : is_last ? 0u : raw.w;
            const bf16x8 bv = __builtin_bit_cast(bf16x8, b);
#pragma unroll
            for (int fq = 0; fq < FQ; ++fq) {
                a_new[fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[fq][0][cq], bv,
                                                                    cq == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : a_new[fq], 0, 0, 0);
                a_mid[fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[fq][1][cq], bv, a_mid[fq], 0, 0, 0);
                a_end[fq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[fq][2][cq], bv, a_end[fq], 0, 0, 0);
            }
        }
    };

    // Prologue in the shape of half a trip (requests, stores, residual requests), so that the
    // loop's first wait sees the same queue on its way in as on its way round.
    issue_quad(0, L[0]);
    store_quad(-1, acc[4], acc[5], acc[6], acc[7]);
    issue_res(-1);

#pragma clang loop unroll(disable)
    for (int T = 0; T < ntrips; ++T) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            __builtin_amdgcn_sched_barrier(0);
            issue_quad(2 * T + 1 + h, L[1 - h]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cq = 0; cq < CQ; ++cq)
                transpose_rows4(L[h][4 * cq], L[h][4 * cq + 1], L[h][4 * cq + 2], L[h][4 * cq + 3]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int u = 4 * h + r;
                step_fn(L[h], r, acc[u], acc[(u + 7) % 8], acc[(u + 6) % 8]);
                if (r == 1) {
                    // rows 4 * (2T - 1 + h) .. + 3 are complete: sets 4..7 in the first half, 0..3 in the second
                    __builtin_amdgcn_sched_barrier(0);
                    store_quad(2 * T - 1 + h, acc[4 - 4 * h], acc[5 - 4 * h], acc[6 - 4 * h], acc[7 - 4 * h]);
                    issue_res(2 * T + h);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
namespace {

struct CfgR {
    int CQ, FQ, D, OCC;
};
// filter quads per wave are limited by the registers the banded operands take (12 * CQ * FQ)
// D = 0: the four-rows-at-a-time form (conv_row16q)
const CfgR kCfgR[] = {{2, 2, 4, 4}, {2, 4, 4, 2}, {2, 1, 4, 4}, {4, 2, 4, 2}, {4, 1, 4, 2}, {2, 2, 8, 2},
                      {2, 2, 0, 2}, {2, 1, 0, 2}, {4, 1, 0, 2}};
constexpr int kNumCfgR = sizeof(kCfgR) / sizeof(kCfgR[0]);

template <int CQ, int FQ, int D, int OCC>
hipError_t launchR(const ConvParams &p, const TileR &t, hipStream_t s) {
    if (p.res || p.relu)
        hipLaunchKernelGGL((conv_row16b<CQ, FQ, D, 2, true>), dim3((t.items + 3) / 4), dim3(256), 0, s, p, t);
    else
        hipLaunchKernelGGL((conv_row16b<CQ, FQ, D, OCC, false>), dim3((t.items + 3) / 4), dim3(256), 0, s, p, t);
    return hipGetLastError();
}

template <int CQ, int FQ>
hipError_t launchQ(const ConvParams &p, const TileR &t, hipStream_t s) {
    if (p.res || p.relu)
        hipLaunchKernelGGL((conv_row16q<CQ, FQ, true>), dim3((t.items + 3) / 4), dim3(256), 0, s, p, t);
    else
        hipLaunchKernelGGL((conv_row16q<CQ, FQ, false>), dim3((t.items + 3) / 4), dim3(256), 0, s, p, t);
    return hipGetLastError();
}

}  // namespace

bool plan_row_bf16(const ConvParams &p, const PackGeom &g, RowB16Plan *out) {
    if (!p.in_bf16 || !p.wr || !g.row_bytes || p.KH != 3 || p.KW != 3 || p.stride != 1 || p.pad != 1) return false;
    if (p.W % 4 || p.W < 8 || p.W > 64) return false;
    static const char *off = std::getenv("GSPC_ROWB");   // "0" turns the kernel off (measurement aid)
    if (off && off[0] == '0') return false;
    const int CQ = g.CPGt / 4, FQT = g.KPGt / 4;
    static const char *force = std::getenv("GSPC_TILER");
    int inst = -1;
    const int forced = force ? std::atoi(force) : tuned_config(p, 'r');
    // preference: four rows at a time (6, 7), then one row at a time; with 16 channels per group the
    // one-row form with two filter quads per wave comes first (the four-row form has registers for
    // one quad only and then four waves read the same input: 31 against 41 us on 128 -> 128, 28x28,
    // g = 8 at batch 256); 5 (seven rows in flight) only on request
    static const int order[] = {6, 7, 3, 8, 0, 1, 2, 4, 5};
    for (int k = 0; k < kNumCfgR && inst < 0; ++k) {
        const int i = order[k];
        if (forced >= 0 && forced != i) continue;
        if (forced < 0 && i == 5) continue;
        if (kCfgR[i].CQ == CQ && FQT % kCfgR[i].FQ == 0) inst = i;
    }
    if (inst < 0) return false;
    const CfgR &c = kCfgR[inst];
    TileR t{};
    t.nwin = p.W / 4;
    t.WPR = t.nwin > 8 ? 16 : t.nwin > 4 ? 8 : t.nwin > 2 ? 4 : 2;
    t.wpr_shift = t.WPR == 16 ? 4 : t.WPR == 8 ? 3 : t.WPR == 4 ? 2 : 1;
    t.SPW = 16 / t.WPR;
    t.gt = g.gt;
    t.CPGt = g.CPGt;
    t.KPGt = g.KPGt;
    t.FQT = FQT;
    t.FS = FQT / c.FQ;
    // Row bands: enough wave items for two per SIMD, bands of at least 8 rows (a band re-reads
    // two rows of its neighbours and reloads the banded operands).
    const long per_band = (long)((p.N + t.SPW - 1) / t.SPW) * t.gt * t.FS;
    static const char *fb = std::getenv("GSPC_ROWB_BANDS");
    int bands = 1;
    if (fb) bands = std::atoi(fb);
    else
        while (per_band * bands < 2L * 4 * kNumCU && p.H / (bands * 2) >= 8) bands *= 2;
    if (bands < 1) bands = 1;
    if (bands > p.H) bands = p.H;
    t.TH = (p.H + bands - 1) / bands;
    t.bands = (p.H + t.TH - 1) / t.TH;
    const long items = per_band * t.bands;
    if (items >= 2147483647L / 4) return false;
    t.items = (unsigned)items;
    t.m_FS = div_magic(t.FS);
    t.m_bands = div_magic(t.bands);
    t.m_gt = div_magic(t.gt);
    if ((double)items * t.FS >= 4.0e9 || (double)items * t.bands >= 4.0e9 || (double)items * t.gt >= 4.0e9) return false;
    const double xb = (double)p.N * p.Cin * p.H * p.W * 2, yb = (double)p.N * p.Cout * p.H * p.W * 4;
    if (xb >= (double)kOob || yb >= (double)kOob || (double)g.row_bytes >= (double)kOob) return false;
    t.x_bytes = (unsigned)xb;
    t.y_bytes = (unsigned)yb;
    t.w_bytes = (unsigned)g.row_bytes;
    out->inst = inst;
    std::memcpy(out->data, &t, sizeof(t));
    return true;
}

hipError_t launch_row_bf16(const ConvParams &p, const RowB16Plan &plan, hipStream_t s, const char **name) {
    TileR t;
    std::memcpy(&t, plan.data, sizeof(t));
    const CfgR &c = kCfgR[plan.inst];
    *name = c.D == 0 ? intern_name("conv_row16q<" + std::to_string(c.CQ) + "," + std::to_string(c.FQ) + ">/" +
                                   std::to_string(t.bands) + "b")
                     : intern_name("conv_row16b<" + std::to_string(c.CQ) + "," + std::to_string(c.FQ) + "," +
                                   std::to_string(c.D) + "," + std::to_string(c.OCC) + ">/" + std::to_string(t.bands) + "b");
    switch (plan.inst) {
    case 0: return launchR<2, 2, 4, 4>(p, t, s);
    case 1: return launchR<2, 4, 4, 2>(p, t, s);
    case 2: return launchR<2, 1, 4, 4>(p, t, s);
    case 3: return launchR<4, 2, 4, 2>(p, t, s);
    case 4: return launchR<4, 1, 4, 2>(p, t, s);
    case 5: return launchR<2, 2, 8, 2>(p, t, s);
    case 6: return launchQ<2, 2>(p, t, s);
    case 7: return launchQ<2, 1>(p, t, s);
    case 8: return launchQ<4, 1>(p, t, s);
    }
    return hipErrorNotSupported;
}

}  // namespace gspc
