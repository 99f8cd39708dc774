// Internal declarations shared by the host API and the HIP kernels of libgspc.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gspc.h"

namespace gspc {

constexpr uint32_t kPackedMagic = 0x47535043u;  // "GSPC"
constexpr int kVersion = 1;

// Matrix-core tile variants of the implicit-GEMM kernels.  The value is the
// number of output channels one MFMA instruction covers.
enum MfmaVariant { kMfmaNone = 0, kMfma4 = 4, kMfma16 = 16 };

// Reduction slots one MFMA instruction consumes per variant (its K extent):
// v_mfma_f32_16x16x4_f32 contracts 4, v_mfma_f32_4x4x1_16b_f32 contracts 1.
__host__ __device__ constexpr int mfma_ksub(int variant) { return variant == 16 ? 4 : 1; }

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// Geometry of the two sections of a packed-weight buffer.
//   direct section : fp32 [g][Kred][KPGd], Kred = CPG*KH*KW ordered (c, kh, kw),
//                    KPGd = KPG rounded up to a multiple of 4, zero padded.
//   mfma section   : (KPG >= 5) fp32 [g][ksteps][ceil(KPG/16)][64], the A operand
//                    of one v_mfma_f32_16x16x4_f32 per (k-step, filter tile,
//                    lane); k-steps ordered (c / 4, kh, kw) with CPG zero-padded
//                    to a multiple of 4; lane l holds filter l % 16 of its tile
//                    at reduction slot c = cblk*4 + l / 16; filters past KPG in
//                    the last tile are zero.
//   variant 16 = KPG a multiple of 16 (no padding filters).  Variant 4 (KPG a
//   multiple of 4 but not of 16) can also run the 4x4x1 MFMA kernel, which
//   reads its operands from the direct section.
struct PackGeom {
    int CPG, KPG, Kred, KPGd;
    int variant;   // MfmaVariant
    int ksub, CPGp, ksteps, mtiles;
    size_t direct_bytes, mfma_bytes, mfma_offset, total_bytes;
    // bf16 matrix-core section (GSPC_BF16 handles, 3x3, KPG % 4 == 0, CPG % 8 == 0):
    // bf16 [g][chunk][k-step][ceil(KPG/16)][64 lanes][8], the A operand of one
    // v_mfma_f32_16x16x32_bf16 per (chunk, k-step, filter tile, lane).  A chunk
    // covers ckb input channels; its reduction is cut into units of 8 channels
    // at one tap, unit u = tap*(ckb/8) + channel block; lane l of k-step s holds
    // unit 4*s + l/16 of filter l%16 (zeros past the last unit).
    // Layers with fewer than 8 channels per group reach this section by merging mb
    // consecutive groups into one block-diagonal group (gb = groups / mb groups of CPGb = mb * CPG
    // channels and KPGb = mb * KPG filters; weights between channels and filters of different
    // original groups are zero, which is what Section II's definition of G(g) says they are).
    int ckb, ks_b, nchunks_b, mtiles_b;
    int mb, gb, CPGb, KPGb;
    size_t bf16_bytes, bf16_offset;
    // Row-product section (GSPC_BF16 handles, 3x3, merged groups of CPGt in {8, 16} channels and
    // KPGt % 4 == 0 filters, mt original groups each): bf16 [gt][KPGt/4][3 kh][CPGt/4][64 lanes][8],
    // the banded A operand of one v_mfma_f32_16x16x32_bf16: lane l, element e holds
    // w[filter 4*fq + (l%16)/4][channel 4*cq + l/16][kh][kw = e - (l%16)%4 - 1], zero outside 0..2
    // (rowb_kernels.hip).
    int mt, gt, CPGt, KPGt;
    size_t row_bytes, row_offset;
    // Winograd F(2x2, 3x3) section (GSPC_F32 handles, 3x3, KPG >= 12, CPG % 4 == 0,
    // CPG >= 8): fp32 U = G g G^T as [g][CPG/4][ceil(KPG/16)][4][64 lanes][4] (filters
    // past KPG in the last tile are zero); lane l holds
    // filter l % 16 of its tile at channel 4*cblk + l / 16, and its four values in
    // quad q are the transformed-domain positions 4*q .. 4*q + 3 (position = 4*xi + nu).
    size_t wino_bytes, wino_offset;
    // Merged direct sections (3x3, fewer than 4 or 8 channels or filters per group, not depthwise):
    // the layer seen as groups / m block-diagonal groups of m * CPG channels and m * KPG filters, in
    // the direct section's layout [groups/m][m*CPG*9][round_up(m*KPG, 4)].  md[0] reaches at least 4
    // channels and filters per group (the smallest the 4x4x1 matrix-core kernel takes), md[1] at
    // least 8 (what the depth-fused runs multiply best); m = 0: none.
    // Quad-k section (GSPC_F32 handles; conv_gpw's operands): fp32 [qk_groups][k-steps / 4][qk_KPG / 16]
    // [64 lanes][4]: lane l, element e holds the weight of filter 16*tile + l % 16 at k-step 4*quad + e,
    // k-steps ordered (c / 4, kh, kw) with channel 4 * (k-step / taps) + l / 16.  For 3x3 layers with
    // Cin = Cout in {32, 64, 128}: qk_m original groups merged until a group has a multiple of 16
    // filters (block-diagonal); for ungrouped 1x1 layers with Cin in {32, 64, 128} and Cout % 16 == 0:
    // the layer itself.
    int qk_m, qk_groups, qk_CPG, qk_KPG;
    size_t qk_bytes, qk_offset;
    struct MergedDirect {
        int m, groups, CPG, KPG, KPGd;
        size_t bytes, offset;
    } md[2];
};
// Geometry of the layer as merged section `which` sees it (sections other than direct: none).
PackGeom merged_geom(const PackGeom &g, int which, int KH, int KW);

PackGeom make_pack_geom(int Cin, int Cout, int KH, int KW, int groups, int dtype);

}  // namespace gspc

struct gspc_packed {
    uint32_t magic;
    int version;
    int Cin, Cout, KH, KW, groups, dtype;
    gspc::PackGeom geom;
    void *dev;
    size_t bytes;
};

namespace gspc {

// Everything a convolution kernel needs, passed by value.
struct ConvParams {
    const void *x;      // [N][Cin][H][W], fp32 or bf16
    const float *wd;    // direct section
    const float *wm;    // mfma section (nullptr if none)
    const void *wb;     // bf16 mfma section (nullptr if none)
    const float *wx;    // Winograd section (nullptr if none)
    const void *wr;     // bf16 row-product section (nullptr if none)
    float *y;           // [N][Cout][Hout][Wout]
    const float *res;   // optional residual, same shape as y
    int N, Cin, H, W, Cout, KH, KW, stride, pad, groups;
    int H0, W0;         // plane size as the caller gave it (H, W may be a re-pitched view of a 1x1 layer's planes)
    int CPG, KPG, Hout, Wout, KPGd;
    int relu;
    int in_bf16;
};

// Each launcher returns hipSuccess / a HIP error, or hipErrorNotSupported when
// the kernel family has no instance for this layer.  *name receives a static
// string naming the kernel that ran.
hipError_t launch_direct(const ConvParams &p, hipStream_t s, const char **name);
hipError_t launch_mfma(const ConvParams &p, const PackGeom &g, hipStream_t s,
                       const char **name);
bool mfma_supported(const ConvParams &p, const PackGeom &g);

// Offline tile table (GSPC_TUNE_FILE, see tune_table.cpp): family letter forced for this layer
// ('\0' = none) and the configuration index forced within a family (-1 = none).
char tuned_family(const ConvParams &p);
int tuned_config(const ConvParams &p, char family);

// bf16 16x16x32 MFMA kernel; plan is opaque to the caller.
struct MfmaB16Plan {
    int inst;
    int data[48];
};
bool plan_mfma_bf16(const ConvParams &p, const PackGeom &g, MfmaB16Plan *out);
hipError_t launch_mfma_bf16(const ConvParams &p, const PackGeom &g, const MfmaB16Plan &plan, hipStream_t s,
                            const char **name);

// bf16 row-product kernel for few channels per group (rowb_kernels.hip).
struct RowB16Plan {
    int inst;
    int data[32];
};
bool plan_row_bf16(const ConvParams &p, const PackGeom &g, RowB16Plan *out);
hipError_t launch_row_bf16(const ConvParams &p, const RowB16Plan &plan, hipStream_t s, const char **name);

// 16x16x4 MFMA kernel with the filter tile resident in LDS (3x3, fp32 input).
struct Mfma16wPlan {
    int inst, ckb;
    int data[48];
};
bool plan_mfma16w(const ConvParams &p, const PackGeom &g, Mfma16wPlan *out);
hipError_t launch_mfma16w(const ConvParams &p, const Mfma16wPlan &plan, hipStream_t s, const char **name);

// Winograd F(2x2, 3x3) on the 16x16x4 MFMA (wino_kernels.hip).  winograd_mode(): 0 = never,
// 1 = wherever a plan exists, -1 (default) = where the launch fills the chip (must_fill).
// Family 'x' of the tile table asks for it per layer.
struct WinoPlan {
    int inst, ckb;
    int data[48];
};
bool plan_wino(const ConvParams &p, const PackGeom &g, bool must_fill, WinoPlan *out);
hipError_t launch_wino(const ConvParams &p, const WinoPlan &plan, hipStream_t s, const char **name);
int winograd_mode();

// 4x4x1 MFMA kernel (weights held in registers); plan is opaque to the caller.
struct Mfma4Plan {
    int inst;        // index of the kernel instance
    int data[40];    // tile geometry, see mfma4_kernels.hip
};
bool plan_mfma4(const ConvParams &p, const PackGeom &g, Mfma4Plan *out);
hipError_t launch_mfma4(const ConvParams &p, const Mfma4Plan &plan, hipStream_t s, const char **name);

// Depthwise 3x3 on whole small planes (dw_kernels.hip); plan is opaque to the caller.
struct DwPlan {
    int data[24];
};
bool plan_dw_planes(const ConvParams &p, DwPlan *out);
hipError_t launch_dw_planes(const ConvParams &p, const DwPlan &plan, hipStream_t s, const char **name);

// Fused run of consecutive grouped 3x3 layers (fused_kernels.hip).
constexpr int kFuseMaxLayers = 16, kFuseMaxTiles = 3, kFuseMaxInputs = 3;
struct FusedLayer {
    const float *w;   // direct section of the layer's packed weights
    float *y;         // HBM destination, or nullptr if a later layer of the run overwrites the buffer
    short src, res, dst, relu;   // LDS tile indices (res, dst: -1 = none)
};
struct FusedRun {
    int N, C, H, W, groups, CPG, KPGd;
    int vec, XO, LW, PLANE, TILE, wfloats;   // tile geometry (floats); 16-byte global accesses allowed
    int nlayers, ninputs, ntiles;
    int rgroups, nitems;                     // groups of NI pixel runs per filter tile; wave items per layer
    unsigned m_groups, m_rgroups, m_hw, m_w, m_hwq, m_wq;
    const float *in_ptr[kFuseMaxInputs];
    int in_tile[kFuseMaxInputs];
    FusedLayer L[kFuseMaxLayers];
};
struct FusedPlan {
    int core;     // pixel runs per wave item (template argument of the kernel)
    int waves;    // waves per block (template argument of the kernel)
    size_t lds;
    FusedRun run;
};
// Number of leading layers of layers[first .. first+count) that one fused launch covers (0 = none).
int plan_fused_run(const gspc_layer_t *layers, int first, int count, void *const *bufs, FusedPlan *out);
hipError_t launch_fused_run(const FusedPlan &plan, hipStream_t s, const char **name);

// Depthwise 3x3 + pointwise 1x1 pair as one kernel; plan is opaque to the caller.
struct DwPwPlan {
    int inst, sd;
    alignas(8) char params[96];
    alignas(8) char tile[128];
};
// 2 if layers[first], layers[first + 1] run as one fused launch, else 0.
int plan_dwpw(const gspc_layer_t *layers, int first, int count, void *const *bufs, DwPwPlan *out);
hipError_t launch_dwpw(const DwPwPlan &plan, hipStream_t s, const char **name);

// Grouped 3x3 + pointwise 1x1 pair as one kernel (gpw_kernels.hip); plan is opaque to the caller.
struct GpwPlan {
    int ct, mta, kt, stride;
    alignas(8) char params[96];
    alignas(8) char tile[128];
};
// 2 if layers[first], layers[first + 1] run as one fused launch, else 0.
int plan_gpw(const gspc_layer_t *layers, int first, int count, void *const *bufs, GpwPlan *out);
hipError_t launch_gpw(const GpwPlan &plan, hipStream_t s, const char **name);
bool gpw_enabled();   // GSPC_GPW=1 in the environment, read at every call

hipError_t launch_pack_weights(const float *w, const gspc_packed *h, hipStream_t s);
hipError_t launch_unpack_weights(const gspc_packed *h, int which, float *w, hipStream_t s);
hipError_t launch_cast_bf16(const float *in, size_t count, uint16_t *out, hipStream_t s);

hipError_t launch_relu(const float *x, float *y, size_t count, hipStream_t s);
hipError_t launch_add(const float *a, const float *b, float *y, size_t count,
                      int relu, hipStream_t s);
hipError_t launch_maxpool(const float *x, float *y, int N, int C, int H, int W,
                          int K, int stride, int pad, int Hout, int Wout,
                          hipStream_t s);

}  // namespace gspc
