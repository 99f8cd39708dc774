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
enum MfmaVariant { kMfmaNone = 0, kMfma4 = 4, kMfma16 = 16, kMfma32 = 32 };

// Reduction slots one MFMA instruction consumes per variant (its K extent).
__host__ __device__ constexpr int mfma_ksub(int variant) {
    return variant == 32 ? 2 : variant == 16 ? 4 : 1;
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// Geometry of the two sections of a packed-weight buffer.
//   direct section : fp32 [g][Kred][KPGd], Kred = CPG*KH*KW ordered (c, kh, kw),
//                    KPGd = KPG rounded up to a multiple of 4, zero padded.
//   mfma section   : fp32 [g][KPG/variant][ksteps][64], the A operand of one
//                    MFMA per (k-step, lane); k-steps ordered (c / ksub, kh, kw)
//                    with CPG zero-padded to a multiple of ksub; lane l holds
//                    filter (l % variant) [all variants] and reduction slot
//                    c = cblk*ksub + l / variant [variants 32, 16].
struct PackGeom {
    int CPG, KPG, Kred, KPGd;
    int variant;   // MfmaVariant
    int ksub, CPGp, ksteps, mtiles;
    size_t direct_bytes, mfma_bytes, mfma_offset, total_bytes;
};

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
    float *y;           // [N][Cout][Hout][Wout]
    const float *res;   // optional residual, same shape as y
    int N, Cin, H, W, Cout, KH, KW, stride, pad, groups;
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
