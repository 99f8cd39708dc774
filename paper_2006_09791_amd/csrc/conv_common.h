// Device and host helpers shared by the convolution kernels of libgspc.
#pragma once

#include <mutex>
#include <set>
#include <string>

#include "gspc_internal.h"

namespace gspc {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// n / d with mul = floor(2^32 / d) + 1 (mul = 0 encodes d = 1); exact while n * d < 2^32.
__device__ __forceinline__ unsigned fast_div(unsigned n, unsigned mul) {
    return mul ? __umulhi(n, mul) : n;
}

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Buffer descriptors: raw (stride 0) buffers whose out-of-range loads return
// zero and whose out-of-range stores are dropped by the hardware, so invalid
// lanes are given the byte offset kOob instead of being branched around.
constexpr unsigned kOob = 0xffffff00u;
constexpr int kRsrcFlags = 0x00020000;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, kRsrcFlags);
}
// Four (vec) or one consecutive input elements as fp32.
template <typename TIN> __device__ __forceinline__ f32x4 buf_load_in(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, int vec);
template <> __device__ __forceinline__ f32x4 buf_load_in<float>(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, int vec) {
    if (vec) return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
    return f32x4{__uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0)), 0.f, 0.f, 0.f};
}
template <> __device__ __forceinline__ f32x4 buf_load_in<uint16_t>(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, int vec) {
    if (vec) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        return f32x4{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                     __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u)};
    }
    const unsigned h = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    return f32x4{__uint_as_float(h << 16), 0.f, 0.f, 0.f};
}


// ---- host-side helpers --------------------------------------------------------
// Kernel names are reported as the template arguments of the instance that ran,
// so they can be matched one to one with a profiler's kernel names.  The
// returned pointer stays valid for the life of the process.
inline const char *intern_name(const std::string &s) {
    static std::mutex mu;
    static std::set<std::string> names;
    std::lock_guard<std::mutex> lock(mu);
    return names.insert(s).first->c_str();
}

constexpr int kNumCU = 256;

inline unsigned div_magic(int d) { return d > 1 ? (unsigned)(0xffffffffu / (unsigned)d + 1u) : 0u; }

// Splits the output into NB images x TH rows per block for a pixel capacity PB.
inline bool split_pixels(const ConvParams &p, int PB, int *NB, int *TH) {
    if (p.Wout > PB) return false;
    const int HWo = p.Hout * p.Wout;
    if (HWo <= PB) {
        *TH = p.Hout;
        *NB = PB / HWo;
        if (*NB > p.N) *NB = p.N;
    } else {
        *NB = 1;
        const int thmax = PB / p.Wout;
        const int rbk = (p.Hout + thmax - 1) / thmax;
        *TH = (p.Hout + rbk - 1) / rbk;
    }
    return true;
}

}  // namespace gspc
