// Helpers shared by the vector-ALU kernels (forward/decode and backward): workgroup shape, typed loads of
// fp32 / bf16 rows (bf16 is widened exactly), LDS tile staging, LDS dot products.
#pragma once

#include "llla_common.hpp"

namespace llla {
namespace valu {

constexpr int NT = 256;   // threads per workgroup
constexpr int KT = 32;    // keys per slot per tile

template <int D>
struct Cfg {
    static constexpr int TS = (D >= 64) ? 8 : 4;        // register tile edge
    static constexpr int TG = D / TS;                    // tiles per matrix edge
    static constexpr int TPQ = TG * TG;                  // threads per slot
    static constexpr int QB = NT / TPQ;                  // slots per workgroup
    static constexpr int LDK = D + 4;                    // LDS row pitch of K/V tiles (16 B aligned)
    static constexpr int P = D + 1;                      // unknowns of the augmented system
    static constexpr int LDS_SYS = (D + 2) | 1;          // odd pitch of [At | rhs]
};

template <typename T>
struct Io;
template <>
struct Io<float> {
    static constexpr int VEC = 4;
    __device__ static void load(const float *g, float *dst)
    {
        const float4 v = *reinterpret_cast<const float4 *>(g);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __device__ static void store1(float *g, float v) { *g = v; }
};
template <>
struct Io<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static void load(const bf16_t *g, float *dst)
    {
        const uint4 v = *reinterpret_cast<const uint4 *>(g);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dst[2 * i] = __uint_as_float(u[i] << 16);
            dst[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
        }
    }
    __device__ static void store1(bf16_t *g, float v) { *g = f32_to_bf16(v); }
};

// rows [row0, row0+rows_tile) of a [*, D] global matrix -> LDS tile (pitch LDK), zero beyond nvalid
template <int D, typename T>
__device__ inline void load_tile(float *lds, const T *g, int64_t row_stride, int row0, int rows_tile,
                                 int nvalid, int tid)
{
    constexpr int VEC = Io<T>::VEC;
    constexpr int CH = D / VEC;                          // chunks per row
    constexpr int LDK = Cfg<D>::LDK;
    for (int idx = tid; idx < rows_tile * CH; idx += NT) {
        const int r = idx / CH, c = (idx % CH) * VEC;
        float v[VEC];
        if (row0 + r < nvalid) {
            Io<T>::load(g + (int64_t)(row0 + r) * row_stride + c, v);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < VEC; i += 4)
            *reinterpret_cast<float4 *>(lds + r * LDK + c + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
    }
}

template <int D>
__device__ inline float dot_lds(const float *a, const float *b)
{
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
    for (int c = 0; c < D; c += 4) {
        const float4 x = *reinterpret_cast<const float4 *>(a + c);
        const float4 y = *reinterpret_cast<const float4 *>(b + c);
        s0 = fmaf(x.x, y.x, s0); s1 = fmaf(x.y, y.y, s1);
        s2 = fmaf(x.z, y.z, s2); s3 = fmaf(x.w, y.w, s3);
    }
    return (s0 + s1) + (s2 + s3);
}

}  // namespace valu
}  // namespace llla
