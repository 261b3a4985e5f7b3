// A row of head_dim elements (a value row, a block representative) spread over 16 lanes.
#pragma once
#include "alaya_internal.h"

namespace alaya {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// A value row is spread over 16 lanes; each lane owns EPL = D / 16 consecutive elements.
template <int DT, int D> struct RowSlice {
    static constexpr int EPL = D / 16;
    static constexpr int BYTES = EPL * (DT == 0 ? 2 : 4);
    static constexpr int WORDS = BYTES / 4;
    struct Raw { uint32_t w[WORDS]; }; // a lane's slice as loaded
    // row: first byte of the token's value row; sub = lane % 16.  STREAM: the row is read once, in order
    // with its neighbours (dense attention): non-temporal load.  Rows gathered at random are loaded plainly
    // (measured: the hint costs the gather 5 to 10 %).
    template <bool STREAM = false>
    __device__ static __forceinline__ Raw load_raw(const char *row, int sub)
    {
        const char *p = row + (size_t)sub * BYTES;
        Raw r;
        if constexpr (WORDS == 8) {
            const uint4 a = STREAM ? load_stream((const uint4 *)p) : *(const uint4 *)p;
            const uint4 b = STREAM ? load_stream((const uint4 *)(p + 16)) : *(const uint4 *)(p + 16);
            r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z; r.w[3] = a.w; r.w[4] = b.x; r.w[5] = b.y; r.w[6] = b.z; r.w[7] = b.w;
        } else if constexpr (WORDS == 4) {
            const uint4 a = STREAM ? load_stream((const uint4 *)p) : *(const uint4 *)p;
            r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z; r.w[3] = a.w;
        } else {
            const uint2 a = *(const uint2 *)p;
            r.w[0] = a.x; r.w[1] = a.y;
        }
        return r;
    }
    __device__ static __forceinline__ void widen(const Raw &r, float *f)
    {
        if constexpr (DT == 0) {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) { f[2 * i] = bf16_lo(r.w[i]); f[2 * i + 1] = bf16_hi(r.w[i]); }
        } else {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) f[i] = __uint_as_float(r.w[i]);
        }
    }
    template <bool STREAM = false>
    __device__ static __forceinline__ void load(const char *row, int sub, float *f)
    {
        widen(load_raw<STREAM>(row, sub), f);
    }
};

} // namespace alaya
