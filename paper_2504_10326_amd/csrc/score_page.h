// Scores of one page of keys against the query heads of a GQA group: shared by the scoring passes and by
// dense attention.  s[h][j] = q_h . k_{h/G, j} (numerator of Eq. 1; the inner product of Def. 2).
#pragma once
#include "alaya_internal.h"

namespace alaya {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                           false);
}

// Scores of the 64 tokens of one page (lane = token) for the G heads of a group.
// base: this lane's first 16-byte slice of the page's K tile; qh: the group's queries (wave-uniform).
template <int DT, int D, int G>
__device__ __forceinline__ void score_page(const uint4 *__restrict__ base, const uint4 *__restrict__ qh, float *acc)
{
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16; // 16-byte chunks per key
    constexpr int QW = D * (DT == 0 ? 2 : 4) / 4;  // 32-bit words per query head
    uint4 kc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) kc[c] = load_stream(base + c * 64);
    // The query (QW * G words) is streamed through scalar registers for every page.  The offset
    // is opaque to the compiler so that it does not hoist all of it out of the page loop.
    int opaque_zero = 0;
    asm volatile("" : "+s"(opaque_zero));
    const uint4 *qp = qh + opaque_zero;
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 qc = qp[g * (QW / 4) + c];
            if constexpr (DT == 0) {
                acc[g] = dot2_bf16(kc[c].x, qc.x, acc[g]);
                acc[g] = dot2_bf16(kc[c].y, qc.y, acc[g]);
                acc[g] = dot2_bf16(kc[c].z, qc.z, acc[g]);
                acc[g] = dot2_bf16(kc[c].w, qc.w, acc[g]);
            } else {
                acc[g] = fmaf(__uint_as_float(kc[c].x), __uint_as_float(qc.x), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].y), __uint_as_float(qc.y), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].z), __uint_as_float(qc.z), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].w), __uint_as_float(qc.w), acc[g]);
            }
        }
    }
}

// The same with the group's queries in LDS (G heads of QW words, head after head).  All lanes read the same
// 16 bytes at a time - a broadcast - so the queries take no scalar registers: streamed through those, the
// 64 * G words did not fit, and a third of the pass's vector instructions moved scalars in and out of lanes.
template <int DT, int D, int G>
__device__ __forceinline__ void score_page_lds(const uint4 *__restrict__ base, const uint4 (&q_lds)[G * (D * (DT == 0 ? 2 : 4) / 16)],
                                               float *acc)
{
    constexpr int NC = D * (DT == 0 ? 2 : 4) / 16;
    uint4 kc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) kc[c] = load_stream(base + c * 64);
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
    // (the offset is opaque to the compiler so that it reads the queries page by page: hoisted out of the page
    // loop they would take G * NC * 4 vector registers)
    int opaque_zero = 0;
    asm volatile("" : "+v"(opaque_zero));
    const uint4 *ql = &q_lds[0] + opaque_zero;
    // One 16-byte slice of every head at a time, the next slice on its way; a barrier for the instruction
    // scheduler between the steps keeps it from asking for all of them at once.
    uint4 qa[G], qb[G];
#pragma unroll
    for (int g = 0; g < G; ++g) qa[g] = ql[g * NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (c + 1 < NC) {
#pragma unroll
            for (int g = 0; g < G; ++g) qb[g] = ql[g * NC + c + 1];
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 qc = qa[g];
            if constexpr (DT == 0) {
                acc[g] = dot2_bf16(kc[c].x, qc.x, acc[g]);
                acc[g] = dot2_bf16(kc[c].y, qc.y, acc[g]);
                acc[g] = dot2_bf16(kc[c].z, qc.z, acc[g]);
                acc[g] = dot2_bf16(kc[c].w, qc.w, acc[g]);
            } else {
                acc[g] = fmaf(__uint_as_float(kc[c].x), __uint_as_float(qc.x), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].y), __uint_as_float(qc.y), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].z), __uint_as_float(qc.z), acc[g]);
                acc[g] = fmaf(__uint_as_float(kc[c].w), __uint_as_float(qc.w), acc[g]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < G; ++g) qa[g] = qb[g];
    }
    // (the sums are pinned here: otherwise the compiler moves each head's products down to where its score is
    // used, and keeps that head's queries in scratch memory until then)
#pragma unroll
    for (int g = 0; g < G; ++g) asm volatile("" : "+v"(acc[g]));
}

} // namespace alaya
