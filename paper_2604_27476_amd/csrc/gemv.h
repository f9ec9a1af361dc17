// Wave-level GEMV building blocks shared by the per-stage decode kernels and the fused decode-step kernel.
#pragma once
#include "common.h"

namespace efm {

// ------------------------------------------------------------------------------------------------
// One wave computes NR dot products of length K = 8*nvec against the staged vector.
// Each lane keeps up to U*NR independent 16-byte loads in flight before the FMA chain.  The loads of
// the first chunk can be issued ahead of time (wave_prefetch), e.g. before the workgroup stages its
// activation vector: weights never depend on activations.
// ------------------------------------------------------------------------------------------------
template <int NR, int U> struct Chunk {
    u32x4 w[U][NR];
};

template <int NR, int U>
__device__ __forceinline__ void chunk_load(Chunk<NR, U> &c, const uint16_t *const (&rows)[NR], int v0, int nvec) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int v = v0 + u * WAVE;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            if (v < nvec) c.w[u][r] = ld_stream16(rows[r] + (size_t)v * 8);
            else c.w[u][r] = u32x4{0u, 0u, 0u, 0u};
        }
    }
}

template <int DT, int NR, int U>
__device__ __forceinline__ void chunk_fma(const Chunk<NR, U> &c, const float4 *xs, int v0, int nvec, float (&acc)[NR]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int v = v0 + u * WAVE;
        if (v < nvec) {
            const float4 a = xs[v], b = xs[nvec + v];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                float f[8];
                unpack8<DT>(c.w[u][r], f);
                float s = acc[r];
                s = fmaf(f[0], a.x, s); s = fmaf(f[1], a.y, s); s = fmaf(f[2], a.z, s); s = fmaf(f[3], a.w, s);
                s = fmaf(f[4], b.x, s); s = fmaf(f[5], b.y, s); s = fmaf(f[6], b.z, s); s = fmaf(f[7], b.w, s);
                acc[r] = s;
            }
        }
    }
}

// `pre` holds the chunk starting at v0 = lane if have_pre (in flight or arrived); it is clobbered.
template <int DT, int NR, int U>
__device__ __forceinline__ void wave_dots(const uint16_t *const (&rows)[NR], const float4 *xs, int nvec, int lane,
                                          float (&out)[NR], Chunk<NR, U> &pre, bool have_pre) {
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.f;
    for (int v0 = lane; v0 < nvec; v0 += WAVE * U) {  // one register buffer, reused for every chunk
        if (!have_pre) chunk_load<NR, U>(pre, rows, v0, nvec);
        have_pre = false;
        chunk_fma<DT, NR, U>(pre, xs, v0, nvec, acc);
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) out[r] = wave_sum(acc[r]);
}

}  // namespace efm
