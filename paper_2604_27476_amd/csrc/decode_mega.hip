// Fused decode step: ONE persistent kernel per token (Eq. 4 of Section 3.5 as a single launch).
//
// Why: at batch 1 a decoder layer is five dependent stages (QKV, attention, O projection, gate/up, down),
// three of which move only 1-33 MB.  As separate kernels each stage pays a launch/drain bubble of ~3-4 us
// in which HBM idles; 140 bubbles are ~20 % of a 2.5 ms step.  Weights, however, never depend on
// activations.  Here one workgroup per CU stays resident for the whole step, the stages are separated
// by grid barriers, and every wave issues the loads of its first weight chunk of the NEXT stage before
// it enters the barrier, so the HBM stream continues across stage boundaries (Section 3.4's last
// hot-spot class -- launch latency and host synchronisation -- removed instead of hidden in a graph).
//
// Cross-workgroup data (activations of a few KB) is published with agent-scope atomic stores: the L2s of
// the eight XCDs are not coherent with each other, and these stores are written through to the
// device-coherent level, so the barrier needs no L2 write-back (measured: ~6 us per barrier with one
// invalidate per workgroup on the reading side, against ~40-120 us with release/acquire fences in every
// thread).  Readers use ordinary cached loads after that invalidate, so a vector that all 32 CUs of an XCD
// stage is fetched from memory once per XCD.  The barrier is a monotonically
// increasing 64-bit arrival counter; a bounded spin turns a lost workgroup into an error flag instead of
// a hang.
//
// Layout of the work: the unit of a GEMV stage is a pair of weight rows; wave w of workgroup b owns units
// gw, gw + n_waves, ... with gw = w * n_workgroups + b (units spread over the CUs first), and handles two
// units per pass (four rows, 16 16-byte loads per lane in flight).  The staged activation vector lives
// in LDS.
#include "common.h"
#include "gemv.h"
#include "kernels.h"

namespace efm {

constexpr float NEG_BIG_M = -1.0e30f;
constexpr int MEGA_WAVES = 8;       // 512 threads: a 256-register budget per wave
constexpr int MEGA_CHUNK_MIN = 128;    // minimum keys per attention slice
constexpr int MEGA_SPIN_LIMIT = 400000;

template <typename T> __device__ __forceinline__ T aload(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void astore(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct MegaSync {
    unsigned long long *ctr;
    int *err;
    unsigned long long next;  // counter value that completes the next barrier
    unsigned n_wg;
};

// Grid barrier in two halves, so that loads which do not depend on other workgroups (the next stage's weights)
// can be issued between them: the arrival then waits for this stage's stores only, not for those loads.
// arrive: this workgroup's agent-scope stores are complete and counted.
__device__ __forceinline__ void grid_arrive(MegaSync &sy) {
    wait_own_stores();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(sy.ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// wait: every workgroup has arrived.  Thread 0 spins; its wave issues no weight prefetch, so the counter reads
// do not queue behind one (vector-memory returns are in order per wave).
__device__ __forceinline__ void grid_wait(MegaSync &sy) {
    if (threadIdx.x == 0) {
        if (aload(sy.err) == 0) {
            int spins = 0;
            while (aload(sy.ctr) < sy.next) {
                if (++spins > MEGA_SPIN_LIMIT) {  // a workgroup never arrived: flag it and go on (results are void)
                    astore(sy.err, 1);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        // One invalidate per workgroup: drops this CU's L1 and the non-coherent lines of this XCD's L2, so the
        // ordinary (cached, 16-byte, pipelined) loads that follow fetch what the other workgroups published.
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    sy.next += sy.n_wg;
    __syncthreads();
}
__device__ __forceinline__ void grid_barrier(MegaSync &sy) {
    grid_arrive(sy);
    grid_wait(sy);
}

// Stage a vector that other workgroups produced (agent-scope loads), optionally RMSNorm * gain, into the
// split LDS layout of gemv.h (lo[v] = x[8v..8v+3], hi[v] = x[8v+4..8v+7]).
template <int DT, bool NORM, bool COHERENT>
__device__ __forceinline__ void stage_shared_vec(const float *x, const uint16_t *gain, int n, float eps, float4 *xs,
                                                 float *red, float *export_to) {
    const int nvec = n >> 3;
    float ss = 0.f;
#pragma unroll 2
    for (int v = threadIdx.x; v < nvec; v += blockDim.x) {  // barely unrolled: this runs while prefetched weight
        // chunks occupy most of the register file
        const float4 p = reinterpret_cast<const float4 *>(x)[2 * v], q = reinterpret_cast<const float4 *>(x)[2 * v + 1];
        xs[v] = p;
        xs[nvec + v] = q;
        ss += p.x * p.x + p.y * p.y + p.z * p.z + p.w * p.w + q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
    }
    if constexpr (NORM) {
        ss = block_sum(ss, red);
        const float rstd = 1.0f / sqrtf(ss / (float)n + eps);
#pragma unroll 1
        for (int v = threadIdx.x; v < nvec; v += blockDim.x) {  // each thread rescales what it wrote
            float g[8];
            unpack8<DT>(ld16(gain + 8 * v), g);
            float4 a = xs[v], b = xs[nvec + v];
            a.x = a.x * rstd * g[0]; a.y = a.y * rstd * g[1]; a.z = a.z * rstd * g[2]; a.w = a.w * rstd * g[3];
            b.x = b.x * rstd * g[4]; b.y = b.y * rstd * g[5]; b.z = b.z * rstd * g[6]; b.w = b.w * rstd * g[7];
            xs[v] = a;
            xs[nvec + v] = b;
            if (export_to) {
                reinterpret_cast<float4 *>(export_to)[2 * v] = a;
                reinterpret_cast<float4 *>(export_to)[2 * v + 1] = b;
            }
        }
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// attention of one (kv head, context slice) by a 16-wave workgroup; see k_attn_decode for the scheme.
// Differences: q, and the new K/V row of this step, arrive un-rotated in fp32 from the QKV stage
// (qkv_raw); RoPE, the rounding to the cache dtype and the cache write happen here.
// ------------------------------------------------------------------------------------------------
template <int KDT, int D, int GQ>
__device__ __forceinline__ void mega_attention(const MegaArgs &a, int layer, int pos, int kvh, int s, int n_active,
                                               int chunk, float *wst /* [16][GQ][D+2], aliases the vector buffer */,
                                               float *qs /* [GQ][D] */, float *knew, float *vnew, float *sm, float *sl,
                                               uint32_t *ticket_s) {
    constexpr int EPL = 8, LPR = D / EPL, RW = WAVE / LPR, UR = 2, NW = MEGA_WAVES, PS = D + 2, HALF = D / 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, li = lane % LPR;
    const int n_keys = pos + 1;
    const int j0 = s * chunk, j1 = min(n_keys, j0 + chunk);
    const bool has_new = (j1 == n_keys);  // this slice ends with the position written in this step
    const int qd = a.nq * D, kvd = a.nkv * D;
    uint16_t *kc = a.kcache + (size_t)layer * a.kv_layer_stride + (size_t)kvh * a.max_seq * D;
    uint16_t *vc = a.vcache + (size_t)layer * a.kv_layer_stride + (size_t)kvh * a.max_seq * D;

    // rotate q (and the new k), round the new k/v to the cache dtype
    for (int p = tid; p < (GQ + 1) * HALF; p += blockDim.x) {
        const int hh = p / HALF, i = p - hh * HALF;
        const float c = a.rope_cos[(size_t)pos * HALF + i], sn = a.rope_sin[(size_t)pos * HALF + i];
        if (hh < GQ) {
            const float *src = a.qkv_raw + (size_t)(kvh * GQ + hh) * D;
            const float v0 = src[i], v1 = src[i + HALF];
            qs[hh * D + i] = (v0 * c - v1 * sn) * a.scale;
            qs[hh * D + i + HALF] = (v1 * c + v0 * sn) * a.scale;
        } else if (has_new) {
            const float *src = a.qkv_raw + qd + (size_t)kvh * D;
            const float v0 = src[i], v1 = src[i + HALF];
            const uint16_t b0 = down1<KDT>(v0 * c - v1 * sn), b1 = down1<KDT>(v1 * c + v0 * sn);
            knew[i] = up1<KDT>(b0);
            knew[i + HALF] = up1<KDT>(b1);
            kc[(size_t)pos * D + i] = b0;  // cache write: read by later launches only
            kc[(size_t)pos * D + i + HALF] = b1;
            const float *vs = a.qkv_raw + qd + kvd + (size_t)kvh * D;
            const uint16_t w0 = down1<KDT>(vs[i]), w1 = down1<KDT>(vs[i + HALF]);
            vnew[i] = up1<KDT>(w0);
            vnew[i + HALF] = up1<KDT>(w1);
            vc[(size_t)pos * D + i] = w0;
            vc[(size_t)pos * D + i + HALF] = w1;
        }
    }
    __syncthreads();

    float m[GQ], l[GQ], acc[GQ][EPL];
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
        m[h] = NEG_BIG_M;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }
    // one update of the online-softmax state with UR rows (kf, vf: row values of this lane's EPL elements)
    auto update = [&](const float (&kf)[UR][EPL], const float (&vf)[UR][EPL], const bool (&ok)[UR]) {
        float sc[UR][GQ];
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
            const float4 qa = *reinterpret_cast<const float4 *>(qs + h * D + li * EPL);
            const float4 qb = *reinterpret_cast<const float4 *>(qs + h * D + li * EPL + 4);
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                float t = qa.x * kf[u][0];
                t = fmaf(qa.y, kf[u][1], t); t = fmaf(qa.z, kf[u][2], t); t = fmaf(qa.w, kf[u][3], t);
                t = fmaf(qb.x, kf[u][4], t); t = fmaf(qb.y, kf[u][5], t); t = fmaf(qb.z, kf[u][6], t);
                t = fmaf(qb.w, kf[u][7], t);
#pragma unroll
                for (int off = LPR / 2; off > 0; off >>= 1) t += __shfl_xor(t, off, WAVE);
                sc[u][h] = ok[u] ? t : NEG_BIG_M;
            }
        }
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
            float mn = m[h];
#pragma unroll
            for (int u = 0; u < UR; ++u) mn = fmaxf(mn, sc[u][h]);
            const float corr = __expf(m[h] - mn);
            m[h] = mn;
            l[h] *= corr;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] *= corr;
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const float p = ok[u] ? __expf(sc[u][h] - mn) : 0.f;
                l[h] += p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(p, vf[u][e], acc[h][e]);
            }
        }
    };

    const int jc = has_new ? j1 - 1 : j1;  // rows [j0, jc) come from the cache
    for (int jb = j0 + wave * (RW * UR); jb < jc; jb += NW * RW * UR) {
        u32x4 kv[UR], vv[UR];
        bool ok[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int j = jb + u * RW + sub;
            ok[u] = j < jc;
            const int jj = ok[u] ? j : j0;
            kv[u] = ld16(kc + (size_t)jj * D + li * EPL);
            vv[u] = ld16(vc + (size_t)jj * D + li * EPL);
        }
        float kf[UR][EPL], vf[UR][EPL];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            unpack8<KDT>(kv[u], kf[u]);
            unpack8<KDT>(vv[u], vf[u]);
        }
        update(kf, vf, ok);
    }
    if (has_new && wave == 0) {  // the row of this step, taken from LDS by lane group 0
        float kf[UR][EPL], vf[UR][EPL];
        bool ok[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            ok[u] = (u == 0) && (sub == 0);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                kf[u][e] = knew[li * EPL + e];
                vf[u][e] = vnew[li * EPL + e];
            }
        }
        update(kf, vf, ok);
    }

    // merge the lane groups of the wave, then the waves (LDS), then write the slice record
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
        float mw = m[h];
#pragma unroll
        for (int off = LPR; off < WAVE; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off, WAVE));
        const float c = __expf(m[h] - mw);
        float lw = l[h] * c;
#pragma unroll
        for (int off = LPR; off < WAVE; off <<= 1) lw += __shfl_xor(lw, off, WAVE);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float v = acc[h][e] * c;
#pragma unroll
            for (int off = LPR; off < WAVE; off <<= 1) v += __shfl_xor(v, off, WAVE);
            acc[h][e] = v;
        }
        if (sub == 0) {
            float *w = wst + ((size_t)wave * GQ + h) * PS;
            if (li == 0) {
                w[0] = mw;
                w[1] = lw;
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) w[2 + li * EPL + e] = acc[h][e];
        }
    }
    __syncthreads();
    float *prec = a.part + ((size_t)(kvh * GQ) * a.S + s) * PS;
    for (int idx = tid; idx < GQ * D; idx += blockDim.x) {
        const int h = idx / D, i = idx - h * D;
        float mt = NEG_BIG_M;
#pragma unroll
        for (int w = 0; w < NW; ++w) mt = fmaxf(mt, wst[((size_t)w * GQ + h) * PS]);
        float lt = 0.f, at = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float *ws = wst + ((size_t)w * GQ + h) * PS;
            const float c = __expf(ws[0] - mt);
            lt += ws[1] * c;
            at += ws[2 + i] * c;
        }
        float *rec = prec + (size_t)h * a.S * PS;
        if (i == 0) {
            astore(rec + 0, mt);
            astore(rec + 1, lt);
        }
        astore(rec + 2 + i, at);
    }
    wait_own_stores();
    __syncthreads();
    if (tid == 0) *ticket_s = __hip_atomic_fetch_add(&a.counters[kvh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*ticket_s != (uint32_t)(n_active - 1)) return;
    // last slice to arrive: combine all slices of this KV head in index order
    if (tid == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
    for (int idx = tid; idx < GQ * n_active; idx += blockDim.x) {
        const int h = idx / n_active, t = idx - h * n_active;
        const float *rec = a.part + ((size_t)(kvh * GQ + h) * a.S + t) * PS;
        sm[h * 64 + t] = rec[0];
        sl[h * 64 + t] = rec[1];
    }
    __syncthreads();
    for (int idx = tid; idx < GQ * D; idx += blockDim.x) {
        const int h = idx / D, i = idx - h * D;
        const float *rec = a.part + ((size_t)(kvh * GQ + h) * a.S) * PS + 2 + i;
        float mt = NEG_BIG_M;
        for (int t = 0; t < n_active; ++t) mt = fmaxf(mt, sm[h * 64 + t]);
        float lt = 0.f, at = 0.f;
#pragma unroll 8
        for (int t = 0; t < n_active; ++t) {
            const float c = __expf(sm[h * 64 + t] - mt);
            lt += sl[h * 64 + t] * c;
            at += rec[(size_t)t * PS] * c;
        }
        astore(a.o + (size_t)(kvh * GQ + h) * D + i, at / lt);
    }
    if (tid == 0) astore(&a.counters[kvh], 0u);
}

// ------------------------------------------------------------------------------------------------
// The step is a table of stages (built once on the host): per layer QKV, attention, O projection,
// gate/up, down; then lm_head.  One generic loop walks the table, so the chunk registers have one
// consumer and the kernel stays small.
// ------------------------------------------------------------------------------------------------
// Pass depth: 4 rows x MEGA_U 16-byte vectors per lane (64 registers).  Deeper passes spill: the compiler keeps
// the loop-carried chunk and the in-loop chunk in separate registers.
constexpr int MEGA_U = 4;
typedef Chunk<4, MEGA_U> Chunk4;

// The stage table is read-only for the whole launch.  Reading it through the constant address space lets
// the compiler use scalar loads (one copy per wave in SGPRs); through an ordinary global pointer every
// field would sit in vector registers, because the kernel also writes global memory.
template <typename T> __device__ __forceinline__ T cload(const T *p) {
    return *reinterpret_cast<const __attribute__((address_space(4))) T *>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ MegaStage load_stage(const MegaStage *p) {
    MegaStage d;
    const uint64_t *q = reinterpret_cast<const uint64_t *>(p);
    d.W = reinterpret_cast<const uint16_t *>(cload(q + 0));
    d.bias = reinterpret_cast<const uint16_t *>(cload(q + 1));
    d.gain = reinterpret_cast<const uint16_t *>(cload(q + 2));
    d.vec = reinterpret_cast<const float *>(cload(q + 3));
    d.out = reinterpret_cast<float *>(cload(q + 4));
    const int *r = reinterpret_cast<const int *>(q + 5);
    d.K = cload(r + 0); d.n_units = cload(r + 1); d.rows = cload(r + 2); d.aux = cload(r + 3);
    d.epi = cload(r + 4); d.vec_kind = cload(r + 5); d.layer = cload(r + 6); d.pad = 0;
    return d;
}

__device__ __forceinline__ void unit_rows(const MegaStage &s, int u, const uint16_t *&r0, const uint16_t *&r1) {
    int a, b;
    if (s.rows == MROWS_SPLIT) { a = u; b = s.aux + u; }
    else if (s.rows == MROWS_PAIR_CLAMP) { a = 2 * u; b = min(2 * u + 1, s.aux - 1); }
    else { a = 2 * u; b = 2 * u + 1; }
    r0 = s.W + (size_t)a * s.K;
    r1 = s.W + (size_t)b * s.K;
}

// Issue the loads of this wave's first pass of stage s (units gw and gw + gstride).  The loads are
// predicated per lane (a wave without a unit passes nvec = 0), never skipped by a branch.
__device__ __forceinline__ void stage_prefetch(Chunk4 &pre, const MegaStage &s, int gw, int gstride, int lane,
                                               bool enabled) {
    const bool va = enabled && gw < s.n_units, vb = enabled && gw + gstride < s.n_units;
    const uint16_t *rows[4];
    unit_rows(s, va ? gw : 0, rows[0], rows[1]);
    unit_rows(s, vb ? gw + gstride : (va ? gw : 0), rows[2], rows[3]);
    chunk_load<4, MEGA_U>(pre, rows, lane, va ? (s.K >> 3) : 0);
}

template <int WDT, int KDT, int D, int GQ>
__global__ void __launch_bounds__(MEGA_WAVES * 64)
k_decode_mega(const MegaArgs a) {
    extern __shared__ float4 smem[];  // staged vector; attention wave states alias it
    __shared__ float red[32];
    __shared__ float qs[GQ * D], knew[D], vnew[D], sm[GQ * 64], sl[GQ * 64];
    __shared__ uint32_t ticket_s;
    __shared__ unsigned long long base_s;
    __shared__ float bv[MEGA_WAVES];
    __shared__ int bi[MEGA_WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: unit indices and row pointers stay scalar
    const int n_wg = gridDim.x;
    const int gw = wave * n_wg + blockIdx.x, gstride = n_wg * MEGA_WAVES;  // CU-major unit ownership
    const int pos = a.d_pos[0], token = a.d_token[0];

    MegaSync sy;
    sy.ctr = a.bar;
    sy.err = a.err;
    sy.n_wg = (unsigned)n_wg;
    if (tid == 0) {  // the counter only grows; this launch starts at the last multiple of (barriers * workgroups)
        const unsigned long long per_launch = (unsigned long long)a.n_stages * n_wg;
        base_s = aload(a.bar) / per_launch * per_launch;
    }
    __syncthreads();
    sy.next = base_s + n_wg;

    // attention geometry of this step (same in every layer)
    const int n_keys = pos + 1;
    int chunk = (n_keys + a.S - 1) / a.S;
    if (chunk < MEGA_CHUNK_MIN) chunk = MEGA_CHUNK_MIN;
    const int n_active = (n_keys + chunk - 1) / chunk;
    const bool attn_wg = (int)blockIdx.x < a.nkv * n_active;

    float best = -INFINITY;
    int best_i = 0x7fffffff;
    // optional stage trace (workgroup 0): constant-rate clock at stage entry, after the barrier, after staging,
    // after the last unit
    const bool tracing = a.trace != nullptr && blockIdx.x == 0 && tid == 0;
    auto stamp = [&](int st, int k) {
        if (tracing) a.trace[4 * st + k] = wall_clock64();
    };
    Chunk4 pre;
    // Every stage ends with: arrive at the grid barrier (this stage's stores are complete), THEN issue the loads of
    // the next GEMV stage's first pass, and the next stage begins with the wait half of the barrier: the weight
    // stream goes on while the workgroups meet.  Wave 0 holds the thread that spins on the arrival counter and
    // therefore never prefetches.
    const bool pf_wave = wave != 0;
    bool have_pre = false;  // `pre` holds this wave's first pass of the coming GEMV stage
    // The loop starts one stage early (st = -1 only prefetches stage 0): the chunk registers then have no
    // definition outside the loop, which keeps the compiler from holding two copies of them.
    for (int st = -1; st < a.n_stages; ++st) {
        const MegaStage d = load_stage(a.stages + (st < 0 ? 0 : st));
        if (st < 0) {
            stage_prefetch(pre, d, gw, gstride, lane, pf_wave);
            have_pre = pf_wave;
            continue;
        }
        stamp(st, 0);
        if (d.epi == MEPI_ATTN) {
            // Workgroups without an attention slice already stream their first O-projection pass; the others
            // issue it after the attention (the chunk registers are free during it).
            grid_wait(sy);
            stamp(st, 1);
            if (attn_wg) {
                const int kvh = (int)blockIdx.x % a.nkv, s = (int)blockIdx.x / a.nkv;
                mega_attention<KDT, D, GQ>(a, d.layer, pos, kvh, s, n_active, chunk, reinterpret_cast<float *>(smem), qs,
                                           knew, vnew, sm, sl, &ticket_s);
            }
            grid_arrive(sy);
            if (attn_wg) {
                stage_prefetch(pre, load_stage(a.stages + st + 1), gw, gstride, lane, pf_wave);
                have_pre = pf_wave;
            }
            stamp(st, 3);
            continue;
        }
        // ---- inputs of this stage are complete; stage its activation vector in LDS ----
        if (st > 0) grid_wait(sy);
        stamp(st, 1);
        const int nvec = d.K >> 3;
        if (d.vec_kind == MVEC_EMBED) {
            // x = E[token], read directly by every workgroup; workgroup 0 also publishes it as the residual
            const uint16_t *row = a.embed + (size_t)token * d.K;
            float ss = 0.f;
#pragma unroll 1
            for (int v = tid; v < nvec; v += blockDim.x) {
                float f[8];
                unpack8<WDT>(ld16(row + 8 * v), f);
                smem[v] = make_float4(f[0], f[1], f[2], f[3]);
                smem[nvec + v] = make_float4(f[4], f[5], f[6], f[7]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    ss += f[e] * f[e];
                    if (blockIdx.x == 0) astore(a.x + 8 * v + e, f[e]);
                }
            }
            ss = block_sum(ss, red);
            const float rstd = 1.0f / sqrtf(ss / (float)d.K + a.eps);
#pragma unroll 1
            for (int v = tid; v < nvec; v += blockDim.x) {
                float g[8];
                unpack8<WDT>(ld16(d.gain + 8 * v), g);
                float4 p = smem[v], q = smem[nvec + v];
                p.x = p.x * rstd * g[0]; p.y = p.y * rstd * g[1]; p.z = p.z * rstd * g[2]; p.w = p.w * rstd * g[3];
                q.x = q.x * rstd * g[4]; q.y = q.y * rstd * g[5]; q.z = q.z * rstd * g[6]; q.w = q.w * rstd * g[7];
                smem[v] = p;
                smem[nvec + v] = q;
            }
            __syncthreads();
        } else if (d.gain) {
            stage_shared_vec<WDT, true, true>(d.vec, d.gain, d.K, a.eps, smem, red,
                                              (d.epi == MEPI_LOGITS && blockIdx.x == 0) ? a.hidden : nullptr);
        } else {
            stage_shared_vec<WDT, false, true>(d.vec, nullptr, d.K, 0.f, smem, red, nullptr);
        }
        stamp(st, 2);
        // ---- the wave's units, two per pass; the first pass was prefetched (not by wave 0) ----
        bool first = have_pre;
        have_pre = false;
        for (int ua = gw; ua < d.n_units; ua += 2 * gstride) {
            const int ub = ua + gstride;
            const bool vb = ub < d.n_units;
            const uint16_t *rows[4];
            unit_rows(d, ua, rows[0], rows[1]);
            unit_rows(d, vb ? ub : ua, rows[2], rows[3]);
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            int v0 = lane;
            if (first) {
                chunk_fma<WDT, 4, MEGA_U>(pre, smem, v0, nvec, acc);
                v0 += WAVE * MEGA_U;
                first = false;
            }
            for (; v0 < nvec; v0 += WAVE * MEGA_U) {
                chunk_load<4, MEGA_U>(pre, rows, v0, nvec);
                chunk_fma<WDT, 4, MEGA_U>(pre, smem, v0, nvec, acc);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = wave_sum(acc[r]);
            if (lane == 0) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    if (half == 1 && !vb) break;
                    const int u = half ? ub : ua;
                    float d0 = acc[2 * half], d1 = acc[2 * half + 1];
                    if (d.epi == MEPI_STORE) {  // fused QKV: raw q, k, v (+ bias)
                        if (d.bias) {
                            d0 += up1<WDT>(d.bias[2 * u]);
                            d1 += up1<WDT>(d.bias[2 * u + 1]);
                        }
                        astore(d.out + 2 * u, d0);
                        astore(d.out + 2 * u + 1, d1);
                    } else if (d.epi == MEPI_RESID) {  // O / down projection: residual add
                        astore(d.out + 2 * u, d.out[2 * u] + d0);
                        astore(d.out + 2 * u + 1, d.out[2 * u + 1] + d1);
                    } else if (d.epi == MEPI_SWIGLU) {  // gate/up: h = silu(gate) * up
                        astore(d.out + u, d0 / (1.0f + expf(-d0)) * d1);
                    } else {  // lm_head: logits + running argmax (rows are visited in increasing order per wave)
                        const int r0 = 2 * u, r1 = min(2 * u + 1, d.aux - 1);
                        d.out[r0] = d0;
                        if (d0 > best) { best = d0; best_i = r0; }
                        if (r1 != r0) {
                            d.out[r1] = d1;
                            if (d1 > best) { best = d1; best_i = r1; }
                        }
                    }
                }
            }
        }
        stamp(st, 3);
        // ---- publish, then (weights never depend on activations) start the next GEMV stage's first pass ----
        if (st + 1 < a.n_stages) {
            grid_arrive(sy);
            const MegaStage nx = load_stage(a.stages + st + 1);
            if (nx.epi != MEPI_ATTN) {
                stage_prefetch(pre, nx, gw, gstride, lane, pf_wave);
                have_pre = pf_wave;
            } else if (!attn_wg) {
                stage_prefetch(pre, load_stage(a.stages + st + 2), gw, gstride, lane, pf_wave);
                have_pre = pf_wave;
            }
        }
    }
    // ---------------- greedy argmax over the lm_head partials ----------------------------------------
    if (lane == 0) {
        bv[wave] = best;
        bi[wave] = best_i;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < MEGA_WAVES; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < best_i)) { best = bv[w]; best_i = bi[w]; }
        astore(a.part_val + blockIdx.x, best);
        astore(a.part_idx + blockIdx.x, best_i);
    }
    grid_barrier(sy);
    // ---------------- finish: token feedback and position advance (Section 3.10) ---------------------
    if (blockIdx.x == 0 && wave == 0) {
        best = -INFINITY;
        best_i = 0x7fffffff;
        for (int p = lane; p < n_wg; p += WAVE) {
            const float v = aload(a.part_val + p);
            const int i = aload(a.part_idx + p);
            if (v > best || (v == best && i < best_i)) { best = v; best_i = i; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float v = __shfl_xor(best, o, WAVE);
            const int i = __shfl_xor(best_i, o, WAVE);
            if (v > best || (v == best && i < best_i)) { best = v; best_i = i; }
        }
        if (lane == 0) {
            if (best_i == 0x7fffffff) best_i = 0;
            a.d_next[0] = best_i;
            a.d_token[0] = best_i;
            a.d_pos[0] = pos + 1;
        }
    }
}

// ================================================================================================
// host side
// ================================================================================================
struct MegaKey {
    int wdt, kvdt, d, g;
};
template <int WDT, int KDT, int D, int GQ> static const void *mega_fn() {
    return reinterpret_cast<const void *>(&k_decode_mega<WDT, KDT, D, GQ>);
}

// The fused kernel is compiled for the shapes of the target workloads (Section 3.8: shape-specific
// operators); other shapes use the per-stage kernels.
static const void *mega_lookup(const Dims &D) {
    const int g = D.g();
#define MEGA_CASE(WDT, KDT, DD, GQ) \
    if (D.wdt == WDT && D.kvdt == KDT && D.d == DD && g == GQ) return mega_fn<WDT, KDT, DD, GQ>();
    MEGA_CASE(DT_BF16, DT_BF16, 128, 7)  // 7B-shaped
    MEGA_CASE(DT_BF16, DT_BF16, 128, 6)  // 1.5B-shaped
    MEGA_CASE(DT_BF16, DT_BF16, 64, 7)   // 0.5B-shaped
    MEGA_CASE(DT_F16, DT_F16, 64, 2)     // tiny
#undef MEGA_CASE
    return nullptr;
}

// Stage table of one decode step: per layer QKV, attention, O, gate/up, down; then lm_head.
void mega_build_stages(const Dims &D, const LayerW *lw, const MegaArgs &a, MegaStage *out) {
    const int H = D.H, I = D.I, qd = D.qd(), R = D.R();
    int n = 0;
    for (int l = 0; l < D.L; ++l) {
        MegaStage q = {};
        q.W = lw[l].wqkv; q.bias = D.qkv_bias ? lw[l].bqkv : nullptr; q.gain = lw[l].attn_norm; q.vec = a.x;
        q.out = a.qkv_raw; q.K = H; q.n_units = R / 2; q.rows = MROWS_PAIR; q.aux = 0; q.epi = MEPI_STORE;
        q.vec_kind = l == 0 ? MVEC_EMBED : MVEC_SHARED; q.layer = l;
        out[n++] = q;
        MegaStage at = {};
        at.epi = MEPI_ATTN; at.layer = l;
        out[n++] = at;
        MegaStage o = {};
        o.W = lw[l].wo; o.vec = a.o; o.out = a.x; o.K = qd; o.n_units = H / 2; o.rows = MROWS_PAIR; o.epi = MEPI_RESID;
        o.vec_kind = MVEC_SHARED; o.layer = l;
        out[n++] = o;
        MegaStage g = {};
        g.W = lw[l].w_gate_up; g.gain = lw[l].mlp_norm; g.vec = a.x; g.out = a.h; g.K = H; g.n_units = I;
        g.rows = MROWS_SPLIT; g.aux = I; g.epi = MEPI_SWIGLU; g.vec_kind = MVEC_SHARED; g.layer = l;
        out[n++] = g;
        MegaStage dn = {};
        dn.W = lw[l].w_down; dn.vec = a.h; dn.out = a.x; dn.K = I; dn.n_units = H / 2; dn.rows = MROWS_PAIR;
        dn.epi = MEPI_RESID; dn.vec_kind = MVEC_SHARED; dn.layer = l;
        out[n++] = dn;
    }
    MegaStage lm = {};
    lm.W = a.lm; lm.gain = a.final_norm; lm.vec = a.x; lm.out = a.logits; lm.K = H; lm.n_units = (D.V + 1) / 2;
    lm.rows = MROWS_PAIR_CLAMP; lm.aux = D.V; lm.epi = MEPI_LOGITS; lm.vec_kind = MVEC_SHARED; lm.layer = D.L;
    out[n++] = lm;
}

size_t mega_lds_bytes(const Dims &D) {
    size_t vec = (size_t)(D.H > D.I ? D.H : D.I) * 4;
    if ((size_t)D.qd() * 4 > vec) vec = (size_t)D.qd() * 4;
    const size_t wst = (size_t)MEGA_WAVES * D.g() * (D.d + 2) * 4;
    return vec > wst ? vec : wst;
}

bool mega_supported(const Dims &D, const Geo &G) {
    if (!mega_lookup(D)) return false;
    if (D.H % 16 || D.R() % 2 || D.V < 2) return false;
    if (D.nkv * MEGA_CHUNK_MIN > 0 && D.nkv > G.n_cu) return false;
    return true;
}

int mega_splits(const Dims &D, const Geo &G) {
    int s = G.n_cu / D.nkv;
    return s > 64 ? 64 : (s < 1 ? 1 : s);
}

hipError_t mega_prepare(const Dims &D, const Geo &G) {
    const void *fn = mega_lookup(D);
    if (!fn) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)mega_lds_bytes(D));
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, MEGA_WAVES * 64, mega_lds_bytes(D));
    if (e != hipSuccess) return e;
    return per_cu >= 1 ? hipSuccess : hipErrorLaunchOutOfResources;
}

hipError_t launch_decode_mega(const Dims &D, const Geo &G, const MegaArgs &args, hipStream_t st) {
    const void *fn = mega_lookup(D);
    if (!fn) return hipErrorInvalidValue;
    MegaArgs a = args;
    void *params[] = {&a};
    return hipLaunchKernel(fn, dim3(G.n_cu), dim3(MEGA_WAVES * 64), params, mega_lds_bytes(D), st);
}

}  // namespace efm
