// Register-resident signature kernels for full truncations (all words of length <= N over D letters).
//
// Mapping ("one path per wavefront"): a wavefront works on ONE path; its 64 lanes are 64 work units of
// that path's word tree.  A unit is a prefix p of K letters (the chain, recomputed by every unit that shares
// it), a slice of the children of p (WQ groups of four letters), and the complete sub-trees under those
// children.  All coefficients of a unit stay in registers for all L segments.  The segment increments
// dX_j/(t+1) are staged per wavefront in LDS, a tile of T segments at a time, with coalesced loads of the
// path.
//
// Update of a word u of length k per segment (Algorithm 1 with shared intermediates):
//     A_k[t](u) = S(u) + dX^{(u_k)}/(t+1) * A_{k-1}[t+1](parent u),   t = 0..N-k,   A_0 = 1,
// A_k[0] being the new S(u).  The chain (k <= K, per-lane letters) runs on the vector ALU, everything
// below it on the matrix cores (see below).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.hpp"

namespace sig {
namespace {

constexpr int kWave = 64;

__host__ __device__ constexpr int ipow(int b, int e)
{
    int r = 1;
    for (int q = 0; q < e; ++q) r *= b;
    return r;
}
// first canonical index of the words of length n (n >= 1): sum_{m=1}^{n-1} D^m
__host__ __device__ constexpr int level_start(int D, int n)
{
    int r = 0;
    for (int m = 1; m < n; ++m) r += ipow(D, m);
    return r;
}

__device__ __forceinline__ constexpr float inv1(int t) { return 1.0f / (float)(t + 1); }

// ---------------------------------------------------------------------------------------------------------
// Matrix-core cascade.  The update of all children of 64 parent words by 4 letters,
//     child(u, 4g + j) (+)= A(u) * dX^{(4g+j)}/(t+1),
// is a batch of rank-1 updates, which is what v_mfma_f32_4x4x1_16b_f32 computes: 16 independent 4x4 outer
// products per instruction (K = 1), FP32 in and out.
// Operand layout (verified on gfx950): lane l = 4*blk + i supplies A[blk][i] and B[blk][i]; the result
// D[blk][i][j] = A[blk][i] * B[blk][j] + C[blk][i][j] sits in lane 4*blk + j, register i of the 4-vector.
// So one instruction takes a "word vector" (64 words, one per lane) and a per-lane increment
// (letter 4g + lane%4) and updates four child word vectors: register r holds, in lane 4*blk + j, the
// child with letter 4g + j of the parent word held by lane 4*blk + r.  Each result register is again a
// word vector and feeds the next level directly, so everything below the chain runs on the matrix
// cores; the chain (top K letters, per-lane) stays on the vector ALU.
// For D = 16 the levels below the slice use v_mfma_f32_16x16x1_4b_f32 instead (64 parents x 16 letters per
// instruction): register 4*blk + r of lane 16*g + j holds the child with letter j of the parent in lane
// 16*blk + 4*g + r.
// The B-lane-group-pattern modifier (values 4..7: take the B operand of lanes 16c..16c+15 for every group of
// 16 lanes) lets one register carry the increments of four (letter group, scale) combinations, so a segment
// needs one or two LDS reads for all matrix-core operands.

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <int SEL>
__device__ __forceinline__ v4f mfma4_blgp(float a, float b, v4f c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 4 + SEL);
}
// sel becomes a constant once the caller's loops are unrolled
__device__ __forceinline__ v4f mfma4(float a, float b, v4f c, int sel)
{
    switch (sel & 3) {
        case 0: return mfma4_blgp<0>(a, b, c);
        case 1: return mfma4_blgp<1>(a, b, c);
        case 2: return mfma4_blgp<2>(a, b, c);
        default: return mfma4_blgp<3>(a, b, c);
    }
}
template <int SEL>
__device__ __forceinline__ v16f mfma16_blgp(float a, float b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, c, 0, 0, 4 + SEL);
}
__device__ __forceinline__ v16f mfma16(float a, float b, v16f c, int sel)
{
    switch (sel & 3) {
        case 0: return mfma16_blgp<0>(a, b, c);
        case 1: return mfma16_blgp<1>(a, b, c);
        case 2: return mfma16_blgp<2>(a, b, c);
        default: return mfma16_blgp<3>(a, b, c);
    }
}

// number of 4-vectors of state below one parent word vector whose children have length lev (all Q groups)
__host__ __device__ constexpr int casc_size(int D, int N, int lev)
{
    int r = D / 4;
    for (int q = N; q > lev; --q) r = (D / 4) * (1 + 4 * r);
    return r;
}
// D = 16: number of 16-vectors below one parent word vector whose children have length lev
__host__ __device__ constexpr int casc16_size(int N, int lev)
{
    int r = 1;
    for (int q = N; q > lev; --q) r = 1 + 16 * r;
    return r;
}

template <int D, int N, int K, int WQ>
struct MGeo {
    static_assert(D % 4 == 0, "letters are processed in groups of four");
    static_assert(K >= 1 && K < N, "chain length must be in [1, N)");
    static constexpr int Q = D / 4;
    static_assert(Q % WQ == 0, "slice width must divide the number of letter groups");
    static constexpr int NP = ipow(D, K);
    static_assert(NP % kWave == 0, "a wavefront holds 64 prefixes of one path");
    static constexpr int NSL = Q / WQ;
    static constexpr int WAVES = (NP / kWave) * NSL;      // wavefronts per path
    static constexpr bool WIDE = (D == 16);               // 16x16x1 below the slice
    static constexpr int NTS = N - K;                     // scaled copies the slice level needs (t = 0..N-K-1)
    static constexpr int NTU = N - K - 1;                 // ... the levels below it
    static constexpr int BELOW4 = (K + 1 < N && !WIDE) ? casc_size(D, N, K + 2) : 0;    // 4-vectors below one slice vector
    static constexpr int BELOW16 = (K + 1 < N && WIDE) ? casc16_size(N, K + 2) : 0;     // 16-vectors below one slice vector
    static constexpr int NV4 = WQ * (1 + 4 * BELOW4);
    static constexpr int NV16 = WQ * 4 * BELOW16;
    static constexpr int NBS = (NTS * WQ + 3) / 4;        // B registers of the slice level
    static constexpr int NCU = WIDE ? NTU : NTU * Q;      // (scale[, group]) combinations below the slice
    static constexpr int NBU = (NCU + 3) / 4;
};

// 4x4x1 cascade: children of length LEV of one parent word vector.  gpar[t] = A_{LEV-1}[t] of the parent (t >= 1);
// B[(t * NG + g) / 4] with lane-group selector (t * NG + g) % 4 carries dX^{(4 g' + lane%4)}/(t+1) of group g.
template <int D, int N, int LEV, int NG, int NV4, int NB>
__device__ __forceinline__ void casc_fwd(v4f (&S)[NV4], int off, const float* gpar, const float (&Bt)[NB],
                                         const float* Bu_ptr)
{
    constexpr int Q = D / 4;
    constexpr int CSZ = (LEV < N) ? casc_size(D, N, LEV + 1) : 0;
    constexpr int NBU = ((N - LEV - 0) * Q + 3) / 4 > 0 ? ((N - LEV) * Q + 3) / 4 : 1;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int o = off + g * (1 + 4 * CSZ);
        if constexpr (LEV < N) {
            v4f G[N - LEV + 1];
#pragma unroll
            for (int t = N - LEV; t >= 1; --t) G[t] = mfma4(gpar[t + 1], Bt[(t * NG + g) / 4], S[o], (t * NG + g) % 4);
            S[o] = mfma4(gpar[1], Bt[g / 4], S[o], g % 4);
            float Bu[NBU];
#pragma unroll
            for (int q = 0; q < NBU; ++q) Bu[q] = Bu_ptr[q];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float gp[N - LEV + 2];
#pragma unroll
                for (int t = 1; t <= N - LEV; ++t) gp[t] = G[t][r];
                casc_fwd<D, N, LEV + 1, Q, NV4, NBU>(S, o + 1 + r * CSZ, gp, Bu, Bu_ptr);
            }
        } else {
            S[o] = mfma4(gpar[1], Bt[g / 4], S[o], g % 4);
        }
    }
}

// 16x16x1 cascade (D = 16): all 16 children of length LEV of one parent word vector.  B[t / 4] with selector t % 4
// carries dX^{(lane%16)}/(t+1).
template <int N, int LEV, int NV16, int NB>
__device__ __forceinline__ void casc16_fwd(v16f (&S)[NV16], int off, const float* gpar, const float (&B)[NB])
{
    if constexpr (LEV < N) {
        constexpr int CSZ = casc16_size(N, LEV + 1);
        v16f G[N - LEV + 1];
#pragma unroll
        for (int t = N - LEV; t >= 1; --t) G[t] = mfma16(gpar[t + 1], B[t / 4], S[off], t % 4);
        S[off] = mfma16(gpar[1], B[0], S[off], 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float gp[N - LEV + 2];
#pragma unroll
            for (int t = 1; t <= N - LEV; ++t) gp[t] = G[t][r];
            casc16_fwd<N, LEV + 1, NV16, NB>(S, off + 1 + r * CSZ, gp, B);
        }
    } else {
        S[off] = mfma16(gpar[1], B[0], S[off], 0);
    }
}

// Writes the words of a 4x4x1 cascade.  phi_par: per lane, the base-D encoding of the parent vector's word in this
// lane.  g0: first letter group handled (slice offset).
template <int D, int N, int LEV, int NG, int NV4>
__device__ __forceinline__ void casc_store(const v4f (&S)[NV4], int off, int phi_par, int g0, int lane,
                                           float* __restrict__ out)
{
    constexpr int Q = D / 4;
    constexpr int CSZ = (LEV < N) ? casc_size(D, N, LEV + 1) : 0;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int o = off + g * (1 + 4 * CSZ);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // lane 4*blk + j holds the child with letter 4(g0+g) + j of the word in the parent's lane 4*blk + r
            const int phi = __shfl(phi_par, (lane & ~3) + r) * D + 4 * (g0 + g) + (lane & 3);
            out[level_start(D, LEV) + phi] = S[o][r];
            if constexpr (LEV < N) casc_store<D, N, LEV + 1, Q, NV4>(S, o + 1 + r * CSZ, phi, 0, lane, out);
        }
    }
}

template <int N, int LEV, int NV16>
__device__ __forceinline__ void casc16_store(const v16f (&S)[NV16], int off, int phi_par, int lane, float* __restrict__ out)
{
    constexpr int CSZ = (LEV < N) ? casc16_size(N, LEV + 1) : 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        // register 4*blk + rr of lane 16*g + j: child with letter j of the word in the parent's lane 16*blk + 4*g + rr
        const int src = 16 * (r / 4) + 4 * (lane / 16) + (r % 4);
        const int phi = __shfl(phi_par, src) * 16 + (lane & 15);
        out[level_start(16, LEV) + phi] = S[off][r];
        if constexpr (LEV < N) casc16_store<N, LEV + 1, NV16>(S, off + 1 + r * CSZ, phi, lane, out);
    }
}

// Software pipeline of the segment loop (one wavefront per SIMD cannot hide latencies by switching waves):
//   stage 0  LDS reads of the increments, two segments ahead (one ahead for the levels below the slice)
//   stage 1  chain on the vector ALU + first cascade level (slice) on the matrix core, one segment ahead
//   stage 2  remaining cascade levels of the current segment
// so neither the LDS latency nor the matrix-core result latency between the first and second cascade level is
// exposed.  The increments live in a two-tile LDS ring filled one tile ahead from registers that were loaded
// from global memory a further tile ahead.  Segments past the end of the path carry dX = 0 (no-ops).
// A workgroup is four independent wavefronts (one per SIMD of a compute unit: with single-wavefront workgroups
// the dispatcher sometimes puts two on one SIMD, which then takes twice as long).  They share nothing: each has
// its own LDS region, and ordering inside a wavefront only needs a fence, not a barrier.
constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int D, int N, int K, int WQ, int T>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void trunc_mfma_fwd_kernel(const float* __restrict__ path,
                                                                                int64_t B, int64_t P,
                                                                                float* __restrict__ coeffs)
{
    using G = MGeo<D, N, K, WQ>;
    constexpr int Q = G::Q;
    constexpr int NV4 = G::NV4;
    constexpr int NV16 = G::NV16 > 0 ? G::NV16 : 1;
    constexpr int NTS = G::NTS, NTU = G::NTU;
    constexpr int NTU1 = NTU > 0 ? NTU : 1;
    constexpr int NBS = G::NBS;
    constexpr int NBU = G::NBU > 0 ? G::NBU : 1;
    constexpr int NC = (N + 3) / 4 * 4;               // chain table row length
    constexpr int EPL = (T * D + kWave - 1) / kWave;
    static_assert(T % 2 == 0 && T >= 4, "the segment loop is unrolled by two");
    __shared__ float E_all[kWavesPerBlock][2 * T][N][D];   // ring of two tiles; E[row][t][i] = dX^{(i)} / (t+1)
    __shared__ __attribute__((aligned(16))) float Ec_all[kWavesPerBlock][2 * T][D][NC];   // scale index fastest (chain reads)

    const int lane = threadIdx.x % kWave;
    const int wib = threadIdx.x / kWave;
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + wib;
    if (wave >= B * G::WAVES) return;                     // no barriers below: a whole wavefront may leave
    float (*E)[N][D] = E_all[wib];
    float (*Ec)[D][NC] = Ec_all[wib];
    const int64_t b = wave / G::WAVES;
    const int wip = (int)(wave % G::WAVES);               // wavefront inside the path
    const int slice = wip % G::NSL;
    const int p = (wip / G::NSL) * kWave + lane;          // this lane's prefix (base-D number of K letters)
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const int g0 = slice * WQ;
    const float* X = path + b * P * D;
    const int64_t L = P - 1;

    // per-lane offsets (in floats, inside one row of E) of the matrix-core B operands: register r serves the
    // combinations 4r..4r+3, one per group of 16 lanes
    int offS[NBS], offU[NBU];
#pragma unroll
    for (int r = 0; r < NBS; ++r) {
        const int c = 4 * r + lane / 16;
        offS[r] = c < NTS * WQ ? (c / WQ) * D + 4 * (g0 + c % WQ) + (lane & 3) : 0;
    }
#pragma unroll
    for (int r = 0; r < NBU; ++r) {
        const int c = 4 * r + lane / 16;
        if constexpr (G::WIDE) offU[r] = c < G::NCU ? c * D + (lane & 15) : 0;
        else offU[r] = c < G::NCU ? (c / Q) * D + 4 * (c % Q) + (lane & 3) : 0;
    }

    float Sc[K];
#pragma unroll
    for (int k = 0; k < K; ++k) Sc[k] = 0.0f;
    v4f S[NV4];
#pragma unroll
    for (int r = 0; r < NV4; ++r) S[r] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
    v16f S16[NV16];
#pragma unroll
    for (int r = 0; r < NV16; ++r)
#pragma unroll
        for (int q = 0; q < 16; ++q) S16[r][q] = 0.0f;

    float dxn[EPL];
    auto fetch = [&](int64_t j0) {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            // unconditional loads from a clamped address (no divergent branch, so all loads of a tile are
            // in flight together); out-of-range segments are zeroed afterwards
            const int e = (lane + q * kWave) < T * D ? lane + q * kWave : T * D - 1;
            const int64_t jj = j0 + e / D;
            const int64_t jc = jj < L ? jj : L - 1;
            const int i = e % D;
            const float x1 = X[(jc + 1) * D + i], x0 = X[jc * D + i];
            dxn[q] = jj < L ? x1 - x0 : 0.0f;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = lane + q * kWave;
            if (e < T * D) {
#pragma unroll
                for (int t = 0; t < N; ++t) {
                    const float v = dxn[q] * inv1(t);
                    E[buf * T + e / D][t][e % D] = v;
                    Ec[buf * T + e / D][e % D][t] = v;
                }
            }
        }
    };

    struct RS {
        float ec[K][NC];
        float bs[NBS];
    };
    auto load_rs = [&](RS& R, int row) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const float* src = &Ec[row][letter[k]][0];
#pragma unroll
            for (int t = 0; t <= N - (k + 1); ++t) R.ec[k][t] = src[t];
        }
        const float* Et = &E[row][0][0];
#pragma unroll
        for (int r = 0; r < NBS; ++r) R.bs[r] = Et[offS[r]];
    };
    auto load_u = [&](float (&U)[NBU], int row) {
        const float* Et = &E[row][0][0];
#pragma unroll
        for (int r = 0; r < NBU; ++r) U[r] = Et[offU[r]];
    };
    // chain + slice level
    auto stage1 = [&](const RS& R, v4f (&Gout)[WQ][NTU1]) {
        float a[K + 1][N + 2];
#pragma unroll
        for (int t = 0; t < N + 2; ++t) a[0][t] = 1.0f;
#pragma unroll
        for (int k = 1; k <= K; ++k) {
#pragma unroll
            for (int t = 1; t <= N - k; ++t) a[k][t] = fmaf(R.ec[k - 1][t], a[k - 1][t + 1], Sc[k - 1]);
            Sc[k - 1] = fmaf(R.ec[k - 1][0], a[k - 1][1], Sc[k - 1]);
        }
#pragma unroll
        for (int g = 0; g < WQ; ++g) {
            const int o = g * (1 + 4 * G::BELOW4);
#pragma unroll
            for (int t = NTU; t >= 1; --t)
                Gout[g][t - 1] = mfma4(a[K][t + 1], R.bs[(t * WQ + g) / 4], S[o], (t * WQ + g) % 4);
            S[o] = mfma4(a[K][1], R.bs[g / 4], S[o], g % 4);
        }
    };
    // everything below the slice level
    auto stage2 = [&](const v4f (&Gin)[WQ][NTU1], const float (&U)[NBU]) {
        if constexpr (NTU > 0) {
#pragma unroll
            for (int g = 0; g < WQ; ++g)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float gp[NTU + 2];
#pragma unroll
                    for (int t = 1; t <= NTU; ++t) gp[t] = Gin[g][t - 1][r];
                    if constexpr (G::WIDE)
                        casc16_fwd<N, K + 2, NV16, NBU>(S16, (g * 4 + r) * G::BELOW16, gp, U);
                    else
                        casc_fwd<D, N, K + 2, Q, NV4, NBU>(S, g * (1 + 4 * G::BELOW4) + 1 + r * G::BELOW4, gp, U, U);
                }
        }
    };

    const int64_t ntiles = (L + T - 1) / T;
    fetch(0);
    stage(0);
    fetch(T);
    stage(1);
    wave_lds_fence();

    RS RA, RB;
    v4f GA[WQ][NTU1], GB[WQ][NTU1];
    float UA[NBU], UB[NBU];
    // invariant at the top of a half step for segment s (s even): RB = increments of segment s + 1,
    // GA = slice-level accumulators of segment s, UA = increments of segment s for the lower levels
    load_rs(RA, 0);
    load_u(UA, 0);
    stage1(RA, GA);
    load_rs(RB, 1);
    for (int64_t n = 0; n < ntiles; ++n) {
        fetch((n + 2) * T);
        const int base = (int)(n & 1) * T;
#pragma unroll 1
        for (int tt = 0; tt < T; tt += 2) {
            const int r0 = base + tt;                 // ring row of segment s = n T + tt
            load_rs(RA, (r0 + 2) % (2 * T));
            load_u(UB, (r0 + 1) % (2 * T));
            stage1(RB, GB);                           // segment s + 1
            stage2(GA, UA);                           // segment s
            load_rs(RB, (r0 + 3) % (2 * T));
            load_u(UA, (r0 + 2) % (2 * T));
            stage1(RA, GA);                           // segment s + 2
            stage2(GB, UB);                           // segment s + 1
        }
        wave_lds_fence();
        stage((int)(n & 1));                          // tile n + 2 replaces tile n
        wave_lds_fence();
    }

    float* out = coeffs + b * (int64_t)(level_start(D, N) + ipow(D, N));
    {
        int phi = 0;
#pragma unroll
        for (int k = 1; k <= K; ++k) {
            phi = phi * D + letter[k - 1];
            // a chain word is written by the wavefront of slice 0, by the lane whose remaining letters are zero
            if (p % ipow(D, K - k) == 0 && slice == 0) out[level_start(D, k) + phi] = Sc[k - 1];
        }
        if constexpr (G::WIDE && NTU > 0) {
#pragma unroll
            for (int g = 0; g < WQ; ++g)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int ph = __shfl(phi, (lane & ~3) + r) * D + 4 * (g0 + g) + (lane & 3);
                    out[level_start(D, K + 1) + ph] = S[g][r];
                    casc16_store<N, K + 2, NV16>(S16, (g * 4 + r) * G::BELOW16, ph, lane, out);
                }
        } else {
            casc_store<D, N, K + 1, WQ, NV4>(S, 0, phi, g0, lane, out);
        }
    }
}

template <int D, int N, int K, int WQ>
hipError_t launch_trunc_mfma_fwd(const float* path, int64_t B, int64_t P, float* coeffs, hipStream_t stream)
{
    using G = MGeo<D, N, K, WQ>;
    constexpr int T = 16;
    const int64_t waves = B * G::WAVES;
    const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    trunc_mfma_fwd_kernel<D, N, K, WQ, T><<<(unsigned)blocks, kWave * kWavesPerBlock, 0, stream>>>(path, B, P, coeffs);
    return hipGetLastError();
}

}  // namespace

// (D, N) pairs with a register-resident kernel, and the unit shape used for each.
bool trunc_forward_available(int d, int depth)
{
    return (d == 4 && depth == 6) || (d == 8 && depth == 5) || (d == 16 && depth == 4);
}

hipError_t trunc_forward(int d, int depth, const float* path, int64_t B, int64_t P, float* coeffs, hipStream_t stream)
{
    if (B > 65535) return hipErrorInvalidValue;
    if (d == 4 && depth == 6) return launch_trunc_mfma_fwd<4, 6, 4, 1>(path, B, P, coeffs, stream);
    if (d == 8 && depth == 5) return launch_trunc_mfma_fwd<8, 5, 3, 2>(path, B, P, coeffs, stream);
    if (d == 16 && depth == 4) return launch_trunc_mfma_fwd<16, 4, 2, 1>(path, B, P, coeffs, stream);
    return hipErrorInvalidValue;
}

}  // namespace sig
